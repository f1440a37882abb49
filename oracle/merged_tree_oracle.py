"""CPU oracle for draft trees whose nodes are distinct contexts (Sec. 3, Def. 3.1 and its footnote).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT (see mpv_oracle.py): only the tests, the smoke check
and the benchmark's cpu_baseline leg may import it; it shares no code with the HIP library and
never calls it.

Def. 3.1 makes a node of the draft tree a context, so two drafted paths that agree on a prefix
share the nodes of that prefix; the child list of a node keeps one entry per drafted token, in
order, and can therefore name the same child more than once.  Sec. 5, Def. 5.2 says the same of
delayed trees: paths can overlap after the branching node.

Drafting produces one row of logits, one token and one uniform per drafted token ("slot"), laid
out as a tree in which every path owns its slots.  merge_duplicates() turns that layout into the
tree of Def. 3.1 without moving any data:

* the first slot (lowest index) drafted for a context is the node of that context;
* a later slot drafted for the same context ("repeat") stays in the child list of its parent
  context as a further entry for the same token, with its own uniform; in the merged parent
  array it has no children;
* the children of a repeat become children of the node of its context, so the child list of a
  context holds, in slot order, every token drafted after that context.

The result is an ordinary parent array over the same slots plus, per slot, the node of its
context.  Verification of the merged tree is mpv_oracle's verification with that parent array,
where an accepted entry leads to the node of its context.  That last clause only matters to
SpecTr: under the SpecInfer solver and under Traversal Verification an entry is only tested
again after the first entry for its token was rejected, which leaves no residual mass on that
token, so a repeat is tested with probability 0 and only its residual step remains (App. B,
Alg. 4; the Traversal reading of mpv_oracle); NSS and Naive move to the first child in list order
that carries the drawn token (mpv_oracle.token_walk), which is the node of the context.  SpecTr (App. B,
Alg. 3) tests every entry against the same p / (rho* q) with the entry's own uniform, so a repeat
can be the one that is accepted.

Pinned by tests/test_merged_tree_pins.py: against a construction of Def. 3.1 from the contexts
themselves (a dictionary keyed by token sequences), by exact losslessness over all draft trees of
small context-consistent models (where overlaps are frequent), and by the fact that merging can
only lengthen what SpecInfer accepts.
"""

from __future__ import annotations

import numpy as np

from . import mpv_oracle as base


def merge_duplicates(parent, tokens):
    """One tree.  parent: [N] slot layout (parent[0] = -1, parent[n] < n); tokens: [N] (tokens[0]
    ignored).  Returns (merged_parent, context_node), both lists of N ints: merged_parent[n] is the
    node of the context slot n was drafted after; context_node[n] is the node of slot n's own
    context (n itself unless n is a repeat)."""
    parent = [int(x) for x in parent]
    base.children_lists(parent)                      # raises on an invalid layout
    n_slots = len(parent)
    context_node = list(range(n_slots))
    merged_parent = [-1] * n_slots
    for n in range(1, n_slots):
        merged_parent[n] = context_node[parent[n]]
        for m in range(1, n):                        # an earlier slot with the same context?
            if (context_node[m] == m and merged_parent[m] == merged_parent[n]
                    and int(tokens[m]) == int(tokens[n])):
                context_node[n] = m
                break
    return merged_parent, context_node


def merge_batch(parent, tokens):
    """tokens [B,N] -> (merged_parent [B,N], context_node [B,N]) as int32 arrays."""
    tokens = np.asarray(tokens)
    merged = np.zeros(tokens.shape, dtype=np.int32)
    context = np.zeros(tokens.shape, dtype=np.int32)
    for b in range(tokens.shape[0]):
        merged[b], context[b] = merge_duplicates(parent, tokens[b])
    return merged, context


def verify_tree_merged(method, parent, tokens, target_logits, draft_logits, T, u, u_draw=None):
    """mpv_oracle.verify_tree on the tree of Def. 3.1 built from the slot layout `parent`.
    Returns verify_tree's dictionary; path_nodes name nodes of contexts."""
    merged_parent, context_node = merge_duplicates(parent, tokens)
    return base.verify_tree(method, merged_parent, tokens, target_logits, draft_logits, T, u, u_draw,
                            node_of=context_node)


def enumerate_outcomes_merged(method, parent, tokens, p_of, q_of):
    """mpv_oracle.enumerate_outcomes on the merged tree.  p_of / q_of are asked for slots; a
    context-consistent model answers alike for every slot of one context."""
    merged_parent, context_node = merge_duplicates(parent, tokens)
    return base.enumerate_outcomes(method, merged_parent, tokens, p_of, q_of, node_of=context_node)
