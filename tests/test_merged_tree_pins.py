"""Pins for the merged-tree oracle (Sec. 3, Def. 3.1 with its footnote; Sec. 5, Def. 5.2): draft
trees whose nodes are distinct contexts and whose child lists keep one entry per drafted token.

None of these call the HIP library.
"""

import itertools

import numpy as np
import pytest

from oracle import merged_tree_oracle as merged
from oracle import mpv_oracle as orc
from tests.test_oracle_pins import (ContextModel, METHODS, TOKEN_WALK_METHODS, delayed_parent,
                                    losslessness_error, node_contexts)


# --------------------------------------------------------------------------
# the construction itself, against Def. 3.1 written out with contexts as dictionary keys
# --------------------------------------------------------------------------

def tree_of_contexts(parent, tokens):
    """Def. 3.1 from the contexts themselves: returns (node_of_context, child_entries) where
    node_of_context maps a token sequence to the first slot drafted for it and child_entries maps
    it to the list, in slot order, of the slots drafted right after it."""
    ctx = node_contexts(parent, tokens)
    node_of_context = {}
    child_entries = {}
    for n, c in enumerate(ctx):
        node_of_context.setdefault(c, n)
        child_entries.setdefault(c, [])
        if n > 0:
            child_entries[ctx[parent[n]]].append(n)
    return ctx, node_of_context, child_entries


def random_layout(rng, n_slots):
    return [-1] + [int(rng.integers(0, n)) for n in range(1, n_slots)]


@pytest.mark.parametrize("seed", range(40))
def test_merge_is_definition_3_1(seed):
    rng = np.random.default_rng(seed)
    n_slots = int(rng.integers(2, 14))
    parent = random_layout(rng, n_slots) if seed % 2 else delayed_parent(int(rng.integers(1, 5)), int(rng.integers(0, 3)), int(rng.integers(1, 4)))
    V = int(rng.integers(1, 4))
    tokens = [0] + [int(t) for t in rng.integers(0, V, size=len(parent) - 1)]
    mp, cn = merged.merge_duplicates(parent, tokens)
    ctx, node_of_context, child_entries = tree_of_contexts(parent, tokens)
    for n in range(len(parent)):
        assert cn[n] == node_of_context[ctx[n]]
        if n > 0:
            assert mp[n] == node_of_context[ctx[parent[n]]] and mp[n] < n
    # the merged array is a tree over the same slots; contexts are unchanged by re-parenting
    assert mp[0] == -1 and node_contexts(mp, tokens) == ctx
    children = orc.children_lists(mp)
    for c, node in node_of_context.items():
        assert children[node] == child_entries[c]                  # every drafted token, in slot order
    for n in range(len(parent)):
        if cn[n] != n:                                             # a repeat
            assert children[n] == [] and cn[cn[n]] == cn[n] and cn[n] < n
            assert mp[n] == mp[cn[n]] and tokens[n] == tokens[cn[n]]
    firsts = [n for n in range(len(parent)) if cn[n] == n]
    assert len({ctx[n] for n in firsts}) == len(firsts) == len(node_of_context)


def test_worked_examples():
    two_paths = [-1, 0, 1, 0, 3]                                   # K = 2 paths of length 2, path by path
    assert merged.merge_duplicates(two_paths, [0, 5, 7, 6, 7]) == ([-1, 0, 1, 0, 3], [0, 1, 2, 3, 4])
    assert merged.merge_duplicates(two_paths, [0, 5, 7, 5, 9]) == ([-1, 0, 1, 0, 1], [0, 1, 2, 1, 4])
    assert merged.merge_duplicates(two_paths, [0, 5, 7, 5, 7]) == ([-1, 0, 1, 0, 1], [0, 1, 2, 1, 2])
    three = delayed_parent(3, 1, 2)                                # trunk 1, then 3 paths of length 2
    assert three == [-1, 0, 1, 2, 1, 4, 1, 6]
    # paths (3,8), (4,8), (3,9): the third shares its first token with the first
    assert merged.merge_duplicates(three, [0, 2, 3, 8, 4, 8, 3, 9]) == ([-1, 0, 1, 2, 1, 4, 1, 2], [0, 1, 2, 3, 4, 5, 2, 7])


def test_distinct_tokens_leave_the_layout_alone():
    parent = delayed_parent(4, 2, 3)
    tokens = list(range(len(parent)))
    assert merged.merge_duplicates(parent, tokens) == (parent, list(range(len(parent))))
    mp, cn = merged.merge_batch(parent, np.array([tokens, tokens]))
    assert mp.dtype == np.int32 and mp.tolist() == [parent, parent] and cn.tolist() == [tokens, tokens]


def test_invalid_layout_is_refused():
    with pytest.raises(ValueError):
        merged.merge_duplicates([-1, 1, 0], [0, 1, 1])


# --------------------------------------------------------------------------
# losslessness of verification on merged trees (Sec. 3.2, Def. 3.2), by enumeration of every
# draft tree of a small context-consistent model
# --------------------------------------------------------------------------

def output_distribution_merged(method, parent, model):
    """As tests.test_oracle_pins.output_distribution, every drafted tree merged first.  Also
    returns the number of draft trees that merging changed and the expected number of accepted
    tokens."""
    N = len(parent)
    V = model.V
    out = {}
    changed = 0
    accepted = 0.0
    for toks in itertools.product(range(V), repeat=N - 1):
        tokens = (0,) + toks
        ctx = node_contexts(parent, tokens)
        tree_prob = 1.0
        for n in range(1, N):
            tree_prob *= model.q[ctx[parent[n]]][tokens[n]]
        if tree_prob == 0.0:
            continue
        mp, cn = merged.merge_duplicates(parent, tokens)
        changed += mp != list(parent)
        outcomes = merged.enumerate_outcomes_merged(
            method, parent, tokens, lambda n: model.p[ctx[n]], lambda n: model.q[ctx[n]])
        assert abs(sum(pr for pr, _, _ in outcomes) - 1.0) < 1e-12
        for pr, stop, P in outcomes:
            accepted += tree_prob * pr * len(ctx[stop])
            if method != orc.SPECTR:
                assert cn[stop] == stop, "a repeat was accepted"
            if method in TOKEN_WALK_METHODS:
                seq = ctx[stop] + (int(P),)
                out[seq] = out.get(seq, 0.0) + tree_prob * pr
                continue
            for y in range(V):
                if P[y] > 0:
                    seq = ctx[stop] + (y,)
                    out[seq] = out.get(seq, 0.0) + tree_prob * pr * P[y]
    return out, changed, accepted


MERGED_SHAPES = [(3, 2, 0, 2), (3, 3, 0, 2), (2, 3, 0, 2), (3, 2, 1, 2), (2, 2, 0, 3), (4, 2, 0, 2)]


@pytest.mark.parametrize("method", METHODS + TOKEN_WALK_METHODS)
@pytest.mark.parametrize("V,K,L1,L2", MERGED_SHAPES)
def test_merged_trees_keep_the_target_distribution(method, V, K, L1, L2):
    rng = np.random.default_rng(7000 + 1000 * V + 100 * K + 10 * L1 + L2)
    depth = L1 + L2
    model = ContextModel(rng, V, depth, zero_frac=0.25)
    out, changed, _ = output_distribution_merged(method, delayed_parent(K, L1, L2), model)
    assert changed > 0
    assert abs(sum(out.values()) - 1.0) < 1e-12
    assert losslessness_error(out, model, depth + 1) < 1e-13


def test_merged_irregular_layout_keeps_the_target_distribution():
    parent = [-1, 0, 0, 1, 2, 2]
    model = ContextModel(np.random.default_rng(5), 3, 2, zero_frac=0.2)
    for method in METHODS + TOKEN_WALK_METHODS:
        out, changed, _ = output_distribution_merged(method, parent, model)
        assert changed > 0 and losslessness_error(out, model, 3) < 1e-13


# --------------------------------------------------------------------------
# what merging changes
# --------------------------------------------------------------------------

def expected_accept_len(outcomes, parent):
    depth = orc.node_depths(parent)
    return sum(pr * depth[stop] for pr, stop, _ in outcomes)


@pytest.mark.parametrize("seed", range(6))
def test_specinfer_never_accepts_less_on_the_merged_tree(seed):
    """The child list of a context is the unmerged one followed by further entries, and SpecInfer
    (App. B, Alg. 4) tests the entries in order: what it did without them it still does, and the
    further entries only add chances.  Tree by tree, not only on average."""
    rng = np.random.default_rng(900 + seed)
    V, K, L = 3, 3, 2
    model = ContextModel(rng, V, L)
    parent = delayed_parent(K, 0, L)
    gained = 0
    for toks in itertools.product(range(V), repeat=len(parent) - 1):
        tokens = (0,) + toks
        ctx = node_contexts(parent, tokens)
        p_of, q_of = (lambda n: model.p[ctx[n]]), (lambda n: model.q[ctx[n]])
        mp, _ = merged.merge_duplicates(parent, tokens)
        plain = expected_accept_len(orc.enumerate_outcomes(orc.SPECINFER, parent, tokens, p_of, q_of), parent)
        both = expected_accept_len(merged.enumerate_outcomes_merged(orc.SPECINFER, parent, tokens, p_of, q_of), mp)
        assert both >= plain - 1e-14
        gained += both > plain + 1e-9
    assert gained > 0


def test_spectr_goes_on_below_an_accepted_repeat():
    """App. B, Alg. 3 tests every entry with a uniform of its own, so the second entry for a token
    can be the accepted one; the walk then continues at the node of that context (Def. 3.1) and
    not at the repeat, which has nothing below it."""
    parent = delayed_parent(2, 0, 2)                      # [-1, 0, 1, 0, 3]
    tokens = [0, 1, 2, 1, 0]
    V = 3
    # at the root p = q: rho* = 1 and every entry is accepted with probability 1 if tested
    z = np.zeros((5, V))
    zt = z.copy()
    zt[1] = zt[3] = [0.0, 5.0, 9.0]                       # below (root,1): the target wants token 2
    u = np.array([0.5, 0.999999, 0.5, 0.1, 0.9])
    res = merged.verify_tree_merged(orc.SPECTR, parent, tokens, zt, z, 1.0, u, u_draw=np.full(5, 0.5))
    # p = q at the root makes the test probability exactly 1: the first entry is accepted whatever u is
    assert res["path_nodes"][0] == 1
    # make the first entry fail: the target gives token 1 a third of what the draft gives it
    zt[0] = [np.log(4.0), 0.0, np.log(4.0)]
    res = merged.verify_tree_merged(orc.SPECTR, parent, tokens, zt, z, 1.0, u, u_draw=np.full(5, 0.5))
    first = [d for d in res["decisions"] if d[0] == 1][0]
    second = [d for d in res["decisions"] if d[0] == 3][0]
    assert first[1] == second[1] and 0.0 < first[1] < 1.0         # same probability, own uniforms
    assert not first[3] and second[3]
    assert res["path_nodes"][0] == 1                               # the node of the context, not slot 3
    assert res["accept_len"] >= 1 and set(res["path_nodes"]) <= {1, 2, 4}


@pytest.mark.parametrize("method", METHODS + TOKEN_WALK_METHODS)
def test_block_efficiency_of_a_merged_tree_is_its_expected_accepted_length(method):
    """The block-efficiency oracle on the merged array (with the entries' nodes for the top-down rules)
    against the verification oracle's own outcomes on the same tree: sum of reach probabilities =
    E[accepted length] + 1, and node by node the probability of lying on the accepted path."""
    from oracle import block_efficiency_oracle as beo
    rng = np.random.default_rng(4242)
    V, K, L = 3, 3, 2
    model = ContextModel(rng, V, L, zero_frac=0.2)
    parent = delayed_parent(K, 0, L)
    checked = 0
    for toks in itertools.product(range(V), repeat=len(parent) - 1):
        tokens = (0,) + toks
        mp, cn = merged.merge_duplicates(parent, tokens)
        if mp == list(parent) and checked % 7:
            continue
        ctx = node_contexts(parent, tokens)
        p_of, q_of = (lambda n: model.p[ctx[n]]), (lambda n: model.q[ctx[n]])
        node_of = cn if method in TOKEN_WALK_METHODS + [orc.SPECINFER] else None
        reach = beo.reach_probabilities(method, mp, tokens, p_of, q_of, node_of if method != orc.TRAVERSAL else None)
        on_path = np.zeros(len(parent))
        for pr, stop, _ in merged.enumerate_outcomes_merged(method, parent, tokens, p_of, q_of):
            n = stop
            while n >= 0:
                on_path[n] += pr
                n = mp[n]
        assert np.allclose(reach, on_path, atol=1e-12), (method, tokens)
        checked += 1
    assert checked > 100
