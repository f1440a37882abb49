"""fp64 CPU oracle for the expected block efficiency of a draft tree.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT (see mpv_oracle.py): only the tests,
the smoke check and the benchmark's cpu_baseline leg may import it; it shares no
code with the HIP library and never calls it.

What it computes (citations are to the paper):

* branching probabilities (Sec. 5, Def. 5.3): B(f, x, t) = P(solver f, given the
  draft tokens x_1..x_k of a node, outputs token t), for the OTLP solvers of
  App. B, by the listings of App. D:
    NSS        B(t) = p(t)
    Naive      a = min(1, p(x_1)/q(x_1));  B(t) = (1-a) p_res(t) + a 1{t = x_1},
               p_res = norm (p-q)_+
    SpecTr     rho*, beta, p_acc, gamma as in the solver;  a_i = min(1, p(x_i)/(rho* q(x_i)));
               B(t) = sum_j a_j 1{x_j = t} prod_{l<j} (1-a_l) + p_res(t) prod_l (1-a_l),
               p_res = norm (p - gamma min(p/rho*, q))_+
    SpecInfer  two versions: the listing of App. D (the solver picks the next draft
               token uniformly at random: a recursion over multisets), and the same
               solver with the draft tokens taken in list order, which is what the
               verification oracle and the library do (see the readings list).
* expected block efficiency of one tree (Sec. 5, Eq. 1-3, inner sum):
    E[tau + 1 | tree] = sum over nodes of P(the rule's accepted path contains the node)
  For the top-down rules that probability is the product of the branching
  probabilities along the path from the root (Eq. 3).  In a tree whose equal-token
  siblings are separate nodes, a child the solver accepts is moved to itself, and
  a token the solver draws leads to the first sibling that carries it.
* Traversal Verification is not a top-down solver; its nodes are tested in
  depth-first post-order, each after exactly one history (everything before it
  rejected), so with a_r the probability the r-th node in that order is tested
  with, P(it is the accepted one) = a_r prod_{r'<r} (1 - a_r'), and a node lies on
  the accepted path iff the accepted node is in its subtree.

Every function takes explicit float64 distributions or the stored logits; nothing
is sampled.
"""

from __future__ import annotations

import numpy as np

from . import mpv_oracle as base

SPECINFER = base.SPECINFER
TRAVERSAL = base.TRAVERSAL
NSS = base.NSS
NAIVE = base.NAIVE
SPECTR = base.SPECTR


def _normalised(r, fallback):
    s = float(np.sum(r))
    return r / s if s > 0.0 else np.array(fallback, dtype=np.float64)


class Branching:
    """Output law of a solver restricted to the draft tokens of one node, in two parts:
    accept_at[j]: the solver accepts the draft token at list position j;
    drawn[t]:     it rejects everything it tests and then draws token t (t among the draft tokens).
    by_token[t] = sum of accept_at over the positions that carry t, plus drawn[t], is the
    branching probability B(f, x, t) of Def. 5.3."""

    def __init__(self, xs, accept_at, drawn):
        self.xs = [int(x) for x in xs]
        self.accept_at = [float(a) for a in accept_at]
        self.drawn = {int(t): float(v) for t, v in drawn.items()}
        self.by_token = dict(self.drawn)
        for x, a in zip(self.xs, self.accept_at):
            self.by_token[x] += a


def nss_branching(P, Q, xs):
    """App. D, NSS Branching: {x_i -> p(x_i)} (nothing is tested)."""
    P = np.asarray(P, dtype=np.float64)
    return Branching(xs, [0.0] * len(xs), {int(x): P[x] for x in xs})


def naive_branching(P, Q, xs):
    """App. D, Naive Branching: a = min(1, p(x_1)/q(x_1)), p_res = norm (p-q)_+,
    {x_i -> (1-a) p_res(x_i) + a 1{x_i = x_1}}."""
    P = np.asarray(P, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    a = base._ratio(P[xs[0]], Q[xs[0]])
    p_res = _normalised(np.maximum(P - Q, 0.0), P)
    return Branching(xs, [a] + [0.0] * (len(xs) - 1), {int(x): (1.0 - a) * p_res[x] for x in xs})


def spectr_branching(P, Q, xs):
    """App. D, SpecTr Branching: a_i = min(1, p(x_i)/(rho* q(x_i))),
    {x_i -> sum_j a_j 1{x_j = x_i} prod_{l<j}(1-a_l) + p_res(x_i) prod_l (1-a_l)},
    p_res = norm (p - gamma min(p/rho*, q))_+ ."""
    P = np.asarray(P, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    k = len(xs)
    rho = base.spectr_division_factor(P, Q, k)
    beta = base.spectr_beta(P, Q, rho)
    p_acc = 1.0 - (1.0 - beta) ** k
    gamma = p_acc / beta if beta > 0.0 else 0.0
    p_res = _normalised(np.maximum(P - np.minimum(P / rho, Q) * gamma, 0.0), P)
    accept_at, none_before = [], 1.0
    for x in xs:
        a = base._ratio(P[x], rho * Q[x])
        accept_at.append(a * none_before)
        none_before *= 1.0 - a
    return Branching(xs, accept_at, {int(x): p_res[x] * none_before for x in xs})


def specinfer_branching_in_order(P, Q, xs):
    """SpecInfer (App. B, Alg. 4) with the draft tokens tried in list order:
    a_j = min(1, p_{j-1}(x_j)/q(x_j)), p_j = norm (p_{j-1} - q)_+ ;
    P(output = t) = sum_j a_j 1{x_j = t} prod_{l<j}(1-a_l) + p_k(t) prod_l (1-a_l)."""
    P = np.array(P, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    accept_at, none_before = [], 1.0
    for x in xs:
        a = base._ratio(P[x], Q[x])
        accept_at.append(a * none_before)
        none_before *= 1.0 - a
        P = _normalised(np.maximum(P - Q, 0.0), P)
    return Branching(xs, accept_at, {int(x): P[x] * none_before for x in xs})


def specinfer_branching_random_order(P, Q, xs):
    """App. D, SpecInfer Branching: the solver picks the next draft token uniformly at
    random among those left.  Level i works with the i-times-updated residual p_i and
    its acceptance vector min(1, p_i/q); B_i(S; x) averages over the token t of S tried
    next: accepted (and equal to x), or rejected and on to level i+1 without t."""
    P = np.asarray(P, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    k = len(xs)
    levels = [P.copy()]
    for _ in range(k):
        levels.append(_normalised(np.maximum(levels[-1] - Q, 0.0), levels[-1]))
    accept = [np.array([base._ratio(pi[t], Q[t]) for t in range(len(Q))]) for pi in levels]

    def B(i, S, x):
        if i == k:
            return float(levels[k][x])
        total = 0.0
        for j, t in enumerate(S):
            rest = S[:j] + S[j + 1:]
            total += accept[i][t] * (1.0 if t == x else 0.0) + (1.0 - accept[i][t]) * B(i + 1, rest, x)
        return total / len(S)

    toks = tuple(int(x) for x in xs)
    return {x: B(0, toks, x) for x in set(toks)}


_BRANCHING = {SPECINFER: specinfer_branching_in_order, NSS: nss_branching, NAIVE: naive_branching,
              SPECTR: spectr_branching}


def reach_probabilities(method, parent, tokens, p_of, q_of, node_of=None):
    """P(node lies on the accepted path), for every node of one tree (root: 1).

    p_of(n), q_of(n): node n's target / draft distribution (float64 vectors).
    node_of (top-down rules; Def. 3.1, see mpv_oracle.token_walk): the node an accepted child
    entry stands for; None: itself."""
    children = base.children_lists(parent)
    n_nodes = len(parent)
    reach = np.zeros(n_nodes)
    reach[0] = 1.0
    if method == TRAVERSAL:
        # test probabilities in post-order (reject everything: every node gets tested once)
        order, prob = [], {}

        def observe(n, a, P):
            order.append(n)
            prob[n] = 1.0 if n == 0 else a

        base.traversal_rule(children, tokens, p_of, q_of, lambda c, a: False, observe)
        accepted = np.zeros(n_nodes)
        none_before = 1.0
        for n in order:
            accepted[n] = prob[n] * none_before
            none_before *= 1.0 - prob[n]
        for n in range(1, n_nodes):              # a node is on the path iff the accepted node is it or below it
            m = n
            while m > 0:
                reach[m] += accepted[n]
                m = int(parent[m])
        return reach
    for n in range(n_nodes):                     # parents come before their children
        ch = children[n]
        if not ch:
            continue
        xs = [int(tokens[c]) for c in ch]
        br = _BRANCHING[method](p_of(n), q_of(n), xs)
        seen = set()
        for j, (c, x) in enumerate(zip(ch, xs)):
            b = br.accept_at[j]                  # an accepted child is moved to itself
            if method != SPECINFER and x not in seen:
                # a drawn token leads to the first sibling carrying it (SpecInfer's walk ends with
                # the draw; its residual has no mass on the rejected draft tokens anyway)
                b += br.drawn[x]
                seen.add(x)
            if node_of is None:
                reach[c] = reach[n] * b
            else:
                # an accepted entry is credited to the node it stands for; a drawn token already
                # leads to the first sibling carrying it, which stands for itself
                accepted = br.accept_at[j]
                reach[int(node_of[c])] += reach[n] * accepted
                reach[c] += reach[n] * (b - accepted)
    return reach


def expected_block_efficiency(method, parent, tokens, target_logits, draft_logits, T, node_of=None):
    """E[tau + 1 | tree] (Sec. 5, Eq. 1-3) and the reach probabilities, for one tree given
    its stored logits [N, V].  Returns (expected, reach[N])."""
    p_of = base._RowCache(target_logits, T)
    q_of = base._RowCache(draft_logits, T)
    reach = reach_probabilities(method, parent, tokens, p_of, q_of, node_of)
    return float(np.sum(reach)), reach


def expected_block_efficiency_batch(method, parent, tokens, target_logits, draft_logits, T):
    """The same for a batch: tokens [B,N], logits [B,N,V].  Returns (expected[B], reach[B,N]).
    The estimate of Sec. 5 averages `expected` over the s sampled trees of one context."""
    out = [expected_block_efficiency(method, parent, tokens[b], target_logits[b], draft_logits[b], T)
           for b in range(len(tokens))]
    return np.array([e for e, _ in out]), np.stack([r for _, r in out])
