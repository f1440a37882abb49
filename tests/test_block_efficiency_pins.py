"""Pins for the block-efficiency oracle (Sec. 5, Def. 5.3, Eq. 1-3; App. D).

None of these call the HIP library.  The branching formulas of App. D are checked
against things that do not use them: the exact enumeration of the verification
oracle's own walk, the acceptance rates of App. C, and sample means.
"""

import itertools

import numpy as np
import pytest

from oracle import block_efficiency_oracle as beo
from oracle import mpv_oracle as orc

ALL_METHODS = [orc.SPECINFER, orc.TRAVERSAL, orc.NSS, orc.NAIVE, orc.SPECTR]


def delayed_parent(K, L1, L2):
    parent = [-1]
    last = 0
    for _ in range(L1):
        parent.append(last)
        last = len(parent) - 1
    for _ in range(K):
        prev = last
        for _ in range(L2):
            parent.append(prev)
            prev = len(parent) - 1
    return parent


def random_dist(rng, V, sparsity=0.0):
    x = rng.gamma(0.7, size=V) + 1e-3
    if sparsity > 0:
        mask = rng.random(V) < sparsity
        if mask.all():
            mask[rng.integers(V)] = False
        x = np.where(mask, 0.0, x)
    return x / x.sum()


def random_tree_case(rng, parent, V, sparsity=0.2):
    N = len(parent)
    p_rows = [random_dist(rng, V, sparsity) for _ in range(N)]
    q_rows = [random_dist(rng, V) for _ in range(N)]
    tokens = [0] + [int(rng.integers(V)) for _ in range(N - 1)]      # small V: equal-token siblings are frequent
    return tokens, p_rows, q_rows


def reach_by_enumeration(method, parent, tokens, p_rows, q_rows):
    """P(node on the accepted path) from the exact outcome distribution of the
    verification oracle's own walk (every test branched with its probability)."""
    outs = orc.enumerate_outcomes(method, parent, tokens, lambda n: p_rows[n], lambda n: q_rows[n])
    reach = np.zeros(len(parent))
    for pr, stop, _ in outs:
        reach[0] += pr
        for n in orc.path_to(parent, stop):
            reach[n] += pr
    return reach


SHAPES = [(2, 0, 2), (3, 0, 1), (2, 1, 2), (3, 1, 1), (1, 0, 3), (4, 0, 1), (2, 2, 1)]


@pytest.mark.parametrize("method", ALL_METHODS)
@pytest.mark.parametrize("K,L1,L2", SHAPES)
def test_reach_probabilities_equal_exact_enumeration(method, K, L1, L2):
    # Sec. 5 Eq. (2): E[tau+1 | T] = sum over nodes of P(the solver reaches the node | T);
    # Eq. (3): for a top-down solver that probability is the product of branching probabilities.
    parent = delayed_parent(K, L1, L2)
    for seed in range(6):
        rng = np.random.default_rng(1000 * K + 100 * L1 + 10 * L2 + seed)
        V = 3 + seed % 3
        tokens, p_rows, q_rows = random_tree_case(rng, parent, V)
        want = reach_by_enumeration(method, parent, tokens, p_rows, q_rows)
        got = beo.reach_probabilities(method, parent, tokens, lambda n: p_rows[n], lambda n: q_rows[n])
        np.testing.assert_allclose(got, want, atol=1e-12, rtol=0)
        assert got[0] == 1.0
        # a node is reached only through its parent
        for n in range(1, len(parent)):
            assert got[n] <= got[parent[n]] + 1e-12


def test_irregular_tree_with_equal_token_siblings():
    parent = [-1, 0, 0, 0, 1, 1, 2, 4, 4]
    tokens = [0, 2, 2, 1, 3, 3, 0, 1, 2]          # children of the root: 2, 2, 1; of node 1: 3, 3
    rng = np.random.default_rng(77)
    p_rows = [random_dist(rng, 4, 0.2) for _ in parent]
    q_rows = [random_dist(rng, 4) for _ in parent]
    for method in ALL_METHODS:
        want = reach_by_enumeration(method, parent, tokens, p_rows, q_rows)
        got = beo.reach_probabilities(method, parent, tokens, lambda n: p_rows[n], lambda n: q_rows[n])
        np.testing.assert_allclose(got, want, atol=1e-12, rtol=0)
    # a drawn token never leads to the second of two equal-token siblings: NSS (nothing is tested) and
    # Naive (only the first child is tested) never get there, nor below it
    for method in (orc.NSS, orc.NAIVE):
        got = beo.reach_probabilities(method, parent, tokens, lambda n: p_rows[n], lambda n: q_rows[n])
        assert got[2] == 0.0 and got[6] == 0.0
    assert beo.reach_probabilities(orc.NSS, parent, tokens, lambda n: p_rows[n], lambda n: q_rows[n])[5] == 0.0


def expected_hits(branching, p, q, k):
    """E over x_1..x_k ~ q i.i.d. of P(the solver's output is one of the draft tokens)."""
    V = len(p)
    total = 0.0
    for xs in itertools.product(range(V), repeat=k):
        w = float(np.prod([q[x] for x in xs]))
        if w == 0.0:
            continue
        B = branching(p, q, list(xs)).by_token
        total += w * sum(B[x] for x in set(xs))
    return total


@pytest.mark.parametrize("V,k", [(4, 1), (4, 2), (5, 3), (3, 4)])
def test_branching_probabilities_average_to_appendix_C_acceptance_rates(V, k):
    # App. C: acceptance rate = P(output token among the draft tokens), over the draft tokens too.
    rng = np.random.default_rng(7 * V + k)
    p, q = random_dist(rng, V, 0.2), random_dist(rng, V)
    # NSS Acceptance
    assert expected_hits(beo.nss_branching, p, q, k) == pytest.approx(
        float(np.sum(p * (1.0 - (1.0 - q) ** k))), abs=1e-13)
    # Naive Acceptance
    want = float(np.sum(np.minimum(p, q)) + np.sum(np.maximum(p - q, 0.0) * (1.0 - (1.0 - q) ** (k - 1))))
    assert expected_hits(beo.naive_branching, p, q, k) == pytest.approx(want, abs=1e-13)
    # SpecTr Acceptance
    rho = orc.spectr_division_factor(p, q, k)
    beta = orc.spectr_beta(p, q, rho)
    p_acc = 1.0 - (1.0 - beta) ** k
    res = np.maximum(p - np.minimum(p / rho, q) * (p_acc / beta), 0.0)
    res = res / res.sum() if res.sum() > 0 else res
    r = np.maximum(q - p / rho, 0.0) / (1.0 - beta)
    want = p_acc + (1.0 - p_acc) * float(np.sum(res * (1.0 - (1.0 - r) ** k)))
    assert expected_hits(beo.spectr_branching, p, q, k) == pytest.approx(want, abs=1e-12)
    # SpecInfer Acceptance (App. C): the same for both orders of trying the tokens
    p_rej, m, pi = 1.0, np.ones(V), p.copy()
    for _ in range(k):
        rr = float(np.sum(np.minimum(pi, q)))
        p_rej *= 1.0 - rr
        m = m * (1.0 - np.maximum(q - pi, 0.0) / (1.0 - rr))
        nxt = np.maximum(pi - q, 0.0)
        pi = nxt / nxt.sum()
    want = (1.0 - p_rej) + p_rej * float(np.sum(pi * (1.0 - m)))
    assert expected_hits(beo.specinfer_branching_in_order, p, q, k) == pytest.approx(want, abs=1e-12)
    random_order = lambda p_, q_, xs: beo.Branching(xs, [0.0] * len(xs), beo.specinfer_branching_random_order(p_, q_, xs))
    assert expected_hits(random_order, p, q, k) == pytest.approx(want, abs=1e-12)


@pytest.mark.parametrize("xs", [(0,), (0, 1), (2, 2), (0, 1, 2), (1, 3, 1), (0, 1, 2, 3)])
def test_specinfer_random_order_is_the_average_of_all_orders(xs):
    # App. D "SpecInfer Branching" (uniformly random next token) against the in-order solver
    rng = np.random.default_rng(50 + len(xs))
    p, q = random_dist(rng, 5), random_dist(rng, 5)
    want = beo.specinfer_branching_random_order(p, q, xs)
    perms = list(itertools.permutations(xs))
    for x, b in want.items():
        avg = sum(beo.specinfer_branching_in_order(p, q, list(perm)).by_token[x] for perm in perms) / len(perms)
        assert avg == pytest.approx(b, abs=1e-13)


@pytest.mark.parametrize("method", [orc.NSS, orc.NAIVE, orc.SPECTR])
def test_branching_probabilities_are_the_solver_output_law(method):
    # Def. 5.3: B(f, x, t) = P(f(x) = t), here against the solver itself, enumerated on a depth-1 tree
    rng = np.random.default_rng(5 + method)
    V, k = 5, 3
    p, q = random_dist(rng, V, 0.2), random_dist(rng, V)
    branching = {orc.NSS: beo.nss_branching, orc.NAIVE: beo.naive_branching, orc.SPECTR: beo.spectr_branching}[method]
    for xs in [(0, 1, 2), (3, 3, 1), (4, 0, 4), (2, 2, 2)]:
        parent = [-1] + [0] * k
        outs = orc.enumerate_outcomes(method, parent, (0,) + xs, lambda n: p, lambda n: q)
        law = np.zeros(V)
        for pr, stop, y in outs:
            law[xs[stop - 1] if stop != 0 else y] += pr      # a walk that moved to a child output that child's token
        B = branching(p, q, list(xs)).by_token
        for x in set(xs):
            assert B[x] == pytest.approx(law[x], abs=1e-13)


def test_identical_models():
    # p = q: SpecInfer, Traversal, Naive and SpecTr accept the first path whole; NSS follows p
    parent = delayed_parent(3, 1, 2)
    rng = np.random.default_rng(3)
    V = 6
    rows = [random_dist(rng, V) for _ in parent]
    tokens = [0, 1, 2, 3, 4, 5, 0, 1]
    first_path_len = 1 + 2
    for method in (orc.SPECINFER, orc.TRAVERSAL, orc.NAIVE, orc.SPECTR):
        got = beo.reach_probabilities(method, parent, tokens, lambda n: rows[n], lambda n: rows[n])
        assert float(got.sum()) == pytest.approx(1.0 + first_path_len, abs=1e-9)
    got = beo.reach_probabilities(orc.NSS, parent, tokens, lambda n: rows[n], lambda n: rows[n])
    assert got[1] == pytest.approx(rows[0][tokens[1]])


@pytest.mark.parametrize("method", ALL_METHODS)
def test_expected_block_efficiency_matches_sample_mean(method):
    # Eq. (1): the quantity is the mean of tau + 1 over the verification's randomness
    parent = delayed_parent(3, 1, 2)
    N, V, T = len(parent), 12, 0.9
    rng = np.random.default_rng(40 + method)
    zd = rng.normal(0, 1.5, size=(N, V)).astype(np.float32)
    zt = (zd + rng.normal(0, 0.7, size=(N, V))).astype(np.float32)
    tokens = np.zeros(N, dtype=np.int64)
    for n in range(1, N):
        q = orc.softmax_T(zd[parent[n]], T)
        tokens[n] = rng.choice(V, p=q)
    want, reach = beo.expected_block_efficiency(method, parent, tokens, zt, zd, T)
    assert reach.shape == (N,) and want == pytest.approx(float(reach.sum()))
    runs = 4000
    lens = np.empty(runs)
    for i in range(runs):
        u = rng.random(N).astype(np.float32)
        ud = rng.random(N).astype(np.float32)
        lens[i] = orc.verify_tree(method, parent, tokens, zt, zd, T, u, ud)["accept_len"] + 1
    assert abs(lens.mean() - want) < 5.0 * lens.std() / np.sqrt(runs) + 1e-9


def test_batch_driver_shapes():
    parent = delayed_parent(2, 0, 2)
    rng = np.random.default_rng(0)
    B, N, V = 3, len(parent), 9
    zd = rng.normal(size=(B, N, V)).astype(np.float32)
    zt = rng.normal(size=(B, N, V)).astype(np.float32)
    tokens = rng.integers(V, size=(B, N))
    e, reach = beo.expected_block_efficiency_batch(orc.SPECTR, parent, tokens, zt, zd, 1.0)
    assert e.shape == (B,) and reach.shape == (B, N)
    np.testing.assert_allclose(e, reach.sum(axis=1))


@pytest.mark.parametrize("name,method", [("specinfer", orc.SPECINFER), ("traversal", orc.TRAVERSAL)])
def test_hand_derived_worked_example(name, method):
    # tests/golden/worked_example_v3.json: stopping probabilities and block efficiency derived by hand, in fractions
    import json
    import os
    from fractions import Fraction
    with open(os.path.join(os.path.dirname(__file__), "golden", "worked_example_v3.json")) as f:
        g = json.load(f)
    parent, tokens = g["parent"], g["tokens"]
    p = [np.array(r) if r is not None else None for r in g["p"]]
    q = [np.array(r) if r is not None else None for r in g["q"]]
    reach = beo.reach_probabilities(method, parent, tokens, lambda n: p[n], lambda n: q[n])
    assert float(reach.sum()) == pytest.approx(float(Fraction(g[name]["block_efficiency"])), abs=1e-14)
    # a node is on the accepted path iff the rule stops at it or below it
    stop = {int(s): float(Fraction(fr)) for s, fr in g[name]["stop_prob"].items()}
    want = np.zeros(len(parent))
    for s, w in stop.items():
        want[0] += w
        for n in orc.path_to(parent, s):
            want[n] += w
    np.testing.assert_allclose(reach, want, atol=1e-14)
