"""Pins for the tolerance models the parity tests use (no GPU).

* spectr_conditioning: the bound it states, |d ln rho*| <= kappa * e for relative errors e of the
  V-wide sums, is checked by perturbing P and Q and solving SpecTr's equation again in the form
  the paper prints it (App. B, Alg. 3: p_acc(rho) = rho * beta(rho)).
* the oracle's rewritten root function against the printed one, also where p is close to q (the
  case the rewriting exists for).
* fragile_tests: flags exactly the corner of the zero-mass rule, nothing else.
"""

import numpy as np
import pytest

from oracle import mpv_oracle as orc
from tests import parity_util as pu


def random_dist(rng, V, peak=0.0):
    z = rng.normal(size=V) * 2.0
    if peak:
        z[rng.integers(V)] += peak
    return orc.softmax_T(z, 1.0)


def printed_root(P, Q, k, lo=1.0, hi=None, iters=200):
    """Root of  1 - (1 - beta(rho))^k - rho * beta(rho)  on [1, k], beta = sum min(p/rho, q), by
    bisection on the expression exactly as printed (unnormalised P, Q are allowed: this is what
    a computation with slightly wrong sums effectively solves)."""
    hi = float(k) if hi is None else hi

    def f(rho):
        beta = float(np.sum(np.minimum(P / rho, Q)))
        return 1.0 - (1.0 - beta) ** k - rho * beta

    if f(lo) <= 0.0:
        return lo
    if f(hi) >= 0.0:
        return hi
    for _ in range(iters):
        mid = 0.5 * (lo + hi)
        if f(mid) > 0.0:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


@pytest.mark.parametrize("seed", range(12))
@pytest.mark.parametrize("k", [2, 4, 8])
def test_spectr_conditioning_bounds_the_root_shift(seed, k):
    rng = np.random.default_rng(1000 * k + seed)
    V = int(rng.integers(6, 400))
    # every third case has a dominant token, where the root tends to sit on a kink
    P, Q = random_dist(rng, V, 6.0 if seed % 3 == 0 else 0.0), random_dist(rng, V, 5.0 if seed % 3 == 0 else 0.0)
    rho = orc.spectr_division_factor(P, Q, k)
    kappa = pu.spectr_conditioning(P, Q, k, rho)
    if not (1.0 + 1e-9 < rho < k - 1e-9) or not np.isfinite(kappa):
        pytest.skip("root at an end of [1, k]: nothing to move")
    # the printed form and the oracle's agree to start with
    assert abs(np.log(printed_root(P, Q, k)) - np.log(rho)) < 1e-9
    e = 1e-7
    worst = 0.0
    for sp, sq in ((1, 0), (-1, 0), (0, 1), (0, -1), (1, -1), (-1, 1), (1, 1), (-1, -1)):
        moved = printed_root(P * (1.0 + sp * e), Q * (1.0 + sq * e), k)
        worst = max(worst, abs(np.log(moved) - np.log(rho)))
    # first-order bound, with room for its second-order remainder and the bisection's own 1e-12
    assert worst <= kappa * e * 1.05 + 1e-11, (worst / e, kappa)


def test_spectr_conditioning_is_not_vacuous():
    # a well-conditioned case has a kappa of order one: the bound is tight enough to bite
    rng = np.random.default_rng(5)
    ks = []
    for _ in range(20):
        P, Q = random_dist(rng, 50), random_dist(rng, 50)
        rho = orc.spectr_division_factor(P, Q, 4)
        if 1.0 < rho < 4.0:
            ks.append(pu.spectr_conditioning(P, Q, 4, rho))
    assert ks and np.median(ks) < 20.0 and min(ks) > 0.1


def test_spectr_slack_is_capped():
    # p = q: the root function vanishes identically, the conditioning is unbounded, the slack is not
    z = np.linspace(-2, 2, 33)[None, :].repeat(2, axis=0)
    host = {"target": [z], "draft": [z]}
    capped = []
    s = pu.spectr_slack(host, 0, 0, 1.0, 4, capped)
    assert s <= pu.SPECTR_SLACK_CAP
    assert (s == pu.SPECTR_SLACK_CAP) == (len(capped) == 1)


@pytest.mark.parametrize("seed", range(8))
def test_rewritten_root_function_agrees_with_the_printed_one(seed):
    # App. B, SpecTr: the oracle evaluates p_acc - rho beta as sum (p - rho q)_+ - (sum (q - p/rho)_+)^k.
    # Where p is far from q both forms have the same root to 1e-12; where p is within 1e-9 of q the
    # printed form has lost the root to rounding, and the rewritten form's root still satisfies the
    # printed equation as well as float64 can tell.
    rng = np.random.default_rng(300 + seed)
    V, k = 40, 2 + seed % 5
    Q = random_dist(rng, V)
    P = random_dist(rng, V, 3.0)
    rho = orc.spectr_division_factor(P, Q, k)
    if 1.0 < rho < k:
        assert abs(printed_root(P, Q, k) - rho) < 1e-10
    beta = orc.spectr_beta(P, Q, rho)
    assert abs((1.0 - (1.0 - beta) ** k) - rho * beta) < 1e-12
    # p close to q
    d = rng.normal(size=V)
    d -= d.mean()
    Pn = np.maximum(Q + 1e-9 * d * Q, 0.0)
    Pn /= Pn.sum()
    rho_n = orc.spectr_division_factor(Pn, Q, k)
    beta_n = orc.spectr_beta(Pn, Q, rho_n)
    assert 1.0 <= rho_n <= k
    assert abs((1.0 - (1.0 - beta_n) ** k) - rho_n * beta_n) < 1e-12       # it solves the printed equation
    # and it is the exact root of the rewritten function: the sign changes across it
    def g(r):
        return float(np.sum(np.maximum(Pn - r * Q, 0.0))) - float(np.sum(np.maximum(Q - Pn / r, 0.0))) ** k
    if 1.0 < rho_n < k:
        assert g(rho_n * (1 - 1e-12)) >= 0.0 >= g(rho_n * (1 + 1e-12))


def test_fragile_tests_flags_only_the_zero_mass_corner():
    parent = [-1, 0, 1, 0, 3]
    children = orc.children_lists(parent)
    rng = np.random.default_rng(2)
    V = 12
    zt, zd = rng.normal(size=(5, V)), rng.normal(size=(5, V))
    tokens = np.array([0, 3, 4, 5, 6])
    for method in (orc.SPECINFER, orc.TRAVERSAL):
        ups = []
        orc.all_test_probs(method, parent, tokens, zt, zd, 1.0, ups)
        assert ups, "every rejected child reports an update"
        assert not pu.fragile_tests(method, parent, children, ups).any()
    # identical models: at the root (weight 1) the residual after the first rejection has no mass
    for method in (orc.SPECINFER, orc.TRAVERSAL):
        ups = []
        orc.all_test_probs(method, parent, tokens, zd, zd, 1.0, ups)
        fr = pu.fragile_tests(method, parent, children, ups)
        assert fr[3]                                    # the root's second child follows the corner
        assert not fr[0] and not fr[2]                  # nothing precedes the first leaf's test
        # Traversal: node 1's own test follows the corner at node 1 (its child rejected, weight 1, no mass),
        # and node 4's weight descends from the root's state after the corner at the root
        assert fr[1] == (method == orc.TRAVERSAL)
        assert fr[4] == (method == orc.TRAVERSAL)
    # a zero mass next to a weight well below 1 is the continuous side of the rule: not flagged
    ups = [(1, 2, 0.4, 0.0)]
    assert not pu.fragile_tests(orc.TRAVERSAL, parent, children, ups).any()


def test_update_hooks_report_without_changing_results():
    rng = np.random.default_rng(8)
    parent = [-1, 0, 0, 1, 2]
    V = 9
    zt, zd = rng.normal(size=(5, V)), rng.normal(size=(5, V))
    tokens = rng.integers(V, size=5)
    for method in (orc.SPECINFER, orc.TRAVERSAL):
        a, da = orc.all_test_probs(method, parent, tokens, zt, zd, 0.9)
        ups = []
        b, db = orc.all_test_probs(method, parent, tokens, zt, zd, 0.9, ups)
        assert np.array_equal(a, b, equal_nan=True)
        for x, y in zip(da, db):
            assert np.array_equal(x, y)
        # the masses are those of the definition: sum (a P - q)_+ with the state at that moment
        n, c, w, m = next(u for u in ups if u[0] == 0)             # the root's first update
        P, Q = orc.softmax_T(zt[n], 0.9), orc.softmax_T(zd[n], 0.9)
        assert n == 0 and c == 1 and w == 1.0
        assert abs(m - np.sum(np.maximum(P - Q, 0.0))) < 1e-15


def float32_term_specinfer(P64, Q64, xs):
    """App. B Alg. 4's test probabilities through the state (c, W) over the original rows, W summed
    from float32 terms: a model of what any streaming float32 evaluation can deliver."""
    P, Q = P64.astype(np.float32), Q64.astype(np.float32)
    c, W, out = 0.0, 1.0, []
    for x in xs:
        num = max(P64[x] - c * Q64[x], 0.0)
        out.append(min(1.0, num / (W * Q64[x])) if Q64[x] > 0 else (1.0 if num > 0 else 0.0))
        c2 = c + W
        W2 = float(np.maximum(P - np.float32(c2) * Q, np.float32(0)).astype(np.float64).sum())
        if W2 > 0.0:
            c, W = c2, W2
    return np.array(out)


@pytest.mark.parametrize("seed", range(10))
def test_remote_tolerance_covers_float32_terms(seed):
    # peaked rows, every child carrying the dominant token: each rejection leaves a residual mass
    # orders of magnitude smaller, until it is below float32 resolution
    rng = np.random.default_rng(40 + seed)
    V, k = 3000, 5
    zd = rng.normal(size=V) * 2.0
    zd[rng.integers(V)] += 6.0 + 2.0 * (seed % 4)
    zt = zd + rng.normal(size=V) * 0.7
    T = 0.6
    P, Q = orc.softmax_T(zt, T), orc.softmax_T(zd, T)
    x = int(np.argmax(Q))
    parent = [-1] + [0] * k
    children = orc.children_lists(parent)
    tokens = np.array([0] + [x] * k)
    Zt, Zd = np.stack([zt] * (k + 1)), np.stack([zd] * (k + 1))
    ups = []
    want, _ = orc.all_test_probs(orc.SPECINFER, parent, tokens, Zt, Zd, T, ups)
    got = float32_term_specinfer(P, Q, [x] * k)
    tol = pu.remote_tolerance(orc.SPECINFER, parent, children, ups)
    err = np.abs(got - want[1:])
    assert np.all(err <= tol[1:]), (err, tol[1:])
    assert np.isfinite(tol[1]) and tol[1] < 2e-5          # a clean history keeps (nearly) the plain bar
