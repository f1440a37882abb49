"""Pins for the nucleus (top-p) oracle (Sec. 4.1 names the setting; the definition is the usual one).

None of these call the HIP library."""

import itertools

import numpy as np
import pytest

from oracle import mpv_oracle as orc
from oracle import nucleus_oracle as nuc


def textbook_top_p(z, T, top_p):
    """Sort by probability, cumulative sum, keep up to and including the first index that reaches top_p."""
    p = orc.softmax_T(z, T)
    order = np.argsort(-p, kind="stable")
    csum = np.cumsum(p[order])
    cut = int(np.searchsorted(csum, top_p, side="left"))
    keep = np.zeros(len(z), dtype=bool)
    keep[order[:cut + 1]] = True
    return keep


@pytest.mark.parametrize("top_p", [0.5, 0.9, 0.99])
@pytest.mark.parametrize("T", [0.6, 1.0, 1.3])
def test_equals_the_textbook_procedure_when_logits_are_distinct(top_p, T):
    rng = np.random.default_rng(int(100 * top_p) + int(10 * T))
    for _ in range(20):
        z = rng.normal(0, 2.5, size=200)
        masked = nuc.nucleus_mask(z, T, top_p)
        assert np.array_equal(np.isfinite(masked), textbook_top_p(z, T, top_p))
        assert np.array_equal(masked[np.isfinite(masked)], z[np.isfinite(masked)])


def test_smallest_upper_set_that_reaches_top_p_by_brute_force():
    rng = np.random.default_rng(5)
    for _ in range(200):
        V = int(rng.integers(2, 8))
        z = rng.integers(-3, 4, size=V).astype(np.float64)          # many equal logits
        T = float(rng.choice([0.5, 1.0, 2.0]))
        top_p = float(rng.uniform(0.05, 1.0))
        p = orc.softmax_T(z, T)
        best = None
        for t in np.unique(z):                                        # every upper set {z >= t}
            keep = z >= t
            if p[keep].sum() >= top_p and (best is None or keep.sum() < best.sum()):
                best = keep
        tau, kept, _ = nuc.nucleus_threshold(z, T, top_p)
        assert np.array_equal(z >= tau, best) and kept == int(best.sum())


def test_edge_values_of_top_p_and_invariants():
    rng = np.random.default_rng(9)
    z = rng.normal(0, 3, size=500)
    z[7] = z[11] = z.max()                                            # the maximum is attained three times
    assert np.all(np.isfinite(nuc.nucleus_mask(z, 1.0, 1.0)))         # top_p = 1 keeps everything
    tiny = nuc.nucleus_mask(z, 1.0, 1e-9)
    assert np.count_nonzero(np.isfinite(tiny)) == 3                   # only the (tied) maximum
    for top_p in (0.3, 0.9, 0.99):
        tau, kept, margin = nuc.nucleus_threshold(z, 0.8, top_p)
        p = orc.softmax_T(z, 0.8)
        assert p[z >= tau].sum() >= top_p                             # reaches top_p ...
        assert p[z > tau].sum() < top_p                               # ... and not without its last value
        assert kept == np.count_nonzero(z >= tau) and margin >= 0.0
        # later steps see the renormalised restriction of p
        q = orc.softmax_T(nuc.nucleus_mask(z, 0.8, top_p), 0.8)
        want = np.where(z >= tau, p, 0.0)
        np.testing.assert_allclose(q, want / want.sum(), atol=1e-15)


def test_verification_of_masked_rows_is_lossless_for_the_truncated_target():
    # the transform commutes with everything after it: verification on masked logits is verification
    # with the truncated distributions (exactly lossless for the truncated target, as for any p and q)
    parent = [-1, 0, 0]
    V = 4
    rng = np.random.default_rng(2)
    zt = rng.normal(0, 1.5, size=(3, V))
    zd = rng.normal(0, 1.5, size=(3, V))
    zt_m, _, _, _ = nuc.nucleus_mask_rows(zt, 1.0, 0.8)
    zd_m, _, _, _ = nuc.nucleus_mask_rows(zd, 1.0, 0.8)
    p_rows = [orc.softmax_T(r, 1.0) for r in zt_m]
    q_rows = [orc.softmax_T(r, 1.0) for r in zd_m]
    for method in (orc.SPECINFER, orc.TRAVERSAL):
        out = np.zeros(V)
        for x1, x2 in itertools.product(range(V), repeat=2):
            w = q_rows[0][x1] * q_rows[0][x2]
            if w == 0.0:
                continue
            outs = orc.enumerate_outcomes(method, parent, (0, x1, x2), lambda n: p_rows[n], lambda n: q_rows[n])
            for pr, stop, P in outs:
                if stop == 0:
                    out += w * pr * P
                else:
                    out[(x1, x2)[stop - 1]] += w * pr
        np.testing.assert_allclose(out, p_rows[0], atol=1e-12)       # first emitted token ~ truncated target
