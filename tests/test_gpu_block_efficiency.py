"""Parity of mpv_block_efficiency (Sec. 5, Eq. 1-3) with the fp64 oracle (needs an MI355X).

Through the C ABI (ctypes binding -> libmpv.so).  Bars: reach probabilities within
PROB_ATOL absolute (SpecTr: plus the conditioning slack of its division factor, see
tests/parity_util.py), expected block efficiency within the sum of its nodes' bars.
"""

import numpy as np
import pytest
import torch

import paper_2602_16994_amd as mpv
import workloads
from oracle import block_efficiency_oracle as beo
from oracle import mpv_oracle as orc
from tests.parity_util import PROB_ATOL, node_tolerances

pytestmark = pytest.mark.gpu

SI, TV = mpv.MPV_METHOD_SPECINFER, mpv.MPV_METHOD_TRAVERSAL
NSS, NAIVE, SPECTR = mpv.MPV_METHOD_NSS, mpv.MPV_METHOD_NAIVE, mpv.MPV_METHOD_SPECTR
METHOD_NAME = {SI: "specinfer", TV: "traversal", NSS: "nss", NAIVE: "naive", SPECTR: "spectr"}
ALL_METHODS = [SI, TV, NSS, NAIVE, SPECTR]


def announce(*a):
    print("[case]", *a, flush=True)


def run_library(inputs, T, method):
    res = mpv.mpv_block_efficiency(inputs["parent"], inputs["tokens"], inputs["target"], inputs["draft"], T, method)
    torch.cuda.synchronize()
    return res.expected.cpu().numpy(), res.reach_prob.cpu().numpy(), res.counters.cpu().numpy()


def compare(method, host, T, expected, reach, trees=None):
    B, N = host["tokens"].shape
    trees = range(B) if trees is None else trees
    worst = 0.0
    for b in trees:
        want_e, want_r = beo.expected_block_efficiency(method, host["parent"], host["tokens"][b],
                                                       host["target"][b], host["draft"][b], T,
                                                       node_of=host.get("node_of"))    # trees of distinct contexts
        tol = node_tolerances(method, host, b, T)
        err = np.abs(reach[b].astype(np.float64) - want_r)
        assert np.all(err <= tol), (f"tree {b}: reach probability off by {err.max():.3e} at node {int(err.argmax())} "
                                    f"(bar {tol[int(err.argmax())]:.1e})")
        assert abs(float(expected[b]) - want_e) <= tol.sum(), f"tree {b}: expected {expected[b]} vs {want_e}"
        worst = max(worst, float((err / tol).max()))
    return worst


def check_properties(parent, expected, reach):
    assert np.all(np.isfinite(reach)) and np.all(np.isfinite(expected))
    assert np.all(reach[:, 0] == 1.0)
    assert np.all(reach >= 0.0) and np.all(reach <= 1.0 + 1e-6)
    for n in range(1, len(parent)):
        assert np.all(reach[:, n] <= reach[:, parent[n]] + 1e-6), f"node {n} reached more often than its parent"
    np.testing.assert_allclose(expected, reach.astype(np.float64).sum(axis=1), rtol=0, atol=1e-5)


def run_case(cfg, method, trees=None):
    announce("block efficiency", cfg.name, METHOD_NAME[method], f"B={cfg.B} N={cfg.N} V={cfg.V} {cfg.dtype} T={cfg.T}")
    inputs = workloads.make_inputs(cfg, "cuda")
    expected, reach, counters = run_library(inputs, cfg.T, method)
    assert counters[4] == 0, "dependency wait timed out"
    n_internal = len(set(cfg.parent[1:]))
    assert counters[5] == cfg.B * n_internal, "every internal node's task must have run"
    check_properties(cfg.parent, expected, reach)
    host = workloads.to_host(inputs)
    worst = compare(method, host, cfg.T, expected, reach, trees)
    print("[report] worst error / bar = %.3f, mean expected block efficiency %.4f" % (worst, float(expected.mean())), flush=True)
    return expected, reach, inputs


@pytest.mark.parametrize("method", ALL_METHODS)
def test_tiny(method):
    run_case(workloads.CONFIGS["tiny"], method)


@pytest.mark.parametrize("method", ALL_METHODS)
def test_v32k_root(method):
    run_case(workloads.scaled(workloads.CONFIGS["v32k_root"], B=6), method)


@pytest.mark.parametrize("method", ALL_METHODS)
def test_v128k_delayed(method):
    run_case(workloads.scaled(workloads.CONFIGS["v128k_delayed"], B=4), method)


@pytest.mark.parametrize("method", ALL_METHODS)
def test_v152k_root_small_batch(method):
    run_case(workloads.scaled(workloads.CONFIGS["v152k_root"], B=3), method)


@pytest.mark.parametrize("method", ALL_METHODS)
def test_v262k_delayed(method):
    run_case(workloads.scaled(workloads.CONFIGS["v262k_delayed"], B=2), method)


@pytest.mark.parametrize("method", ALL_METHODS)
def test_more_trees_than_workgroups_ragged_vocabulary(method):
    # several tasks per workgroup; V not a multiple of anything; short rows (streamed, not kept on chip)
    run_case(workloads.scaled(workloads.CONFIGS["v128k_delayed"], B=300, V=1003, dtype="f32"), method)


def small_vocabulary_inputs(parent, B, V, seed, dtype=torch.float32):
    """Rows N(0, 1.5^2) + noise, tokens uniform over a small vocabulary: equal-token siblings are frequent."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    N = len(parent)
    zd = (torch.randn(B, N, V, generator=gen, device="cuda") * 1.5).to(dtype)
    zt = (zd.float() + torch.randn(B, N, V, generator=gen, device="cuda") * 0.8).to(dtype)
    tokens = torch.randint(0, V, (B, N), generator=gen, device="cuda", dtype=torch.int32)
    return {"parent": list(parent), "tokens": tokens, "target": zt, "draft": zd}


@pytest.mark.parametrize("method", ALL_METHODS)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_irregular_tree_with_equal_token_siblings(method, dtype):
    parent = [-1, 0, 0, 0, 1, 1, 2, 4, 4, 4, 3, 10]
    announce("block efficiency irregular tree", METHOD_NAME[method], dtype)
    inputs = small_vocabulary_inputs(parent, B=96, V=7, seed=11, dtype=dtype)
    expected, reach, counters = run_library(inputs, 0.9, method)
    check_properties(parent, expected, reach)
    host = {"parent": parent, "tokens": inputs["tokens"].cpu().numpy(),
            "target": inputs["target"].float().cpu().numpy(), "draft": inputs["draft"].float().cpu().numpy()}
    compare(method, host, 0.9, expected, reach)
    dup = host["tokens"][:, 1] == host["tokens"][:, 2]
    assert dup.any()
    if method in (NSS, NAIVE):                # the second of two equal-token siblings is never moved to
        assert np.all(reach[dup, 2] == 0.0) and np.all(reach[dup, 6] == 0.0)


@pytest.mark.parametrize("method", ALL_METHODS)
def test_root_only_and_single_chain(method):
    announce("block efficiency degenerate trees", METHOD_NAME[method])
    inputs = small_vocabulary_inputs([-1], B=5, V=33, seed=3)
    expected, reach, _ = run_library(inputs, 1.0, method)
    assert np.all(expected == 1.0) and np.all(reach == 1.0)
    parent = [-1, 0, 1, 2, 3]
    inputs = small_vocabulary_inputs(parent, B=40, V=9, seed=4)
    expected, reach, _ = run_library(inputs, 1.3, method)
    check_properties(parent, expected, reach)
    host = {"parent": parent, "tokens": inputs["tokens"].cpu().numpy(),
            "target": inputs["target"].cpu().numpy(), "draft": inputs["draft"].cpu().numpy()}
    compare(method, host, 1.3, expected, reach)


def test_identical_models_reach_the_first_leaf():
    parent = mpv.root_tree(3, 2)
    inputs = small_vocabulary_inputs(parent, B=16, V=50, seed=5)
    inputs["target"] = inputs["draft"].clone()
    for method in (SI, TV, NAIVE, SPECTR):
        expected, reach, _ = run_library(inputs, 1.0, method)
        np.testing.assert_allclose(expected, 3.0, atol=1e-5)
        np.testing.assert_allclose(reach[:, 1:3], 1.0, atol=1e-5)


def test_empty_batch_and_errors():
    parent = [-1, 0]
    z = torch.zeros(0, 2, 16, device="cuda")
    tok = torch.zeros(0, 2, dtype=torch.int32, device="cuda")
    res = mpv.mpv_block_efficiency(parent, tok, z, z, 1.0, SI)
    assert res.expected.numel() == 0
    inputs = small_vocabulary_inputs(parent, B=2, V=16, seed=1)
    with pytest.raises(mpv.MpvError):
        mpv.mpv_block_efficiency(parent, inputs["tokens"], inputs["target"], inputs["draft"], 1.0, 9)
    with pytest.raises(mpv.MpvError):
        mpv.mpv_block_efficiency(parent, inputs["tokens"], inputs["target"], inputs["draft"], -1.0, SI)


def test_mean_accepted_length_of_the_verification_agrees():
    # Eq. (1): the estimate is the mean of tau + 1 over the verification's own randomness
    cfg = workloads.scaled(workloads.CONFIGS["v32k_root"], B=8, V=2000)
    inputs = workloads.make_inputs(cfg, "cuda")
    runs = 300
    for method in ALL_METHODS:
        announce("block efficiency against sample means", METHOD_NAME[method])
        expected, _, _ = run_library(inputs, cfg.T, method)
        total = np.zeros(cfg.B)
        sq = np.zeros(cfg.B)
        out = None
        for r in range(runs):
            u = mpv.mpv_fill_uniforms(1000 + r, cfg.B * cfg.N).view(cfg.B, cfg.N)
            ud = mpv.mpv_fill_uniforms(5000 + r, cfg.B * cfg.N).view(cfg.B, cfg.N)
            out = mpv.mpv_verify(inputs["parent"], inputs["tokens"], inputs["target"], inputs["draft"], cfg.T,
                                 u, method, draw_uniforms=ud, out=out)
            lens = out.accept_len.cpu().numpy() + 1.0
            total += lens
            sq += lens * lens
        mean = total / runs
        sd = np.sqrt(np.maximum(sq / runs - mean * mean, 0.0) / runs)
        assert np.all(np.abs(mean - expected) <= 5.0 * sd + 1e-3), (mean, expected, sd)


def test_benchmark_batch_sampled():
    # the full benchmark batch in the launch configuration bench.py times; three trees through the oracle
    cfg = workloads.CONFIGS["v152k_root"]
    run_case(cfg, TV, trees=[0, 101, 255])
