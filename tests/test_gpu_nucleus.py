"""Parity of mpv_nucleus_mask with the fp64 oracle, and of verification on masked rows (needs an MI355X).

Through the C ABI (ctypes binding -> libmpv.so).  Bars: the kept set, the threshold and the
number of kept tokens must be identical to the oracle's, except where the library's threshold is
the right one for a top_p within MASS_BAND of the one given (its float32 sums may stop a value
earlier or later when the mass of an upper set {z >= t} comes that close to top_p); such rows
are counted and must be few.
"""

import numpy as np
import pytest
import torch

import paper_2602_16994_amd as mpv
import workloads
from oracle import block_efficiency_oracle as beo
from oracle import mpv_oracle as orc
from oracle import nucleus_oracle as nuc
from tests.parity_util import compare_with_oracle, node_tolerances, result_to_host

pytestmark = pytest.mark.gpu

MASS_BAND = 1e-6
ALL_METHODS = [mpv.MPV_METHOD_SPECINFER, mpv.MPV_METHOD_TRAVERSAL, mpv.MPV_METHOD_NSS, mpv.MPV_METHOD_NAIVE,
               mpv.MPV_METHOD_SPECTR]


def announce(*a):
    print("[case]", *a, flush=True)


def check_rows(z, T, top_p, masked, thr, kept):
    """z: the rows given to the library (torch, on the device); the rest: its outputs."""
    zh = z.float().cpu().numpy().reshape(-1, z.shape[-1])
    mh = masked.float().cpu().numpy().reshape(zh.shape)
    th = thr.cpu().numpy().reshape(-1)
    kh = kept.cpu().numpy().reshape(-1)
    near = 0
    for r in range(len(zh)):
        tau, n_kept, margin = nuc.nucleus_threshold(zh[r], T, top_p)
        # whatever the threshold, the output is the input restricted to {z >= threshold}
        keep = zh[r] >= th[r]
        assert np.array_equal(mh[r][keep], zh[r][keep]) and np.all(np.isneginf(mh[r][~keep])), f"row {r}: not a masked copy"
        assert kh[r] == int(keep.sum()), f"row {r}: kept count {kh[r]} vs {int(keep.sum())}"
        if th[r] == tau:
            assert kh[r] == n_kept
            continue
        # another threshold: then it must be the right one for a top_p within the band of the one given,
        # i.e. its set reaches top_p - band and would not reach top_p + band without its smallest value
        p = orc.softmax_T(zh[r], T)
        with_it, without_it = float(p[keep].sum()), float(p[zh[r] > th[r]].sum())
        assert with_it >= top_p - MASS_BAND and without_it < top_p + MASS_BAND, (
            f"row {r}: threshold {th[r]} (mass {with_it:.9f}, {without_it:.9f} without its smallest value) vs "
            f"oracle {tau}, top_p {top_p}, oracle margin {margin:.3e}")
        near += 1
    return near


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("V", [1, 7, 1003, 32000, 151936])
def test_random_rows(dtype, V):
    announce("nucleus random rows", dtype, "V", V)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(V)
    rows = 24 if V > 10000 else 64
    z = (torch.randn(rows, V, generator=gen, device="cuda") * 2.5).to(dtype)
    near = 0
    for T, top_p in ((1.0, 0.9), (1.0, 0.99), (0.6, 0.5), (1.2, 0.999)):
        masked, thr, kept = mpv.mpv_nucleus_mask(z, T, top_p)
        torch.cuda.synchronize()
        near += check_rows(z, T, top_p, masked, thr, kept)
    print("[report] rows within the band:", near, "of", 4 * rows, flush=True)
    # flat rows over a large vocabulary: successive upper sets differ by 1e-7 of mass, less than
    # float32 sums resolve, so the band is hit often there (and only there)
    assert near <= (2 if V < 100000 else rows)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_equal_logits_are_kept_or_dropped_together(dtype):
    announce("nucleus ties", dtype)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(3)
    z = torch.randint(-4, 5, (48, 4099), generator=gen, device="cuda").to(dtype)      # nine distinct values
    for top_p in (0.3, 0.7, 0.95):
        masked, thr, kept = mpv.mpv_nucleus_mask(z, 1.0, top_p)
        torch.cuda.synchronize()
        assert check_rows(z, 1.0, top_p, masked, thr, kept) <= 1
        assert torch.all(kept >= (z == z.max(dim=1, keepdim=True).values).sum(dim=1))


def test_top_p_one_in_place_and_rows_with_dropped_tokens():
    announce("nucleus edge cases")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(8)
    z = (torch.randn(5, 3, 777, generator=gen, device="cuda") * 2).to(torch.bfloat16)     # leading dimensions; odd V
    masked, thr, kept = mpv.mpv_nucleus_mask(z, 1.0, 1.0)
    torch.cuda.synchronize()
    assert torch.equal(masked, z) and torch.all(kept == 777) and tuple(thr.shape) == (5, 3)
    out1, thr1, kept1 = mpv.mpv_nucleus_mask(z, 0.8, 0.9)
    z2 = z.clone()
    out2, thr2, kept2 = mpv.mpv_nucleus_mask(z2, 0.8, 0.9, inplace=True)
    torch.cuda.synchronize()
    assert out2.data_ptr() == z2.data_ptr()
    assert torch.equal(out1.view(torch.int16), out2.view(torch.int16)) and torch.equal(thr1, thr2) and torch.equal(kept1, kept2)
    # rows that already hold -inf entries
    again, thr3, kept3 = mpv.mpv_nucleus_mask(out1, 0.8, 0.5)
    torch.cuda.synchronize()
    assert check_rows(out1, 0.8, 0.5, again, thr3, kept3) <= 1
    assert torch.all(kept3 <= kept1)
    # the result is the same on every call
    out4, _, _ = mpv.mpv_nucleus_mask(z, 0.8, 0.9)
    torch.cuda.synchronize()
    assert torch.equal(out1.view(torch.int16), out4.view(torch.int16))


def test_errors():
    z = torch.zeros(2, 16, device="cuda")
    for bad in (0.0, -0.5, 1.5, float("nan")):
        with pytest.raises(mpv.MpvError):
            mpv.mpv_nucleus_mask(z, 1.0, bad)
    with pytest.raises(mpv.MpvError):
        mpv.mpv_nucleus_mask(z, 0.0, 0.9)
    empty, _, _ = mpv.mpv_nucleus_mask(torch.zeros(0, 16, device="cuda"), 1.0, 0.9)
    assert empty.numel() == 0


def nucleus_inputs(cfg, top_p):
    """cfg's inputs with both logit tensors masked by the library and the draft tokens drawn again
    from the masked draft rows (x ~ q must hold for the truncated q)."""
    inputs = workloads.make_inputs(cfg, "cuda")
    mpv.mpv_nucleus_mask(inputs["target"], cfg.T, top_p, inplace=True)
    mpv.mpv_nucleus_mask(inputs["draft"], cfg.T, top_p, inplace=True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(cfg.seed + 9)
    for n in range(1, cfg.N):
        q = torch.softmax(inputs["draft"][:, cfg.parent[n]].float() / cfg.T, dim=-1)
        inputs["tokens"][:, n] = torch.multinomial(q, 1, generator=gen).squeeze(1).to(torch.int32)
    torch.cuda.synchronize()
    return inputs


@pytest.mark.parametrize("method", ALL_METHODS)
@pytest.mark.parametrize("name,B,top_p", [("v32k_root", 6, 0.9), ("v128k_delayed", 4, 0.99), ("v152k_root", 3, 0.9)])
def test_verification_of_masked_rows(method, name, B, top_p):
    cfg = workloads.scaled(workloads.CONFIGS[name], B=B)
    announce("nucleus + verification", name, "method", method, "top_p", top_p)
    inputs = nucleus_inputs(cfg, top_p)
    assert torch.isneginf(inputs["target"]).any() and torch.isneginf(inputs["draft"]).any()
    res = mpv.mpv_verify(inputs["parent"], inputs["tokens"], inputs["target"], inputs["draft"], cfg.T,
                         inputs["uniforms"], method, debug=True, draw_uniforms=inputs["draw_uniforms"])
    torch.cuda.synchronize()
    got = result_to_host(res)
    host = workloads.to_host(inputs)
    rep = compare_with_oracle(method, host, cfg.T, got)
    print("[report]", rep, flush=True)
    # the bonus token is never a dropped one
    zt = host["target"]
    for b in range(cfg.B):
        stop = got["path_nodes"][b][got["accept_len"][b] - 1] if got["accept_len"][b] > 0 else 0
        if method in (mpv.MPV_METHOD_SPECINFER, mpv.MPV_METHOD_TRAVERSAL):
            assert np.isfinite(zt[b, stop, got["bonus_token"][b]])
    # expected block efficiency on the same masked rows
    be = mpv.mpv_block_efficiency(inputs["parent"], inputs["tokens"], inputs["target"], inputs["draft"], cfg.T, method)
    torch.cuda.synchronize()
    reach = be.reach_prob.cpu().numpy()
    for b in range(cfg.B):
        _, want = beo.expected_block_efficiency(method, host["parent"], host["tokens"][b], host["target"][b],
                                                host["draft"][b], cfg.T)
        tol = node_tolerances(method, host, b, cfg.T)          # 1e-5, plus SpecTr's (capped) conditioning slack
        assert np.all(np.abs(reach[b] - want) <= tol), (b, float(np.max(np.abs(reach[b] - want) - tol)))


def test_benchmark_batch_rows_sampled():
    # every row of the benchmark batch's target tensor in one launch; a sample of rows through the oracle
    cfg = workloads.CONFIGS["v152k_root"]
    announce("nucleus on the benchmark batch", f"rows={cfg.B * cfg.N} V={cfg.V}")
    inputs = workloads.make_inputs(cfg, "cuda")
    z = inputs["target"]
    masked, thr, kept = mpv.mpv_nucleus_mask(z, cfg.T, 0.9)
    torch.cuda.synchronize()
    flat = z.view(-1, cfg.V)
    rows = [0, 1, 4099, 7777, cfg.B * cfg.N - 1]
    near = check_rows(flat[rows], cfg.T, 0.9, masked.view(-1, cfg.V)[rows], thr.view(-1)[rows], kept.view(-1)[rows])
    assert near <= 1
    assert int(kept.min()) >= 1 and int(kept.max()) < cfg.V
