"""mpv_verify_static (the entry point whose scratch is a device array inside the library, for
callers that cannot allocate) against mpv_verify, through the C ABI (needs an MI355X).

Two calls in a row on the same GPU, the second with a smaller input: the array keeps the first
call's contents, so the second call shows that the library clears what it needs.  The bar is the
one of the other parity tests: integer outputs identical, probabilities within 1e-5 (both entry
points run the same kernels, so they are in fact bitwise equal)."""

import numpy as np
import pytest
import torch

import paper_2602_16994_amd as mpv
import workloads
from tests.parity_util import PROB_ATOL, result_to_host

pytestmark = pytest.mark.gpu

SI, TV = mpv.MPV_METHOD_SPECINFER, mpv.MPV_METHOD_TRAVERSAL


def both(inputs, T, method, debug):
    kw = dict(debug=debug, draw_uniforms=inputs["draw_uniforms"])
    ref = mpv.mpv_verify(inputs["parent"], inputs["tokens"], inputs["target"], inputs["draft"], T,
                         inputs["uniforms"], method, **kw)
    torch.cuda.synchronize()
    got = mpv.mpv_verify(inputs["parent"], inputs["tokens"], inputs["target"], inputs["draft"], T,
                         inputs["uniforms"], method, static_scratch=True, **kw)
    torch.cuda.synchronize()
    assert got.workspace is None
    return result_to_host(ref), result_to_host(got)


def same(ref, got):
    for key in ("accept_len", "path_nodes", "path_tokens", "bonus_token"):
        assert np.array_equal(ref[key], got[key]), key
    assert got["counters"][4] == 0 and ref["counters"][4] == 0
    for key in ("accept_prob", "edge_probs", "final_residual"):
        if ref[key] is not None:
            assert np.max(np.abs(ref[key].astype(np.float64) - got[key].astype(np.float64))) <= PROB_ATOL, key


@pytest.mark.parametrize("method", [SI, TV])
def test_static_scratch_matches_workspace_entry_point_twice(method):
    big = workloads.Config("static_big", B=40, V=20011, K=3, L1=1, L2=3, dtype="bf16", T=0.9,
                           methods=[method], draft_sigma=2.0, target_sigma=1.0, seed=611)
    small = workloads.Config("static_small", B=3, V=777, K=2, L1=0, L2=2, dtype="f32", T=1.1,
                             methods=[method], draft_sigma=2.0, target_sigma=1.0, seed=612)
    for cfg in (big, small):
        print("[case] static scratch", cfg.name, method, f"B={cfg.B} N={cfg.N} V={cfg.V}", flush=True)
        inputs = workloads.make_inputs(cfg, "cuda")
        for debug in (False, True):
            ref, got = both(inputs, cfg.T, method, debug)
            same(ref, got)


def test_static_scratch_call_can_be_captured_in_a_graph():
    """The callers the entry point is for: a HIP graph that holds one call, replayed several times
    with the program's own eager calls and synchronisations in between and with new inputs written
    into the same tensors; every replay must give what the eager call gives on the same inputs."""
    cfg = workloads.Config("static_graph", B=24, V=5003, K=3, L1=1, L2=2, dtype="bf16", T=1.0,
                           methods=[TV], draft_sigma=2.0, target_sigma=1.0, seed=613)
    print("[case] static scratch under graph capture", f"B={cfg.B} N={cfg.N} V={cfg.V}", flush=True)
    inputs = workloads.make_inputs(cfg, "cuda")
    args = (inputs["parent"], inputs["tokens"], inputs["target"], inputs["draft"], cfg.T, inputs["uniforms"], TV)
    # outputs exist before the capture starts, and the library has looked up its array (first eager call)
    out = mpv.mpv_verify(*args, static_scratch=True)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        mpv.mpv_verify(*args, static_scratch=True, out=out)
    torch.cuda.synchronize()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(99)
    for replay in range(4):
        if replay:
            inputs["uniforms"].copy_(torch.rand(cfg.B, cfg.N, generator=gen, device="cuda"))
        eager = mpv.mpv_verify(*args)                      # the program's own work between replays
        torch.cuda.synchronize()
        want = result_to_host(eager)
        out.accept_len.fill_(-7)
        out.bonus_token.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        same(want, result_to_host(out))
