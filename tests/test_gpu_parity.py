"""Parity of the HIP library with the fp64 oracle (needs an MI355X).

Every test goes through the C ABI (ctypes binding -> libmpv.so).  Each case
prints its name and shape before touching the GPU.
"""

import numpy as np
import pytest
import torch

import paper_2602_16994_amd as mpv
import workloads
from oracle import mpv_oracle as orc
from tests.parity_util import check_properties, compare_with_oracle, result_to_host

pytestmark = pytest.mark.gpu

SI, TV = mpv.MPV_METHOD_SPECINFER, mpv.MPV_METHOD_TRAVERSAL
NSS, NAIVE, SPECTR = mpv.MPV_METHOD_NSS, mpv.MPV_METHOD_NAIVE, mpv.MPV_METHOD_SPECTR
METHOD_NAME = {SI: "specinfer", TV: "traversal", NSS: "nss", NAIVE: "naive", SPECTR: "spectr"}
ALL_METHODS = [SI, TV, NSS, NAIVE, SPECTR]


def announce(*a):
    print("[case]", *a, flush=True)


def run_library(inputs, T, method, debug=True):
    res = mpv.mpv_verify(inputs["parent"], inputs["tokens"], inputs["target"], inputs["draft"], T,
                         inputs["uniforms"], method, debug=debug, draw_uniforms=inputs.get("draw_uniforms"))
    torch.cuda.synchronize()
    return result_to_host(res)


def run_case(cfg, method, trees=None, debug=True):
    announce(cfg.name, METHOD_NAME[method], f"B={cfg.B} N={cfg.N} V={cfg.V} {cfg.dtype} T={cfg.T}")
    inputs = workloads.make_inputs(cfg, "cuda")
    got = run_library(inputs, cfg.T, method, debug)
    if debug:
        # the production path (no debug outputs: irrelevant node tasks are skipped) must decide alike
        lean = run_library(inputs, cfg.T, method, debug=False)
        for key in ("accept_len", "path_nodes", "path_tokens", "bonus_token"):
            assert np.array_equal(got[key], lean[key]), f"{key} differs between debug and production runs"
        assert lean["counters"][4] == 0 and got["counters"][4] == 0, "dependency wait timed out"
        assert lean["counters"][5] <= got["counters"][5]
    host = workloads.to_host(inputs)
    check_properties(host["parent"], cfg.V, got, host["tokens"])
    rep = compare_with_oracle(method, host, cfg.T, got, trees=trees, check_debug=debug)
    print("[report]", rep, "counters", got["counters"].tolist(), flush=True)
    return rep, got


def assert_everything_compared(cfg, rep):
    """On the five benchmark configurations: every test that can be performed with probability above
    1e-6 is compared at the flat bar (compare_with_oracle does that for every input).  The others
    ("remote": they follow rejections that cannot happen, or the seventh and eighth rejection under
    one node) are compared with the bar float32 terms allow for the residual mass they are computed
    from; only where that mass is below float32 resolution, or at the zero-mass corner, is a number
    left out (parity_util.remote_tolerance, fragile_tests), and those must stay a minority.
    No SpecTr tolerance may hit its cap."""
    left_out = rep["fragile_tests"] + rep["noise_tests"]
    tests = rep["trees"] * (cfg.N - 1)
    assert left_out <= rep["remote_tests"] + rep["fragile_tests"] and left_out < 0.5 * tests, rep
    assert rep.get("capped_slacks", 0) == 0, rep


def run_benchmark_config(cfg, method):
    """One of the five benchmark configurations (possibly with fewer trees)."""
    rep, got = run_case(cfg, method)
    assert_everything_compared(cfg, rep)
    return rep, got


# ---------------------------------------------------------------- the five configurations

@pytest.mark.parametrize("method", ALL_METHODS)
def test_config1_tiny(method):
    run_benchmark_config(workloads.CONFIGS["tiny"], method)


def test_config2_v32k_root_specinfer():
    # full vocabulary and tree, 6 of the 64 trees
    run_benchmark_config(workloads.scaled(workloads.CONFIGS["v32k_root"], B=6), SI)


@pytest.mark.parametrize("method", ALL_METHODS)
def test_config3_v128k_delayed(method):
    run_benchmark_config(workloads.scaled(workloads.CONFIGS["v128k_delayed"], B=4), method)


def test_config4_v152k_root_traversal_small_batch():
    run_benchmark_config(workloads.scaled(workloads.CONFIGS["v152k_root"], B=3), TV)


@pytest.mark.parametrize("method", ALL_METHODS)
def test_config5_v262k_delayed(method):
    run_benchmark_config(workloads.scaled(workloads.CONFIGS["v262k_delayed"], B=2), method)


@pytest.mark.parametrize("method", [NSS, NAIVE, SPECTR])
def test_config2_and_4_token_following_walks(method):
    # the two root-expanded configurations with the solvers whose output token may be another draft token
    run_benchmark_config(workloads.scaled(workloads.CONFIGS["v32k_root"], B=6), method)
    run_benchmark_config(workloads.scaled(workloads.CONFIGS["v152k_root"], B=3), method)


@pytest.mark.parametrize("method", [NSS, NAIVE, SPECTR])
@pytest.mark.parametrize("V,dtype", [(12, "bf16"), (37, "f32")])
def test_drawn_tokens_are_followed_in_small_vocabularies(method, V, dtype):
    """With a dozen tokens the drawn token is a child's token most of the time (and equal-token
    siblings are common): the walk must move to the first such child, draw again there, and so on."""
    cfg = workloads.Config(f"follow_V{V}", B=300, V=V, K=4, L1=0, L2=3, dtype=dtype, T=1.1,
                           methods=[method], draft_sigma=1.0, target_sigma=0.6, seed=4242 + V)
    rep, got = run_case(cfg, method)
    assert rep["mean_accept_len"] > 0.1               # the walks do get somewhere
    assert np.any(got["accept_len"] >= 2)             # and some follow more than one token


class TreeRows:
    """host["target"] / host["draft"] for a batch too large to copy at once: tree b's rows are
    copied to the host (widened to float32, which is exact) when the oracle asks for them."""

    def __init__(self, tensor):
        self.tensor = tensor
        self.last = (None, None)

    def __getitem__(self, b):
        if self.last[0] != b:
            self.last = (b, self.tensor[b].float().cpu().numpy())
        return self.last[1]


def full_size_case(cfg, method, debug_trees):
    """A benchmark configuration at full size, in the launch configuration the benchmark times (no
    debug outputs): every tree's decisions against the oracle; then the per-node probabilities of
    `debug_trees`, run as a batch of their own with the debug outputs on, which must decide alike."""
    announce(cfg.name, METHOD_NAME[method], "full size", f"B={cfg.B} N={cfg.N} V={cfg.V}")
    inputs = workloads.make_inputs(cfg, "cuda")
    got = run_library(inputs, cfg.T, method, debug=False)
    assert got["counters"][4] == 0, "dependency wait timed out"
    host = {
        "parent": inputs["parent"],
        "tokens": inputs["tokens"].cpu().numpy(),
        "uniforms": inputs["uniforms"].cpu().numpy(),
        "draw_uniforms": inputs["draw_uniforms"].cpu().numpy(),
        "target": TreeRows(inputs["target"]),
        "draft": TreeRows(inputs["draft"]),
    }
    check_properties(host["parent"], cfg.V, got, host["tokens"])
    rep = compare_with_oracle(method, host, cfg.T, got, check_debug=False)
    assert rep["trees"] == cfg.B
    print("[report]", rep, "counters", got["counters"].tolist(),
          "mean accepted length (all trees)", float(got["accept_len"].mean()), flush=True)
    sub = {k: (v[debug_trees].contiguous() if torch.is_tensor(v) else v) for k, v in inputs.items()}
    got2 = run_library(sub, cfg.T, method, debug=True)
    rep2 = compare_with_oracle(method, workloads.to_host(sub), cfg.T, got2)
    if method in (SI, TV):
        assert_everything_compared(cfg, rep2)
    for key in ("accept_len", "path_nodes", "path_tokens", "bonus_token"):
        assert np.array_equal(got2[key], got[key][debug_trees]), key
    print("[report]", rep2, flush=True)


def test_config4_full_size_every_tree():
    # the batch the benchmark times: all 256 trees against the oracle, per-node probabilities of 16
    full_size_case(workloads.CONFIGS["v152k_root"], TV, list(range(0, 256, 16)))


@pytest.mark.parametrize("name,method", [("v32k_root", SI), ("v128k_delayed", SI), ("v128k_delayed", TV),
                                         ("v262k_delayed", SI), ("v262k_delayed", TV)])
def test_configs_2_3_5_full_size_every_tree(name, method):
    cfg = workloads.CONFIGS[name]
    full_size_case(cfg, method, list(range(0, cfg.B, max(1, cfg.B // 4)))[:4])


# ---------------------------------------------------------------- shapes, tails, edge cases

RAGGED = [
    # (V, dtype, K, L1, L2, B, T)
    (1000, "f32", 3, 0, 2, 5, 1.0),       # V % 4 == 0 but rows of 4000 B
    (1023, "f32", 2, 1, 2, 4, 0.7),       # rows misaligned to 16 B
    (1001, "bf16", 3, 1, 1, 4, 1.2),      # odd V: rows start at 2-byte offsets
    (50257, "bf16", 4, 0, 3, 3, 0.8),     # several tiles and a ragged tail
    (50257, "f32", 2, 2, 2, 2, 0.2),      # cold temperature
    (7, "f32", 2, 0, 2, 9, 1.0),          # vocabulary smaller than a vector tile
    (1, "bf16", 2, 0, 1, 2, 1.0),         # a single token
    (4096, "bf16", 16, 0, 1, 3, 1.0),     # maximum children under one node
    (2048, "f32", 1, 0, 12, 3, 1.0),      # one deep chain (single path)
    (8192, "bf16", 1, 5, 0, 3, 1.0),      # trunk only (K=1, L2=0)
    (3000, "bf16", 4, 3, 4, 2, 1.0),      # N = 20
]


@pytest.mark.parametrize("method", ALL_METHODS)
@pytest.mark.parametrize("V,dtype,K,L1,L2,B,T", RAGGED)
def test_ragged_shapes(method, V, dtype, K, L1, L2, B, T):
    cfg = workloads.Config(f"ragged_V{V}_{dtype}_K{K}_{L1}_{L2}", B=B, V=V, K=K, L1=L1, L2=L2, dtype=dtype,
                           T=T, methods=[method], draft_sigma=2.0, target_sigma=1.0, seed=V + 31 * K + L1)
    run_case(cfg, method)


# How a row is split over a team's workgroups (the launch picks the team size from V, B and the
# chip): the cases below sit on the edges of that choice.
TEAM_SHAPES = [
    # (V, dtype, K, L1, L2, B, T, trees compared)
    (151937, "bf16", 2, 0, 2, 130, 1.0, 12),   # more trees than teams: the fewest members that hold a row (not a power
                                              # of two), one slot per lane beyond the kept ones; odd V: misaligned rows,
                                              # head elements with the first member, tail with the last
    (450001, "bf16", 2, 0, 1, 2, 0.9, 2),      # beyond what 16 members keep on chip: the rest is read again in every sweep
    (1 << 21, "bf16", 2, 0, 1, 1, 1.0, 1),     # the largest vocabulary the boundary admits
    (300001, "f32", 2, 1, 1, 2, 1.0, 2),       # float rows, 16 members, ragged tail
    (24577, "bf16", 3, 0, 2, 200, 1.0, 8),     # a row that just fits one workgroup, many trees
]


@pytest.mark.parametrize("method", [SI, TV, mpv.MPV_METHOD_SPECTR])
@pytest.mark.parametrize("V,dtype,K,L1,L2,B,T,ntrees", TEAM_SHAPES)
def test_team_shapes(method, V, dtype, K, L1, L2, B, T, ntrees):
    cfg = workloads.Config(f"team_V{V}_{dtype}_B{B}", B=B, V=V, K=K, L1=L1, L2=L2, dtype=dtype,
                           T=T, methods=[method], draft_sigma=2.0, target_sigma=1.0, seed=V % 9973 + B)
    step = max(1, B // ntrees)
    run_case(cfg, method, trees=list(range(0, B, step))[:ntrees])


@pytest.mark.parametrize("method", [SI, TV])
@pytest.mark.parametrize("scale", [2000.0, 2e-4])
def test_logit_magnitudes(method, scale):
    """bf16 rows are kept on chip in half precision: logits of thousands and of thousandths (with a
    temperature to match) must come out as exactly as ordinary ones."""
    cfg = workloads.Config(f"scale_{scale}", B=4, V=40000, K=3, L1=1, L2=2, dtype="bf16", T=0.5 * scale,
                           methods=[method], draft_sigma=2.0 * scale, target_sigma=1.0 * scale, seed=77)
    run_case(cfg, method)


@pytest.mark.parametrize("method", ALL_METHODS)
def test_root_only_tree(method):
    # N = 1: nothing to verify, the bonus token is a plain sample from p(.|root)
    cfg = workloads.Config("root_only", B=5, V=5000, K=1, L1=0, L2=0, dtype="bf16", T=1.0,
                           methods=[method], draft_sigma=2.0, target_sigma=1.0, seed=99)
    rep, got = run_case(cfg, method)
    assert np.all(got["accept_len"] == 0)


@pytest.mark.parametrize("method", ALL_METHODS)
def test_irregular_tree(method):
    parent = [-1, 0, 0, 1, 1, 2, 5, 5, 0, 8, 9]
    announce("irregular tree", METHOD_NAME[method])
    cfg = workloads.Config("irregular", B=6, V=2500, K=1, L1=0, L2=0, dtype="f32", T=0.9,
                           methods=[method], draft_sigma=2.0, target_sigma=1.2, seed=5)
    cfg.parent = parent
    inputs = workloads.make_inputs(cfg, "cuda")
    got = run_library(inputs, cfg.T, method)
    rep = compare_with_oracle(method, workloads.to_host(inputs), cfg.T, got)
    print("[report]", rep, flush=True)


@pytest.mark.parametrize("method", [SI, TV])
def test_identical_models_accept_first_leaf(method):
    announce("p == q", METHOD_NAME[method])
    cfg = workloads.Config("same", B=4, V=3000, K=3, L1=1, L2=2, dtype="bf16", T=1.0,
                           methods=[method], draft_sigma=2.0, target_sigma=0.0, seed=17)
    inputs = workloads.make_inputs(cfg, "cuda")
    inputs["target"] = inputs["draft"].clone()
    got = run_library(inputs, cfg.T, method)
    assert np.all(got["accept_len"] == 3)
    assert np.all(got["path_nodes"] == np.array([1, 2, 3]))
    compare_with_oracle(method, workloads.to_host(inputs), cfg.T, got)


@pytest.mark.parametrize("method", ALL_METHODS)
def test_duplicate_sibling_tokens_and_masked_vocabulary(method):
    # equal tokens under one parent are separate nodes; -inf logits have zero mass
    announce("duplicates + -inf", METHOD_NAME[method])
    cfg = workloads.Config("dups", B=8, V=640, K=4, L1=0, L2=2, dtype="f32", T=1.0,
                           methods=[method], draft_sigma=1.5, target_sigma=1.5, seed=23)
    inputs = workloads.make_inputs(cfg, "cuda")
    inputs["tokens"][:, 3] = inputs["tokens"][:, 1]          # chains 1 and 2 start with the same token
    inputs["tokens"][:, 5] = inputs["tokens"][:, 1]
    inputs["target"][:, :, 100:200] = float("-inf")           # tokens the target can never emit
    got = run_library(inputs, cfg.T, method)
    host = workloads.to_host(inputs)
    compare_with_oracle(method, host, cfg.T, got)
    assert not np.any((got["bonus_token"] >= 100) & (got["bonus_token"] < 200))
    for b in range(cfg.B):
        for t in got["path_tokens"][b][: got["accept_len"][b]]:
            assert not (100 <= t < 200)


@pytest.mark.parametrize("method", ALL_METHODS)
@pytest.mark.parametrize("T", [0.2, 1.0])
def test_peaked_rows_long_vocabulary(method, T):
    """Rows kept on chip use a per-lane reference fixed at the start of the sweep;
    a few logits far above everything else (40 units, T = 0.2: 288 binary orders)
    overflow that form and must take the online repeat."""
    announce("peaked rows", METHOD_NAME[method], T)
    cfg = workloads.Config("peaked", B=3, V=131072, K=3, L1=1, L2=1, dtype="bf16", T=T,
                           methods=[method], draft_sigma=1.0, target_sigma=0.7, seed=77)
    inputs = workloads.make_inputs(cfg, "cuda")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    for name, boost in (("draft", 40.0), ("target", 38.0)):
        idx = torch.randint(4096, cfg.V, (cfg.B, cfg.N, 3), generator=gen, device="cuda")
        inputs[name].scatter_add_(2, idx, torch.full(idx.shape, boost, device="cuda", dtype=inputs[name].dtype))
    # draft tokens must still come from the (now peaked) draft rows
    for n in range(1, cfg.N):
        q = torch.softmax(inputs["draft"][:, cfg.parent[n]].float() / T, dim=-1)
        inputs["tokens"][:, n] = torch.multinomial(q, 1, generator=gen).squeeze(1).to(torch.int32)
    got = run_library(inputs, T, method)
    rep = compare_with_oracle(method, workloads.to_host(inputs), T, got)
    print("[report]", rep, flush=True)


@pytest.mark.parametrize("method", ALL_METHODS)
def test_many_small_tasks_through_the_queue(method):
    """Far more node tasks than workgroups, short rows, a bushy tree: the task queue hands out
    thousands of tasks, Traversal appends children level after level.  Decisions of every tree
    are compared with the oracle; per-node probabilities on a sample."""
    announce("queue stress", METHOD_NAME[method])
    cfg = workloads.Config("queue_stress", B=1500, V=96, K=1, L1=0, L2=0, dtype="f32", T=1.0,
                           methods=[method], draft_sigma=1.0, target_sigma=0.7, seed=404)
    cfg.parent = [-1, 0, 0, 0, 1, 1, 2, 4, 4, 5, 6, 6, 7, 9, 9, 10, 12, 13]
    inputs = workloads.make_inputs(cfg, "cuda")
    host = workloads.to_host(inputs)
    lean = run_library(inputs, cfg.T, method, debug=False)
    assert lean["counters"][4] == 0
    rep = compare_with_oracle(method, host, cfg.T, lean, check_debug=False)
    print("[report]", rep, "counters", lean["counters"].tolist(), flush=True)
    full = run_library(inputs, cfg.T, method, debug=True)
    compare_with_oracle(method, host, cfg.T, full, trees=range(0, cfg.B, 50))
    for key in ("accept_len", "path_nodes", "path_tokens", "bonus_token"):
        assert np.array_equal(full[key], lean[key])


@pytest.mark.parametrize("method", [SI, TV])
def test_more_trees_than_workgroups_delayed_tree(method):
    """More trees than workgroups, a trunk before the branching node: Traversal then handles the
    first branch before the rest of the branching node (which gets a second task only if
    nothing in that branch is accepted), SpecInfer runs only the nodes on the accepted path.
    Decisions of every tree against the oracle, and against the run that computes every node."""
    announce("many trees, delayed tree", METHOD_NAME[method])
    cfg = workloads.Config("many_delayed", B=700, V=1536, K=3, L1=2, L2=2, dtype="bf16", T=0.9,
                           methods=[method], draft_sigma=1.5, target_sigma=1.0, seed=808)
    inputs = workloads.make_inputs(cfg, "cuda")
    host = workloads.to_host(inputs)
    lean = run_library(inputs, cfg.T, method, debug=False)
    assert lean["counters"][4] == 0
    rep = compare_with_oracle(method, host, cfg.T, lean, check_debug=False)
    print("[report]", rep, "counters", lean["counters"].tolist(), flush=True)
    full = run_library(inputs, cfg.T, method, debug=True)
    compare_with_oracle(method, host, cfg.T, full, trees=range(0, cfg.B, 35))
    for key in ("accept_len", "path_nodes", "path_tokens", "bonus_token"):
        assert np.array_equal(full[key], lean[key])
    n_internal = 3 + 3                                   # root, trunk, branching node, first node of each branch
    assert full["counters"][5] == cfg.B * n_internal     # every node task ran
    assert lean["counters"][5] < full["counters"][5]     # not so when only decisions are wanted


def test_out_of_range_tokens_are_counted_not_followed():
    announce("bad tokens")
    cfg = workloads.Config("badtok", B=3, V=500, K=2, L1=0, L2=2, dtype="f32", T=1.0,
                           methods=[SI], draft_sigma=1.0, target_sigma=1.0, seed=3)
    inputs = workloads.make_inputs(cfg, "cuda")
    inputs["tokens"][:, 1] = cfg.V + 5
    inputs["tokens"][:, 3] = -2
    for method in (SI, TV):
        got = run_library(inputs, cfg.T, method, debug=False)
        assert got["counters"][3] == 2 * cfg.B
        assert np.all(got["accept_len"] == 0)


def test_empty_batch_is_a_no_op():
    announce("B = 0")
    z = torch.empty(0, 3, 16, device="cuda")
    res = mpv.mpv_verify([-1, 0, 0], torch.empty(0, 3, dtype=torch.int32, device="cuda"), z, z, 1.0,
                         torch.empty(0, 3, device="cuda"), SI, max_depth=1)
    torch.cuda.synchronize()
    assert res.accept_len.numel() == 0


def test_results_are_bitwise_reproducible():
    announce("determinism")
    cfg = workloads.scaled(workloads.CONFIGS["v128k_delayed"], B=8, V=40000)
    inputs = workloads.make_inputs(cfg, "cuda")
    a = run_library(inputs, cfg.T, TV)
    b = run_library(inputs, cfg.T, TV)
    for k in a:
        if a[k] is not None:
            assert np.array_equal(a[k], b[k], equal_nan=True), k


def test_every_uniform_decides_as_the_oracle_does():
    """Many decisions on few logits: one tree's rows are shared by 512 batch
    entries that differ only in their uniforms, so every branch of both rules is
    exercised against the oracle (whose per-node probabilities are computed once)."""
    announce("uniform sweep")
    cfg = workloads.Config("usweep", B=1, V=1500, K=3, L1=1, L2=2, dtype="bf16", T=1.0,
                           methods=[SI, TV], draft_sigma=2.0, target_sigma=1.5, seed=41)
    one = workloads.make_inputs(cfg, "cuda")
    B = 512
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)
    inputs = {
        "parent": one["parent"],
        "tokens": one["tokens"].expand(B, -1).contiguous(),
        "target": one["target"].expand(B, -1, -1).contiguous(),
        "draft": one["draft"].expand(B, -1, -1).contiguous(),
        "uniforms": torch.rand(B, cfg.N, generator=gen, device="cuda"),
    }
    host = workloads.to_host(inputs)
    for method in (SI, TV):
        got = run_library(inputs, cfg.T, method, debug=False)
        rep = compare_with_oracle(method, host, cfg.T, got, check_debug=False)
        stops = {tuple(r[:l]) for r, l in zip(got["path_nodes"].tolist(), got["accept_len"].tolist())}
        print("[report]", METHOD_NAME[method], rep, "distinct accepted paths", len(stops), flush=True)
        assert len(stops) >= 3


# ---------------------------------------------------------------- the other entry points

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("V", [1, 5, 1024, 4099, 151936])
def test_row_stats(dtype, V):
    announce("row_stats", dtype, V)
    rows = 7
    gen = torch.Generator(device="cuda")
    gen.manual_seed(V)
    z = (torch.randn(rows, V, generator=gen, device="cuda") * 4).to(dtype)
    for T in (0.2, 1.0, 1.2):
        out = mpv.mpv_row_stats(z, T).cpu().numpy().astype(np.float64)
        zz = z.float().cpu().numpy().astype(np.float64)
        m = zz.max(axis=1)
        lz = np.log(np.exp((zz - m[:, None]) / T).sum(axis=1))
        assert np.array_equal(out[:, 0], m)
        np.testing.assert_allclose(out[:, 1], lz, atol=1e-5)


def test_fill_uniforms_matches_the_documented_generator():
    announce("fill_uniforms")
    for seed, count in [(0, 1), (12345, 1000), (2 ** 63 + 11, 257)]:
        got = mpv.mpv_fill_uniforms(seed, count).cpu().numpy()
        want = orc.uniforms_from_seed(seed, count)
        assert got.dtype == np.float32 and np.array_equal(got, want)
