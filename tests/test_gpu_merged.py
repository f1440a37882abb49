"""Parity of mpv_verify_merged with the fp64 oracle on draft trees of distinct contexts
(Sec. 3, Def. 3.1; Sec. 5, Def. 5.2).  Needs an MI355X; every call goes through the C ABI.

Inputs: workloads.make_context_inputs (rows are functions of the context, so drafted paths that
share a prefix share its rows).  The merged parent arrays come from the library's own
mpv_merge_duplicates and are compared with the oracle's before anything runs on the GPU.
"""

import copy

import numpy as np
import pytest
import torch

import paper_2602_16994_amd as mpv
import workloads
from oracle import merged_tree_oracle as merged
from oracle import mpv_oracle as orc
from tests.parity_util import check_properties, compare_with_oracle, result_to_host

pytestmark = pytest.mark.gpu

SI, TV = mpv.MPV_METHOD_SPECINFER, mpv.MPV_METHOD_TRAVERSAL
NSS, NAIVE, SPECTR = mpv.MPV_METHOD_NSS, mpv.MPV_METHOD_NAIVE, mpv.MPV_METHOD_SPECTR
NAMES = {SI: "specinfer", TV: "traversal", NSS: "nss", NAIVE: "naive", SPECTR: "spectr"}


def announce(*a):
    print("[case]", *a, flush=True)


def merged_arrays(cfg, inputs):
    tokens = inputs["tokens"].cpu().numpy()
    got_p, got_c = mpv.mpv_merge_duplicates(cfg.parent, tokens)
    want_p, want_c = merged.merge_batch(cfg.parent, tokens)
    assert np.array_equal(got_p, want_p) and np.array_equal(got_c, want_c)
    assert np.array_equal(got_c, inputs["context_node"])          # the generator's own record of the contexts
    return got_p, got_c


def run_merged(inputs, cfg, method, merged_parent, debug, context_node=None):
    on_device = None
    if method == SPECTR:
        on_device = torch.as_tensor(np.ascontiguousarray(context_node, dtype=np.int32), device="cuda")
    res = mpv.mpv_verify(cfg.parent, inputs["tokens"], inputs["target"], inputs["draft"], cfg.T, inputs["uniforms"],
                         method, debug=debug, draw_uniforms=inputs["draw_uniforms"], merged_parent=merged_parent,
                         context_node=on_device)
    torch.cuda.synchronize()
    return result_to_host(res)


def runs_of(rows):
    """[(b0, b1)] runs of consecutive equal rows."""
    out = []
    b0 = 0
    for b in range(1, len(rows) + 1):
        if b == len(rows) or not np.array_equal(rows[b], rows[b0]):
            out.append((b0, b))
            b0 = b
    return out


def compare_trees(cfg, method, inputs, merged_parent, got, debug, context_node=None):
    host = workloads.to_host(inputs)
    report = {"trees": 0, "near_tie_paths": 0, "near_tie_bonus": 0, "mean_accept_len": 0.0, "max_prob_err": 0.0}
    for b in range(cfg.B):
        one = dict(host)
        one["parent"] = [int(x) for x in merged_parent[b]]
        if method == SPECTR:
            one["node_of"] = [int(x) for x in context_node[b]]
        rep = compare_with_oracle(method, one, cfg.T, got, trees=[b], check_debug=debug)
        for k in ("trees", "near_tie_paths", "near_tie_bonus"):
            report[k] += rep[k]
        report["mean_accept_len"] += rep["mean_accept_len"]
        report["max_prob_err"] = max(report["max_prob_err"], rep["max_prob_err"])
        # the oracle's merged entry point says the same as its plain one on the merged array
        if b < 4:
            ref = merged.verify_tree_merged(method, cfg.parent, host["tokens"][b], host["target"][b], host["draft"][b],
                                            cfg.T, host["uniforms"][b], host["draw_uniforms"][b])
            plain = orc.verify_tree(method, one["parent"], host["tokens"][b], host["target"][b], host["draft"][b],
                                    cfg.T, host["uniforms"][b], host["draw_uniforms"][b], node_of=one.get("node_of"))
            assert ref["path_nodes"] == plain["path_nodes"] and ref["bonus_token"] == plain["bonus_token"]
    report["mean_accept_len"] /= max(1, report["trees"])
    return report


CASES = [
    # name, B, V, K, L1, L2, dtype, T
    ("root_V6", 96, 6, 3, 0, 3, "f32", 1.0),
    ("delayed_V9", 80, 9, 4, 2, 2, "bf16", 0.8),
    ("odd_V37", 60, 37, 2, 0, 3, "f32", 1.1),            # N = 7: rows of later runs start at addresses that are not multiples of 16
    ("root_V4_k8", 64, 4, 8, 0, 2, "bf16", 1.0),         # up to eight entries under one context, most of them repeats
]


@pytest.mark.parametrize("method", [SI, TV, NSS, NAIVE, SPECTR])
@pytest.mark.parametrize("name,B,V,K,L1,L2,dtype,T", CASES)
def test_merged_trees_small_vocabularies(method, name, B, V, K, L1, L2, dtype, T):
    cfg = workloads.Config(name, B=B, V=V, K=K, L1=L1, L2=L2, dtype=dtype, T=T, methods=[method],
                           draft_sigma=1.0, target_sigma=0.6, seed=8100 + V)
    inputs = workloads.make_context_inputs(cfg, "cuda")
    mp, cn = merged_arrays(cfg, inputs)
    n_runs = len(runs_of(mp))
    announce(name, NAMES[method], f"B={B} N={cfg.N} V={V} {dtype} runs={n_runs} repeats={int((cn != np.arange(cfg.N)).sum())}")
    assert n_runs > 4
    got = run_merged(inputs, cfg, method, mp, debug=True, context_node=cn)
    lean = run_merged(inputs, cfg, method, mp, debug=False, context_node=cn)
    for key in ("accept_len", "path_nodes", "path_tokens", "bonus_token"):
        assert np.array_equal(got[key], lean[key]), key
    assert got["counters"][4] == 0 and lean["counters"][4] == 0
    rep = compare_trees(cfg, method, inputs, mp, got, debug=True, context_node=cn)
    print("[report]", rep, "counters", got["counters"].tolist(), flush=True)
    # no repeat is ever on an accepted path
    for b in range(B):
        for n in got["path_nodes"][b][:int(got["accept_len"][b])]:
            assert cn[b, int(n)] == int(n)


def test_merged_call_is_the_sum_of_its_runs():
    """One mpv_verify_merged call against one mpv_verify call per run of equal shapes on slices of
    the same tensors: every output bit for bit, counters added up."""
    cfg = workloads.Config("runs", B=60, V=301, K=3, L1=1, L2=2, dtype="bf16", T=0.9, methods=[TV],
                           draft_sigma=2.5, target_sigma=1.0, top_boost_k=2, top_boost=6.0, seed=8207)
    inputs = workloads.make_context_inputs(cfg, "cuda")
    mp, _ = merged_arrays(cfg, inputs)
    runs = runs_of(mp)
    announce("runs", f"B={cfg.B} N={cfg.N} V={cfg.V} runs={len(runs)}")
    assert 3 < len(runs) < cfg.B
    for method in (SI, TV, NAIVE):
        got = run_merged(inputs, cfg, method, mp, debug=True)
        total = np.zeros(8, dtype=np.int64)
        for b0, b1 in runs:
            part = mpv.mpv_verify([int(x) for x in mp[b0]], inputs["tokens"][b0:b1], inputs["target"][b0:b1],
                                  inputs["draft"][b0:b1], cfg.T, inputs["uniforms"][b0:b1], method, debug=True,
                                  draw_uniforms=inputs["draw_uniforms"][b0:b1], max_depth=got["path_nodes"].shape[1])
            torch.cuda.synchronize()
            part = result_to_host(part)
            for key in ("accept_len", "path_nodes", "path_tokens", "bonus_token", "accept_prob", "final_residual",
                        "stats", "edge_probs"):
                if got[key] is not None:
                    assert np.array_equal(got[key][b0:b1], part[key], equal_nan=True), (method, key, b0, b1)
            total += part["counters"].astype(np.int64)
        # counters that do not depend on which team happened to run what
        for c in (2, 3, 4):
            assert int(got["counters"][c]) == int(total[c]), (method, c)
        assert int(got["counters"][5]) > 0


def test_without_repeats_the_merged_call_is_the_plain_call():
    cfg = workloads.scaled(workloads.CONFIGS["v32k_root"], B=5)
    inputs = workloads.make_inputs(cfg, "cuda")
    tokens = inputs["tokens"].cpu().numpy()
    # make every tree free of shared prefixes: sibling tokens made distinct
    for b in range(cfg.B):
        for n in range(1, cfg.N):
            tokens[b, n] = (tokens[b, n] // 64) * 64 + n
    inputs["tokens"] = torch.as_tensor(tokens, device="cuda")
    mp, cn = mpv.mpv_merge_duplicates(cfg.parent, tokens)
    assert np.array_equal(mp, np.tile(np.array(cfg.parent, dtype=np.int32), (cfg.B, 1)))
    announce("no repeats", f"B={cfg.B} N={cfg.N} V={cfg.V}")
    for method in (SI, TV):
        a = run_merged(inputs, cfg, method, mp, debug=False)
        b = result_to_host(mpv.mpv_verify(cfg.parent, inputs["tokens"], inputs["target"], inputs["draft"], cfg.T,
                                          inputs["uniforms"], method))
        for key in ("accept_len", "path_nodes", "path_tokens", "bonus_token"):
            assert np.array_equal(a[key], b[key]), key


def test_large_vocabulary_sorted_and_unsorted():
    """Config 3's vocabulary and tree (trunk 2, then 4 paths of depth 3) with a draft that repeats
    itself often; the batch as drafted and the same batch with trees of equal shape laid next to
    each other must give every tree the same result."""
    cfg = workloads.scaled(workloads.CONFIGS["v128k_delayed"], B=12, top_boost_k=3, top_boost=8.0)
    inputs = workloads.make_context_inputs(cfg, "cuda")
    mp, cn = merged_arrays(cfg, inputs)
    order = sorted(range(cfg.B), key=lambda b: tuple(mp[b]))
    announce("v128k_delayed merged", f"B={cfg.B} N={cfg.N} V={cfg.V} runs={len(runs_of(mp))} sorted runs={len(runs_of(mp[order]))}")
    assert int((cn != np.arange(cfg.N)).sum()) > 0
    for method in (SI, TV):
        got = run_merged(inputs, cfg, method, mp, debug=True)
        assert got["counters"][4] == 0
        rep = compare_trees(cfg, method, inputs, mp, got, debug=True)
        print("[report]", rep, flush=True)
        moved = workloads.reorder_trees(inputs, order)
        again = run_merged(moved, cfg, method, mp[order], debug=False)
        for key in ("accept_len", "path_nodes", "path_tokens", "bonus_token"):
            assert np.array_equal(again[key], got[key][order]), key


def test_spectr_goes_on_below_an_accepted_repeat():
    """SpecTr tests every entry with its own uniform, so a repeat can be the accepted entry; the walk
    must then continue at the context node (whose rows and children are the repeat's context's).  A
    target much flatter than the draft makes rho* large and every single test unlikely: first entries
    fail often and later entries for the same token get their chance."""
    cfg = workloads.Config("spectr_repeats", B=400, V=5, K=6, L1=0, L2=2, dtype="f32", T=1.0, methods=[SPECTR],
                           draft_sigma=2.0, target_sigma=0.2, target_scale=0.3, seed=8421)
    inputs = workloads.make_context_inputs(cfg, "cuda")
    mp, cn = merged_arrays(cfg, inputs)
    announce("spectr repeats", f"B={cfg.B} N={cfg.N} V={cfg.V} runs={len(runs_of(mp))}")
    got = run_merged(inputs, cfg, SPECTR, mp, debug=True, context_node=cn)
    assert got["counters"][4] == 0
    rep = compare_trees(cfg, SPECTR, inputs, mp, got, debug=True, context_node=cn)
    print("[report]", rep, flush=True)
    # how often the oracle's accepted entry was a repeat (the case this test is about)
    host = workloads.to_host(inputs)
    through_repeat = 0
    for b in range(cfg.B):
        ref = merged.verify_tree_merged(SPECTR, cfg.parent, host["tokens"][b], host["target"][b], host["draft"][b],
                                        cfg.T, host["uniforms"][b], host["draw_uniforms"][b])
        through_repeat += sum(1 for node, _, _, ok in ref["decisions"] if ok and cn[b, node] != node)
    print("[report] walks that went through an accepted repeat:", through_repeat, flush=True)
    assert through_repeat >= 10
    # without the context nodes the call is refused
    with pytest.raises(mpv.MpvError) as e:
        mpv.mpv_verify(cfg.parent, inputs["tokens"], inputs["target"], inputs["draft"], cfg.T, inputs["uniforms"],
                       SPECTR, draw_uniforms=inputs["draw_uniforms"], merged_parent=mp)
    assert e.value.code == -1


@pytest.mark.parametrize("method", [SI, TV, NSS, NAIVE, SPECTR])
def test_block_efficiency_of_merged_trees(method):
    """mpv_block_efficiency_merged against the block-efficiency oracle on each tree's merged array,
    and against the unmerged estimate: under SpecInfer merging can only raise it (the child list of
    a context is the unmerged one followed by further entries)."""
    from tests.test_gpu_block_efficiency import compare
    cfg = workloads.Config("be_merged", B=48, V=11, K=3, L1=1, L2=3, dtype="bf16", T=0.9, methods=[method],
                           draft_sigma=1.2, target_sigma=0.7, seed=8311)
    inputs = workloads.make_context_inputs(cfg, "cuda")
    mp, cn = merged_arrays(cfg, inputs)
    announce("block efficiency merged", NAMES[method], f"B={cfg.B} N={cfg.N} V={cfg.V} runs={len(runs_of(mp))}")
    on_device = torch.as_tensor(cn, device="cuda") if method == SPECTR else None
    res = mpv.mpv_block_efficiency(cfg.parent, inputs["tokens"], inputs["target"], inputs["draft"], cfg.T, method,
                                   merged_parent=mp, context_node=on_device)
    torch.cuda.synchronize()
    expected, reach, counters = res.expected.cpu().numpy(), res.reach_prob.cpu().numpy(), res.counters.cpu().numpy()
    assert counters[4] == 0
    host = workloads.to_host(inputs)
    internal = 0
    for b in range(cfg.B):
        one = dict(host)
        one["parent"] = [int(x) for x in mp[b]]
        if method == SPECTR:
            one["node_of"] = [int(x) for x in cn[b]]
        compare(method, one, cfg.T, expected, reach, trees=[b])
        internal += len(set(one["parent"][1:]))
        if method in (SI, TV, SPECTR):
            # a repeat is never accepted (SpecInfer, Traversal) or its acceptance is credited to the context's node (SpecTr)
            assert np.all(reach[b][cn[b] != np.arange(cfg.N)] == 0.0)
    assert counters[5] == internal                                     # every internal node's task ran, summed over the runs
    plain = mpv.mpv_block_efficiency(cfg.parent, inputs["tokens"], inputs["target"], inputs["draft"], cfg.T, method)
    torch.cuda.synchronize()
    if method == SI:
        assert np.all(expected >= plain.expected.cpu().numpy() - 1e-5)
        assert float(expected.mean()) > float(plain.expected.mean())
    with pytest.raises(mpv.MpvError):       # SpecTr without the context nodes
        mpv.mpv_block_efficiency(cfg.parent, inputs["tokens"], inputs["target"], inputs["draft"], cfg.T, SPECTR, merged_parent=mp)


@pytest.mark.parametrize("method", [SI, NSS, NAIVE, SPECTR])
def test_acceptance_rates_of_merged_trees(method):
    """mpv_acceptance_rates_merged against the acceptance-rate oracle on each tree's merged array:
    the rate of a node depends on its two rows and on the length of its child list, in which a
    later entry for an already drafted token counts like any other."""
    from oracle import acceptance_oracle as acc
    from tests.parity_util import PROB_ATOL, spectr_slack
    cfg = workloads.Config("acc_merged", B=40, V=13, K=4, L1=1, L2=2, dtype="f32", T=1.1, methods=[method],
                           draft_sigma=1.2, target_sigma=0.7, seed=8513)
    inputs = workloads.make_context_inputs(cfg, "cuda")
    mp, cn = merged_arrays(cfg, inputs)
    announce("acceptance rates merged", NAMES[method], f"B={cfg.B} N={cfg.N} V={cfg.V} runs={len(runs_of(mp))}")
    alpha, counters = mpv.mpv_acceptance_rates(cfg.parent, inputs["target"], inputs["draft"], cfg.T, method, merged_parent=mp)
    torch.cuda.synchronize()
    got, cnt = alpha.cpu().numpy(), counters.cpu().numpy()
    host = workloads.to_host(inputs)
    internal = 0
    for b in range(cfg.B):
        parent = [int(x) for x in mp[b]]
        children = orc.children_lists(parent)
        internal += sum(1 for ch in children if ch)
        want = acc.acceptance_rates(method, parent, host["target"][b], host["draft"][b], cfg.T)
        one = dict(host)
        one["parent"] = parent
        for n in range(cfg.N):
            if not children[n]:
                assert got[b, n] == 0.0
                continue
            tol = PROB_ATOL
            if method == SPECTR and len(children[n]) > 1:
                tol += len(children[n]) * spectr_slack(one, b, n, cfg.T, len(children[n]))
            assert abs(float(got[b, n]) - want[n]) <= tol, (b, n, got[b, n], want[n])
    assert cnt[4] == 0 and cnt[5] == internal
    with pytest.raises(mpv.MpvError):
        mpv.mpv_acceptance_rates(cfg.parent, inputs["target"], inputs["draft"], cfg.T, TV, merged_parent=mp)
