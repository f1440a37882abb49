"""Host-side checks that need no GPU: the library loads, exports what
include/mpv.h declares, and validates its arguments before launching anything."""

import ctypes
import os
import re

import numpy as np
import pytest

import paper_2602_16994_amd as mpv
from paper_2602_16994_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return mpv.load_library()


def header_text():
    with open(os.path.join(ROOT, "include", "mpv.h")) as f:
        return f.read()


def test_library_exports_every_declared_symbol(lib):
    text = re.sub(r"/\*.*?\*/", "", header_text(), flags=re.S)
    names = set(re.findall(r"\b(mpv_[a-z_]+)\s*\(", text))
    assert {"mpv_version", "mpv_strerror", "mpv_last_hip_error", "mpv_workspace_bytes",
            "mpv_verify", "mpv_verify_static", "mpv_merge_duplicates", "mpv_verify_merged", "mpv_block_efficiency_merged", "mpv_acceptance_rates_merged", "mpv_block_efficiency", "mpv_acceptance_rates", "mpv_nucleus_mask", "mpv_row_stats", "mpv_fill_uniforms", "mpv_timing_enable",
            "mpv_timing_read"} <= names
    for name in names:
        assert getattr(lib, name) is not None, name


def test_version_and_error_strings(lib):
    m = re.search(r"#define MPV_ABI_VERSION (\d+)", header_text())
    assert mpv.mpv_version() == int(m.group(1))
    codes = dict(re.findall(r"#define (MPV_(?:OK|ERR_[A-Z_]+))\s+(-?\d+)", header_text()))
    assert len(codes) >= 10
    seen = set()
    for name, code in codes.items():
        s = mpv.mpv_strerror(int(code))
        assert s and s != "unknown error code", name
        seen.add(s)
    assert len(seen) == len(codes)
    assert mpv.mpv_strerror(-12345) == "unknown error code"


def header_constant(name):
    m = re.search(r"#define %s\s+\(?([^)\n/]+)\)?" % name, header_text())
    return eval(m.group(1))


def problem(B=2, N=3, V=16, method=0, dtype=0, T=1.0, max_depth=2, parent=(-1, 0, 1)):
    return binding._make_problem(B, N, V, method, dtype, T, max_depth, list(parent) if parent is not None else None)


def ws_bytes(lib, prob):
    out = ctypes.c_size_t(0)
    return lib.mpv_workspace_bytes(ctypes.byref(prob), ctypes.byref(out)), out.value


def code(name):
    return header_constant(name)


def test_problem_validation(lib):
    assert ws_bytes(lib, problem())[0] == 0
    assert ws_bytes(lib, problem(B=-1))[0] == code("MPV_ERR_BAD_SHAPE")
    assert ws_bytes(lib, problem(V=0))[0] == code("MPV_ERR_BAD_SHAPE")
    assert ws_bytes(lib, problem(max_depth=1))[0] == code("MPV_ERR_BAD_SHAPE")
    assert ws_bytes(lib, problem(parent=(0, 0, 1)))[0] == code("MPV_ERR_BAD_TREE")
    assert ws_bytes(lib, problem(parent=(-1, 1, 0)))[0] == code("MPV_ERR_BAD_TREE")
    assert ws_bytes(lib, problem(parent=(-1, 0, 2)))[0] == code("MPV_ERR_BAD_TREE")
    assert ws_bytes(lib, problem(parent=(-1, -1, 0)))[0] == code("MPV_ERR_BAD_TREE")
    assert ws_bytes(lib, problem(parent=None))[0] == code("MPV_ERR_NULL")
    assert ws_bytes(lib, problem(T=0.0))[0] == code("MPV_ERR_BAD_TEMPERATURE")
    assert ws_bytes(lib, problem(T=-1.0))[0] == code("MPV_ERR_BAD_TEMPERATURE")
    assert ws_bytes(lib, problem(T=float("nan")))[0] == code("MPV_ERR_BAD_TEMPERATURE")
    assert ws_bytes(lib, problem(T=float("inf")))[0] == code("MPV_ERR_BAD_TEMPERATURE")
    assert ws_bytes(lib, problem(method=5))[0] == code("MPV_ERR_BAD_METHOD")
    assert ws_bytes(lib, problem(method=-1))[0] == code("MPV_ERR_BAD_METHOD")
    assert ws_bytes(lib, problem(method=4))[0] == 0
    assert ws_bytes(lib, problem(dtype=5))[0] == code("MPV_ERR_BAD_DTYPE")
    assert lib.mpv_workspace_bytes(None, ctypes.byref(ctypes.c_size_t(0))) == code("MPV_ERR_NULL")
    assert lib.mpv_workspace_bytes(ctypes.byref(problem()), None) == code("MPV_ERR_NULL")


def test_limits(lib):
    max_nodes, max_children, max_vocab = (header_constant(n) for n in
                                          ("MPV_MAX_NODES", "MPV_MAX_CHILDREN", "MPV_MAX_VOCAB"))
    ok = [-1] + list(range(max_nodes - 1))                    # one chain of the maximum size
    assert ws_bytes(lib, problem(N=max_nodes, parent=ok, max_depth=max_nodes))[0] == 0
    too_many = [-1] + list(range(max_nodes))
    assert ws_bytes(lib, problem(N=max_nodes + 1, parent=too_many, max_depth=99))[0] == code("MPV_ERR_UNSUPPORTED")
    star = [-1] + [0] * max_children
    assert ws_bytes(lib, problem(N=len(star), parent=star, max_depth=1))[0] == 0
    star.append(0)
    assert ws_bytes(lib, problem(N=len(star), parent=star, max_depth=1))[0] == code("MPV_ERR_UNSUPPORTED")
    assert ws_bytes(lib, problem(V=max_vocab))[0] == 0
    assert ws_bytes(lib, problem(V=max_vocab + 1))[0] == code("MPV_ERR_UNSUPPORTED")
    assert ws_bytes(lib, problem(B=(1 << 30) // 5))[0] == 0                      # B * (N + 2) = 2^30 at N = 3
    assert ws_bytes(lib, problem(B=(1 << 30) // 5 + 1))[0] == code("MPV_ERR_UNSUPPORTED")


def test_workspace_size_scales_with_batch_and_nodes(lib):
    rc, a = ws_bytes(lib, problem(B=1))
    rc, b = ws_bytes(lib, problem(B=1000))
    assert a >= 256 and a % 256 == 0 and b % 256 == 0 and b > a
    # a few dozen bytes per (tree, node) and per tree, plus a fixed part (queue control, the teams'
    # exchange areas, the launch block) of under 200 KB
    assert b - a < 1000 * (3 * 64 + 32) and a < 200 * 1024


def test_verify_rejects_bad_arguments_before_any_launch(lib):
    bufs = binding._Buffers()
    prob = problem()
    fake = ctypes.c_void_p(4096)
    # null buffer struct, null members
    assert lib.mpv_verify(ctypes.byref(prob), None, fake, 1 << 20, None) == code("MPV_ERR_NULL")
    assert lib.mpv_verify(ctypes.byref(prob), ctypes.byref(bufs), fake, 1 << 20, None) == code("MPV_ERR_NULL")
    for name, _ in binding._Buffers._fields_[:9]:
        setattr(bufs, name, 4096)
    # misaligned logits
    bufs.target_logits = 4096 + 4
    assert lib.mpv_verify(ctypes.byref(prob), ctypes.byref(bufs), fake, 1 << 20, None) == code("MPV_ERR_ALIGNMENT")
    bufs.target_logits = 4096
    # workspace: null, misaligned, too small
    assert lib.mpv_verify(ctypes.byref(prob), ctypes.byref(bufs), None, 1 << 20, None) == code("MPV_ERR_WORKSPACE")
    assert lib.mpv_verify(ctypes.byref(prob), ctypes.byref(bufs), ctypes.c_void_p(4096 + 8), 1 << 20, None) == code("MPV_ERR_WORKSPACE")
    assert lib.mpv_verify(ctypes.byref(prob), ctypes.byref(bufs), fake, 16, None) == code("MPV_ERR_WORKSPACE")
    # an invalid problem wins over everything else
    assert lib.mpv_verify(ctypes.byref(problem(T=0.0)), ctypes.byref(bufs), fake, 1 << 20, None) == code("MPV_ERR_BAD_TEMPERATURE")
    # an empty batch is a no-op that needs no buffers
    assert lib.mpv_verify(ctypes.byref(problem(B=0)), ctypes.byref(binding._Buffers()), None, 0, None) == 0


def test_other_entry_points_validate(lib):
    assert lib.mpv_row_stats(None, 0, 1, 8, 1.0, None, None) == code("MPV_ERR_NULL")
    assert lib.mpv_row_stats(4096, 0, -1, 8, 1.0, 4096, None) == code("MPV_ERR_BAD_SHAPE")
    assert lib.mpv_row_stats(4096, 7, 1, 8, 1.0, 4096, None) == code("MPV_ERR_BAD_DTYPE")
    assert lib.mpv_row_stats(4096, 0, 1, 8, 0.0, 4096, None) == code("MPV_ERR_BAD_TEMPERATURE")
    assert lib.mpv_row_stats(4096, 0, 0, 8, 1.0, 4096, None) == 0
    assert lib.mpv_fill_uniforms(1, -1, 4096, None) == code("MPV_ERR_BAD_SHAPE")
    assert lib.mpv_fill_uniforms(1, 0, None, None) == 0
    assert lib.mpv_fill_uniforms(1, 5, None, None) == code("MPV_ERR_NULL")


def test_tree_builders():
    assert mpv.root_tree(2, 3) == [-1, 0, 1, 2, 0, 4, 5]
    assert mpv.delayed_tree(4, 2, 3) == [-1, 0, 1, 2, 3, 4, 2, 6, 7, 2, 9, 10, 2, 12, 13]
    assert len(mpv.root_tree(8, 5)) == 41 and len(mpv.delayed_tree(8, 3, 3)) == 28
    assert len(mpv.root_tree(4, 4)) == 17
    assert mpv.tree_depth(mpv.delayed_tree(8, 3, 3)) == 6
    with pytest.raises(ValueError):
        mpv.delayed_tree(0, 1, 1)


def test_binding_refuses_host_tensors():
    import torch
    z = torch.zeros(1, 3, 8)
    with pytest.raises(ValueError):
        mpv.mpv_verify([-1, 0, 1], torch.zeros(1, 3, dtype=torch.int32), z, z, 1.0, torch.zeros(1, 3), 0)


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(FileNotFoundError):
        binding.load_library(str(tmp_path / "libmpv.so"))


def test_workload_generator_is_seeded_and_shaped():
    import torch
    import workloads
    cfg = workloads.scaled(workloads.CONFIGS["v128k_delayed"], B=2, V=300)
    a = workloads.make_inputs(cfg, "cpu")
    b = workloads.make_inputs(cfg, "cpu")
    assert a["target"].dtype == torch.bfloat16 and tuple(a["target"].shape) == (2, 15, 300)
    for k in ("tokens", "target", "draft", "uniforms"):
        assert torch.equal(a[k], b[k])
    assert a["tokens"].min() >= 0 and a["tokens"].max() < 300
    assert float(a["uniforms"].min()) >= 0.0 and float(a["uniforms"].max()) < 1.0
    h = workloads.to_host(a)
    assert h["target"].dtype == np.float32
    # the five configurations have the node counts the benchmark definition states
    assert [workloads.CONFIGS[k].N for k in ("tiny", "v32k_root", "v128k_delayed", "v152k_root", "v262k_delayed")] \
        == [7, 17, 15, 41, 28]


def test_estimator_entry_points_reject_bad_arguments_before_any_launch(lib):
    prob = problem()
    fake = ctypes.c_void_p(4096)
    null = ctypes.c_void_p(0)
    # expected block efficiency: null inputs / outputs, alignment, workspace, invalid problem, empty batch
    be = lib.mpv_block_efficiency
    assert be(ctypes.byref(prob), null, fake, fake, fake, 1 << 20, fake, fake, fake, None) == code("MPV_ERR_NULL")
    assert be(ctypes.byref(prob), fake, fake, fake, fake, 1 << 20, fake, null, fake, None) == code("MPV_ERR_NULL")
    assert be(ctypes.byref(prob), fake, fake, fake, fake, 1 << 20, fake, fake, null, None) == code("MPV_ERR_NULL")
    assert be(ctypes.byref(prob), ctypes.c_void_p(4100), fake, fake, fake, 1 << 20, fake, fake, fake, None) == code("MPV_ERR_ALIGNMENT")
    assert be(ctypes.byref(prob), fake, fake, fake, null, 1 << 20, fake, fake, fake, None) == code("MPV_ERR_WORKSPACE")
    assert be(ctypes.byref(prob), fake, fake, fake, fake, 16, fake, fake, fake, None) == code("MPV_ERR_WORKSPACE")
    assert be(ctypes.byref(problem(method=7)), fake, fake, fake, fake, 1 << 20, fake, fake, fake, None) == code("MPV_ERR_BAD_METHOD")
    assert be(ctypes.byref(problem(B=0)), null, null, null, null, 0, null, null, null, None) == 0
    # acceptance rates: the same, and Traversal is not an OTLP solver
    ar = lib.mpv_acceptance_rates
    assert ar(ctypes.byref(problem(method=1)), fake, fake, fake, 1 << 20, fake, fake, None) == code("MPV_ERR_UNSUPPORTED")
    assert ar(ctypes.byref(prob), fake, null, fake, 1 << 20, fake, fake, None) == code("MPV_ERR_NULL")
    assert ar(ctypes.byref(prob), fake, fake, fake, 1 << 20, null, fake, None) == code("MPV_ERR_NULL")
    assert ar(ctypes.byref(prob), fake, fake, fake, 8, fake, fake, None) == code("MPV_ERR_WORKSPACE")
    assert ar(ctypes.byref(problem(B=0)), null, null, null, 0, null, null, None) == 0


def test_nucleus_entry_point_rejects_bad_arguments_before_any_launch(lib):
    nm = lib.mpv_nucleus_mask
    fake = ctypes.c_void_p(4096)
    null = ctypes.c_void_p(0)
    f = ctypes.c_float
    assert nm(fake, fake, 0, -1, 8, f(1.0), f(0.9), null, null, None) == code("MPV_ERR_BAD_SHAPE")
    assert nm(fake, fake, 0, 1, 0, f(1.0), f(0.9), null, null, None) == code("MPV_ERR_BAD_SHAPE")
    assert nm(fake, fake, 0, 1, header_constant("MPV_MAX_VOCAB") + 1, f(1.0), f(0.9), null, null, None) == code("MPV_ERR_UNSUPPORTED")
    assert nm(fake, fake, 9, 1, 8, f(1.0), f(0.9), null, null, None) == code("MPV_ERR_BAD_DTYPE")
    assert nm(fake, fake, 0, 1, 8, f(0.0), f(0.9), null, null, None) == code("MPV_ERR_BAD_TEMPERATURE")
    for bad in (0.0, -1.0, 1.0001, float("nan"), float("inf")):
        assert nm(fake, fake, 0, 1, 8, f(1.0), f(bad), null, null, None) == code("MPV_ERR_BAD_TOP_P")
    assert nm(null, fake, 0, 1, 8, f(1.0), f(0.9), null, null, None) == code("MPV_ERR_NULL")
    assert nm(fake, null, 0, 1, 8, f(1.0), f(0.9), null, null, None) == code("MPV_ERR_NULL")
    assert nm(ctypes.c_void_p(4100), fake, 0, 1, 8, f(1.0), f(0.9), null, null, None) == code("MPV_ERR_ALIGNMENT")
    assert nm(null, null, 0, 0, 8, f(1.0), f(0.9), null, null, None) == 0          # no rows: nothing to do


def test_static_scratch_entry_point_refuses_what_does_not_fit(lib):
    # validation and the size limit come before anything touches a device
    B, N = 4096, 33
    prob = problem(B=B, N=N, V=64, max_depth=N, parent=[-1] + list(range(N - 1)))
    rc, need = ws_bytes(lib, prob)
    limit = eval(re.search(r"#define MPV_STATIC_WORKSPACE_BYTES\s+\(([^)]+)\)", header_text()).group(1).replace("u", ""))
    assert limit == 4 << 20
    assert rc == 0 and need > limit
    bufs = binding._Buffers(*([ctypes.c_void_p(256)] * 9), *([ctypes.c_void_p(0)] * 5))
    assert lib.mpv_verify_static(ctypes.byref(prob), ctypes.byref(bufs), ctypes.c_void_p(0)) == code("MPV_ERR_WORKSPACE")
    assert lib.mpv_verify_static(ctypes.byref(problem(T=0.0)), ctypes.byref(bufs), ctypes.c_void_p(0)) == code("MPV_ERR_BAD_TEMPERATURE")


# ---------------------------------------------------------------- trees of distinct contexts (host logic)

def test_merge_duplicates_agrees_with_the_oracle():
    """mpv_merge_duplicates is host code: it is compared here, bit for bit, with the oracle's
    construction of Def. 3.1 on layouts and tokens where shared prefixes are frequent."""
    from oracle import merged_tree_oracle as merged
    rng = np.random.default_rng(31)
    layouts = [mpv.root_tree(2, 3), mpv.root_tree(8, 5), mpv.delayed_tree(4, 2, 3), mpv.delayed_tree(8, 3, 3),
               [-1, 0, 0, 1, 1, 2, 5, 5, 0, 8, 9], [-1] + list(range(63))]
    for _ in range(6):
        n = int(rng.integers(2, 40))
        layouts.append([-1] + [int(rng.integers(0, k)) for k in range(1, n)])
    some_merge = 0
    for parent in layouts:
        for V in (1, 2, 3, 50):
            tokens = rng.integers(0, V, size=(9, len(parent))).astype(np.int32)
            got_p, got_c = mpv.mpv_merge_duplicates(parent, tokens)
            want_p, want_c = merged.merge_batch(parent, tokens)
            assert got_p.dtype == np.int32 and np.array_equal(got_p, want_p) and np.array_equal(got_c, want_c)
            some_merge += int(np.any(got_c != np.arange(len(parent))))
    assert some_merge > 20


def test_merge_duplicates_validates(lib):
    par = np.array([-1, 0, 1], dtype=np.int32)
    tok = np.zeros((2, 3), dtype=np.int32)
    out = np.zeros((2, 3), dtype=np.int32)
    f = lib.mpv_merge_duplicates
    assert f(par.ctypes.data, tok.ctypes.data, 2, 3, out.ctypes.data, None) == 0
    assert out.tolist() == [[-1, 0, 1], [-1, 0, 1]]
    assert f(None, tok.ctypes.data, 2, 3, out.ctypes.data, None) == code("MPV_ERR_NULL")
    assert f(par.ctypes.data, None, 2, 3, out.ctypes.data, None) == code("MPV_ERR_NULL")
    assert f(par.ctypes.data, tok.ctypes.data, 2, 3, None, None) == code("MPV_ERR_NULL")
    assert f(par.ctypes.data, None, 0, 3, out.ctypes.data, None) == 0
    assert f(par.ctypes.data, tok.ctypes.data, -1, 3, out.ctypes.data, None) == code("MPV_ERR_BAD_SHAPE")
    assert f(par.ctypes.data, tok.ctypes.data, 2, 0, out.ctypes.data, None) == code("MPV_ERR_BAD_SHAPE")
    assert f(par.ctypes.data, tok.ctypes.data, 2, header_constant("MPV_MAX_NODES") + 1, out.ctypes.data, None) \
        == code("MPV_ERR_UNSUPPORTED")
    bad = np.array([-1, 1, 0], dtype=np.int32)
    assert f(bad.ctypes.data, tok.ctypes.data, 2, 3, out.ctypes.data, None) == code("MPV_ERR_BAD_TREE")
    with pytest.raises(ValueError):
        mpv.mpv_merge_duplicates([-1, 0], tok)


def test_verify_merged_rejects_bad_arguments_before_any_launch(lib):
    f = lib.mpv_verify_merged
    bufs = binding._Buffers()
    for name, _ in binding._Buffers._fields_[:9]:
        setattr(bufs, name, 4096)
    fake = ctypes.c_void_p(4096)
    prob = problem(parent=None)                       # problem->parent is not read
    rows = np.array([[-1, 0, 1], [-1, 0, 0]], dtype=np.int32)
    ok = rows.ctypes.data
    assert f(None, ok, None, ctypes.byref(bufs), fake, 1 << 20, None) == code("MPV_ERR_NULL")
    assert f(ctypes.byref(prob), ok, None, None, fake, 1 << 20, None) == code("MPV_ERR_NULL")
    assert f(ctypes.byref(prob), None, None, ctypes.byref(bufs), fake, 1 << 20, None) == code("MPV_ERR_NULL")
    # SpecTr needs the context nodes on the device
    assert f(ctypes.byref(problem(parent=None, method=4)), ok, None, ctypes.byref(bufs), fake, 1 << 20, None) \
        == code("MPV_ERR_NULL")
    assert f(ctypes.byref(problem(parent=None, T=0.0)), ok, None, ctypes.byref(bufs), fake, 1 << 20, None) \
        == code("MPV_ERR_BAD_TEMPERATURE")
    # the second tree's array is invalid / deeper than max_depth / has too many children
    bad = np.array([[-1, 0, 1], [-1, 1, 0]], dtype=np.int32)
    assert f(ctypes.byref(prob), bad.ctypes.data, None, ctypes.byref(bufs), fake, 1 << 20, None) == code("MPV_ERR_BAD_TREE")
    assert f(ctypes.byref(problem(parent=None, max_depth=1)), ok, None, ctypes.byref(bufs), fake, 1 << 20, None) \
        == code("MPV_ERR_BAD_SHAPE")
    n = header_constant("MPV_MAX_CHILDREN") + 2
    star = np.array([[-1] + [0] * (n - 1)], dtype=np.int32)
    assert f(ctypes.byref(problem(B=1, N=n, parent=None)), star.ctypes.data, None, ctypes.byref(bufs), fake, 1 << 20, None) \
        == code("MPV_ERR_UNSUPPORTED")
    # workspace, alignment, null members: as for mpv_verify
    assert f(ctypes.byref(prob), ok, None, ctypes.byref(bufs), None, 1 << 20, None) == code("MPV_ERR_WORKSPACE")
    assert f(ctypes.byref(prob), ok, None, ctypes.byref(bufs), fake, 16, None) == code("MPV_ERR_WORKSPACE")
    bufs.draft_logits = 4096 + 2
    assert f(ctypes.byref(prob), ok, None, ctypes.byref(bufs), fake, 1 << 20, None) == code("MPV_ERR_ALIGNMENT")
    bufs.draft_logits = 4096
    bufs.bonus_token = None
    assert f(ctypes.byref(prob), ok, None, ctypes.byref(bufs), fake, 1 << 20, None) == code("MPV_ERR_NULL")
    assert f(ctypes.byref(problem(B=0, parent=None)), None, None, ctypes.byref(binding._Buffers()), None, 0, None) == 0


def test_block_efficiency_merged_rejects_bad_arguments_before_any_launch(lib):
    f = lib.mpv_block_efficiency_merged
    fake = ctypes.c_void_p(4096)
    null = ctypes.c_void_p(0)
    prob = problem(parent=None)
    rows = np.array([[-1, 0, 1], [-1, 0, 0]], dtype=np.int32)
    ok = rows.ctypes.data
    assert f(None, ok, None, fake, fake, fake, fake, 1 << 20, fake, fake, fake, None) == code("MPV_ERR_NULL")
    assert f(ctypes.byref(prob), None, None, fake, fake, fake, fake, 1 << 20, fake, fake, fake, None) == code("MPV_ERR_NULL")
    # SpecTr needs the context nodes on the device
    assert f(ctypes.byref(problem(parent=None, method=4)), ok, None, fake, fake, fake, fake, 1 << 20, fake, fake, fake, None) \
        == code("MPV_ERR_NULL")
    bad = np.array([[-1, 0, 1], [-1, 0, 2]], dtype=np.int32)
    assert f(ctypes.byref(prob), bad.ctypes.data, None, fake, fake, fake, fake, 1 << 20, fake, fake, fake, None) == code("MPV_ERR_BAD_TREE")
    assert f(ctypes.byref(prob), ok, None, fake, fake, fake, fake, 16, fake, fake, fake, None) == code("MPV_ERR_WORKSPACE")
    assert f(ctypes.byref(prob), ok, None, null, fake, fake, fake, 1 << 20, fake, fake, fake, None) == code("MPV_ERR_NULL")
    assert f(ctypes.byref(prob), ok, None, fake, fake, fake, fake, 1 << 20, fake, null, fake, None) == code("MPV_ERR_NULL")
    assert f(ctypes.byref(prob), ok, None, ctypes.c_void_p(4100), fake, fake, fake, 1 << 20, fake, fake, fake, None) == code("MPV_ERR_ALIGNMENT")
    assert f(ctypes.byref(problem(B=0, parent=None)), None, None, null, null, null, null, 0, null, null, null, None) == 0


def test_bench_runs_on_one_gpu_only():
    """More than one GPU is refused with a message, before anything touches a GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)


def test_acceptance_rates_merged_rejects_bad_arguments_before_any_launch(lib):
    f = lib.mpv_acceptance_rates_merged
    fake = ctypes.c_void_p(4096)
    null = ctypes.c_void_p(0)
    prob = problem(parent=None)
    rows = np.array([[-1, 0, 1], [-1, 0, 0]], dtype=np.int32)
    ok = rows.ctypes.data
    assert f(None, ok, fake, fake, fake, 1 << 20, fake, fake, None) == code("MPV_ERR_NULL")
    assert f(ctypes.byref(prob), None, fake, fake, fake, 1 << 20, fake, fake, None) == code("MPV_ERR_NULL")
    assert f(ctypes.byref(problem(parent=None, method=1)), ok, fake, fake, fake, 1 << 20, fake, fake, None) == code("MPV_ERR_UNSUPPORTED")
    bad = np.array([[-1, 0, 1], [-1, 0, 2]], dtype=np.int32)
    assert f(ctypes.byref(prob), bad.ctypes.data, fake, fake, fake, 1 << 20, fake, fake, None) == code("MPV_ERR_BAD_TREE")
    assert f(ctypes.byref(prob), ok, fake, fake, fake, 16, fake, fake, None) == code("MPV_ERR_WORKSPACE")
    assert f(ctypes.byref(prob), ok, fake, null, fake, 1 << 20, fake, fake, None) == code("MPV_ERR_NULL")
    assert f(ctypes.byref(prob), ok, fake, fake, fake, 1 << 20, null, fake, None) == code("MPV_ERR_NULL")
    assert f(ctypes.byref(prob), ok, ctypes.c_void_p(4100), fake, fake, 1 << 20, fake, fake, None) == code("MPV_ERR_ALIGNMENT")
    assert f(ctypes.byref(problem(B=0, parent=None)), None, null, null, null, 0, null, null, None) == 0


def test_binding_prototypes_have_the_header_s_argument_counts(lib):
    """Every function the binding declares takes as many arguments as include/mpv.h says."""
    text = re.sub(r"/\*.*?\*/", "", header_text(), flags=re.S)
    protos = dict(re.findall(r"\b(mpv_[a-z_]+)\s*\(([^;{]*?)\)\s*;", text, flags=re.S))
    assert len(protos) >= 15
    checked = 0
    for name, params in protos.items():
        fn = getattr(lib, name)
        if fn.argtypes is None:
            continue
        params = params.strip()
        want = 0 if params in ("", "void") else params.count(",") + 1
        assert len(fn.argtypes) == want, f"{name}: binding declares {len(fn.argtypes)} arguments, header {want}"
        checked += 1
    assert checked >= 15
