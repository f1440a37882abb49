"""ctypes binding of libmpv.so: argument marshalling only.

Function names and argument order follow include/mpv.h.  torch is used for
device memory (tensor.data_ptr()) and for the current HIP stream; every step of
the computation runs in the library's kernels.  There is no CPU fallback: if the
library is missing, loading raises.
"""

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

MPV_METHOD_SPECINFER = 0
MPV_METHOD_TRAVERSAL = 1
MPV_METHOD_NSS = 2
MPV_METHOD_NAIVE = 3
MPV_METHOD_SPECTR = 4
# indices into the counters array of a call
MPV_COUNTER_NEAR_TIE_ACCEPT = 0
MPV_COUNTER_NEAR_TIE_BONUS = 1
MPV_COUNTER_ZERO_MASS = 2
MPV_COUNTER_BAD_TOKEN = 3
MPV_COUNTER_DEPENDENCY_TIMEOUT = 4
MPV_COUNTER_NODE_TASKS_RUN = 5
MPV_COUNTER_NODE_TASKS_CANCELLED = 6
MPV_COUNTER_NODE_TASKS_RESUMED = 7
MPV_DTYPE_F32 = 0
MPV_DTYPE_BF16 = 1

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))


def lib_path():
    return os.path.join(_PKG_DIR, "libmpv.so")


class MpvError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        extra = f", hipError {mpv_last_hip_error()}" if code == -9 else ""
        super().__init__(f"{where}: {mpv_strerror(code)} (code {code}{extra})")


class _Problem(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("N", ctypes.c_int32), ("V", ctypes.c_int32),
        ("method", ctypes.c_int32), ("logit_dtype", ctypes.c_int32),
        ("temperature", ctypes.c_float), ("max_depth", ctypes.c_int32),
        ("parent", ctypes.POINTER(ctypes.c_int32)),
    ]


class _Buffers(ctypes.Structure):
    _fields_ = [(name, ctypes.c_void_p) for name in (
        "target_logits", "draft_logits", "tokens", "uniforms",
        "accept_len", "path_nodes", "path_tokens", "bonus_token", "counters",
        "stats", "edge_probs", "accept_prob", "final_residual", "draw_uniforms")]


_lib = None


def load_library(path=None):
    """Load libmpv.so (built by paper_2602_16994_amd.build) and declare prototypes."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    # torch ships its own HIP runtime; import it first so that libmpv.so binds to
    # the same runtime instance (device memory and streams come from torch).
    import torch  # noqa: F401
    path = path or lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} not found: build it with `python -m paper_2602_16994_amd.build` "
            "(there is no fallback implementation)")
    lib = ctypes.CDLL(path)
    lib.mpv_version.restype = ctypes.c_int
    lib.mpv_version.argtypes = []
    lib.mpv_strerror.restype = ctypes.c_char_p
    lib.mpv_strerror.argtypes = [ctypes.c_int]
    lib.mpv_last_hip_error.restype = ctypes.c_int
    lib.mpv_last_hip_error.argtypes = []
    lib.mpv_workspace_bytes.restype = ctypes.c_int
    lib.mpv_workspace_bytes.argtypes = [ctypes.POINTER(_Problem), ctypes.POINTER(ctypes.c_size_t)]
    lib.mpv_verify.restype = ctypes.c_int
    lib.mpv_verify.argtypes = [ctypes.POINTER(_Problem), ctypes.POINTER(_Buffers),
                               ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.mpv_verify_static.restype = ctypes.c_int
    lib.mpv_verify_static.argtypes = [ctypes.POINTER(_Problem), ctypes.POINTER(_Buffers), ctypes.c_void_p]
    lib.mpv_merge_duplicates.restype = ctypes.c_int
    lib.mpv_merge_duplicates.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                         ctypes.c_void_p, ctypes.c_void_p]
    lib.mpv_verify_merged.restype = ctypes.c_int
    lib.mpv_verify_merged.argtypes = [ctypes.POINTER(_Problem), ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(_Buffers),
                                      ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.mpv_block_efficiency.restype = ctypes.c_int
    lib.mpv_block_efficiency.argtypes = [ctypes.POINTER(_Problem), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_void_p]
    lib.mpv_block_efficiency_merged.restype = ctypes.c_int
    lib.mpv_block_efficiency_merged.argtypes = [ctypes.POINTER(_Problem), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                                ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                                ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    lib.mpv_acceptance_rates.restype = ctypes.c_int
    lib.mpv_acceptance_rates.argtypes = [ctypes.POINTER(_Problem), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    lib.mpv_acceptance_rates_merged.restype = ctypes.c_int
    lib.mpv_acceptance_rates_merged.argtypes = [ctypes.POINTER(_Problem), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                                ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p,
                                                ctypes.c_void_p]
    lib.mpv_nucleus_mask.restype = ctypes.c_int
    lib.mpv_nucleus_mask.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32,
                                     ctypes.c_float, ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    lib.mpv_row_stats.restype = ctypes.c_int
    lib.mpv_row_stats.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32,
                                  ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p]
    lib.mpv_fill_uniforms.restype = ctypes.c_int
    lib.mpv_fill_uniforms.argtypes = [ctypes.c_uint64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
    lib.mpv_timing_enable.restype = ctypes.c_int
    lib.mpv_timing_enable.argtypes = [ctypes.c_int32]
    lib.mpv_timing_read.restype = ctypes.c_int
    lib.mpv_timing_read.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int32),
                                    ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]
    _lib = lib
    return lib


def mpv_version():
    return load_library().mpv_version()


def mpv_strerror(code):
    return load_library().mpv_strerror(int(code)).decode()


def mpv_last_hip_error():
    return load_library().mpv_last_hip_error()


def _make_problem(B, N, V, method, logit_dtype, temperature, max_depth, parent):
    arr = (ctypes.c_int32 * len(parent))(*[int(x) for x in parent]) if parent is not None else None
    prob = _Problem(int(B), int(N), int(V), int(method), int(logit_dtype), float(temperature),
                    int(max_depth), arr)
    prob._keepalive = arr
    return prob


def mpv_workspace_bytes(B, N, V, method, logit_dtype, temperature, max_depth, parent):
    prob = _make_problem(B, N, V, method, logit_dtype, temperature, max_depth, parent)
    out = ctypes.c_size_t(0)
    rc = load_library().mpv_workspace_bytes(ctypes.byref(prob), ctypes.byref(out))
    if rc != 0:
        raise MpvError(rc, "mpv_workspace_bytes")
    return out.value


def _stream_ptr(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dtype_id(t):
    import torch
    if t.dtype == torch.float32:
        return MPV_DTYPE_F32
    if t.dtype == torch.bfloat16:
        return MPV_DTYPE_BF16
    raise TypeError(f"logits must be float32 or bfloat16, got {t.dtype}")


class MpvTimeout(RuntimeError):
    """A wait inside the kernels ran into its time limit: the outputs of that call are invalid."""


def _raise_on_timeout(counters, where):
    """Reads the call's counters (this synchronises with the stream the call ran on) and raises
    if the library reported a dependency timeout."""
    n = int(counters[MPV_COUNTER_DEPENDENCY_TIMEOUT].item())
    if n:
        raise MpvTimeout(f"{where}: {n} waits inside the kernels timed out; the outputs are invalid")


@dataclass
class VerifyResult:
    accept_len: "object"
    path_nodes: "object"
    path_tokens: "object"
    bonus_token: "object"
    counters: "object"
    stats: Optional["object"] = None
    edge_probs: Optional["object"] = None
    accept_prob: Optional["object"] = None
    final_residual: Optional["object"] = None
    workspace: Optional["object"] = None

    def raise_on_timeout(self):
        """Synchronises and raises MpvTimeout if the call gave up on a wait (counters[4] != 0)."""
        _raise_on_timeout(self.counters, "mpv_verify")


def mpv_merge_duplicates(parent, tokens):
    """Host call (see include/mpv.h): parent list of N ints, tokens an int32 array [B,N] on the host
    (numpy, or a CPU torch tensor).  Returns (merged_parent, context_node), numpy int32 [B,N]."""
    import numpy as np
    tok = np.ascontiguousarray(np.asarray(tokens), dtype=np.int32)
    if tok.ndim != 2 or tok.shape[1] != len(parent):
        raise ValueError("tokens must be [B,N] with N = len(parent)")
    B, N = tok.shape
    par = np.ascontiguousarray(np.asarray(parent, dtype=np.int32))
    merged = np.empty((B, N), dtype=np.int32)
    context = np.empty((B, N), dtype=np.int32)
    rc = load_library().mpv_merge_duplicates(par.ctypes.data, tok.ctypes.data, B, N,
                                             merged.ctypes.data, context.ctypes.data)
    if rc != 0:
        raise MpvError(rc, "mpv_merge_duplicates")
    return merged, context


def mpv_verify(parent, tokens, target_logits, draft_logits, temperature, uniforms, method,
               max_depth=None, debug=False, out=None, workspace=None, stream=None, draw_uniforms=None,
               static_scratch=False, merged_parent=None, context_node=None):
    """Enqueue one batched verification on the current (or given) torch stream.

    parent: list of N ints (host).  tokens int32 [B,N], target_logits / draft_logits
    [B,N,V] float32 or bfloat16, uniforms float32 [B,N]: CUDA tensors, contiguous.
    Returns a VerifyResult of CUDA tensors (asynchronous; synchronise before reading
    on the host).  `out` may be a previous VerifyResult whose buffers are reused.
    draw_uniforms float32 [B,N] is needed by MPV_METHOD_NSS, MPV_METHOD_NAIVE and MPV_METHOD_SPECTR (the draw at
    each visited node); with those methods debug=True provides accept_prob and final_residual only.
    static_scratch=True calls mpv_verify_static: no workspace tensor, the library's own device array.
    merged_parent (numpy int32 [B,N] on the host, one parent array per tree) calls mpv_verify_merged;
    `parent` then only serves to size the outputs and the workspace.  MPV_METHOD_SPECTR also needs
    context_node: an int32 CUDA tensor [B,N] (what mpv_merge_duplicates returned, copied to the device).
    """
    import torch
    from .trees import tree_depth
    B, N, V = target_logits.shape
    for t, name in ((tokens, "tokens"), (target_logits, "target_logits"),
                    (draft_logits, "draft_logits"), (uniforms, "uniforms")):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous CUDA tensor")
    if tokens.dtype != torch.int32 or uniforms.dtype != torch.float32:
        raise TypeError("tokens must be int32 and uniforms float32")
    if draft_logits.shape != target_logits.shape or draft_logits.dtype != target_logits.dtype:
        raise ValueError("target and draft logits must have the same shape and dtype")
    if tuple(tokens.shape) != (B, N) or tuple(uniforms.shape) != (B, N):
        raise ValueError("tokens and uniforms must be [B,N]")
    if draw_uniforms is not None:
        if (not draw_uniforms.is_cuda or not draw_uniforms.is_contiguous() or draw_uniforms.dtype != torch.float32
                or tuple(draw_uniforms.shape) != (B, N)):
            raise ValueError("draw_uniforms must be a contiguous float32 CUDA tensor [B,N]")
    if max_depth is None:
        max_depth = max(1, tree_depth(list(parent)) if len(parent) == N and N > 0 else 1)
    dev = target_logits.device
    prob = _make_problem(B, N, V, method, _dtype_id(target_logits), temperature, max_depth, parent)
    if out is None:
        i32 = dict(dtype=torch.int32, device=dev)
        out = VerifyResult(
            accept_len=torch.empty(B, **i32),
            path_nodes=torch.empty(B, max_depth, **i32),
            path_tokens=torch.empty(B, max_depth, **i32),
            bonus_token=torch.empty(B, **i32),
            counters=torch.empty(8, dtype=torch.int32, device=dev),
        )
        if debug:
            f32 = dict(dtype=torch.float32, device=dev)
            if method in (MPV_METHOD_SPECINFER, MPV_METHOD_TRAVERSAL):
                out.stats = torch.empty(B, N, 4, **f32)
                out.edge_probs = torch.empty(B, N, 2, **f32)
            out.accept_prob = torch.empty(B, N, **f32)
            out.final_residual = torch.empty(B, V, **f32)
    lib = load_library()

    def ptr(t):
        return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)

    if not static_scratch:
        need = ctypes.c_size_t(0)
        rc = lib.mpv_workspace_bytes(ctypes.byref(prob), ctypes.byref(need))
        if rc != 0:
            raise MpvError(rc, "mpv_workspace_bytes")
        if workspace is None:
            workspace = out.workspace
        if workspace is None or workspace.numel() < need.value:
            workspace = torch.empty(max(need.value, 256), dtype=torch.uint8, device=dev)
        out.workspace = workspace

    bufs = _Buffers(ptr(target_logits), ptr(draft_logits), ptr(tokens), ptr(uniforms),
                    ptr(out.accept_len), ptr(out.path_nodes), ptr(out.path_tokens),
                    ptr(out.bonus_token), ptr(out.counters),
                    ptr(out.stats), ptr(out.edge_probs), ptr(out.accept_prob), ptr(out.final_residual),
                    ptr(draw_uniforms))
    if merged_parent is not None:
        import numpy as np
        rows = np.ascontiguousarray(np.asarray(merged_parent), dtype=np.int32)
        if static_scratch or rows.shape != (B, N):
            raise ValueError("merged_parent must be [B,N] and cannot be combined with static_scratch")
        if context_node is not None and (not context_node.is_cuda or not context_node.is_contiguous()
                                         or context_node.dtype != torch.int32 or tuple(context_node.shape) != (B, N)):
            raise ValueError("context_node must be a contiguous int32 CUDA tensor [B,N]")
        rc = lib.mpv_verify_merged(ctypes.byref(prob), rows.ctypes.data, ptr(context_node), ctypes.byref(bufs),
                                   ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream_ptr(stream))
        if rc != 0:
            raise MpvError(rc, "mpv_verify_merged")
        return out
    if static_scratch:
        rc = lib.mpv_verify_static(ctypes.byref(prob), ctypes.byref(bufs), _stream_ptr(stream))
    else:
        rc = lib.mpv_verify(ctypes.byref(prob), ctypes.byref(bufs), ptr(workspace),
                            ctypes.c_size_t(workspace.numel()), _stream_ptr(stream))
    if rc != 0:
        raise MpvError(rc, "mpv_verify_static" if static_scratch else "mpv_verify")
    return out


@dataclass
class BlockEfficiencyResult:
    expected: "object"          # float32 [B]    E[tau + 1 | tree]
    reach_prob: "object"        # float32 [B,N]  P(node on the accepted path)
    counters: "object"
    workspace: Optional["object"] = None

    def raise_on_timeout(self):
        """Synchronises and raises MpvTimeout if the call gave up on a wait (counters[4] != 0)."""
        _raise_on_timeout(self.counters, "mpv_block_efficiency")


def mpv_block_efficiency(parent, tokens, target_logits, draft_logits, temperature, method,
                         out=None, stream=None, merged_parent=None, context_node=None):
    """Expected block efficiency of every tree of the batch (see include/mpv.h): enqueued on the
    current (or given) torch stream; returns a BlockEfficiencyResult of CUDA tensors.  Arguments as
    for mpv_verify, without uniforms.  `out` may be a previous result whose buffers are reused.
    merged_parent (numpy int32 [B,N] on the host) calls mpv_block_efficiency_merged; MPV_METHOD_SPECTR
    then also needs context_node, an int32 CUDA tensor [B,N]."""
    import torch
    from .trees import tree_depth
    B, N, V = target_logits.shape
    for t, name in ((tokens, "tokens"), (target_logits, "target_logits"), (draft_logits, "draft_logits")):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous CUDA tensor")
    if tokens.dtype != torch.int32 or tuple(tokens.shape) != (B, N):
        raise TypeError("tokens must be int32 [B,N]")
    if draft_logits.shape != target_logits.shape or draft_logits.dtype != target_logits.dtype:
        raise ValueError("target and draft logits must have the same shape and dtype")
    dev = target_logits.device
    max_depth = max(1, tree_depth(list(parent)) if len(parent) == N and N > 0 else 1)
    prob = _make_problem(B, N, V, method, _dtype_id(target_logits), temperature, max_depth, parent)
    lib = load_library()
    need = ctypes.c_size_t(0)
    rc = lib.mpv_workspace_bytes(ctypes.byref(prob), ctypes.byref(need))
    if rc != 0:
        raise MpvError(rc, "mpv_workspace_bytes")
    if out is None:
        out = BlockEfficiencyResult(
            expected=torch.empty(B, dtype=torch.float32, device=dev),
            reach_prob=torch.empty(B, N, dtype=torch.float32, device=dev),
            counters=torch.empty(8, dtype=torch.int32, device=dev))
    if out.workspace is None or out.workspace.numel() < need.value:
        out.workspace = torch.empty(max(need.value, 256), dtype=torch.uint8, device=dev)

    def ptr(t):
        return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)

    if merged_parent is not None:
        import numpy as np
        rows = np.ascontiguousarray(np.asarray(merged_parent), dtype=np.int32)
        if rows.shape != (B, N):
            raise ValueError("merged_parent must be [B,N]")
        if context_node is not None and (not context_node.is_cuda or not context_node.is_contiguous()
                                         or context_node.dtype != torch.int32 or tuple(context_node.shape) != (B, N)):
            raise ValueError("context_node must be a contiguous int32 CUDA tensor [B,N]")
        rc = lib.mpv_block_efficiency_merged(ctypes.byref(prob), rows.ctypes.data, ptr(context_node), ptr(target_logits), ptr(draft_logits),
                                             ptr(tokens), ptr(out.workspace), ctypes.c_size_t(out.workspace.numel()),
                                             ptr(out.reach_prob), ptr(out.expected), ptr(out.counters), _stream_ptr(stream))
        if rc != 0:
            raise MpvError(rc, "mpv_block_efficiency_merged")
        return out
    rc = lib.mpv_block_efficiency(ctypes.byref(prob), ptr(target_logits), ptr(draft_logits), ptr(tokens),
                                  ptr(out.workspace), ctypes.c_size_t(out.workspace.numel()),
                                  ptr(out.reach_prob), ptr(out.expected), ptr(out.counters), _stream_ptr(stream))
    if rc != 0:
        raise MpvError(rc, "mpv_block_efficiency")
    return out


def mpv_acceptance_rates(parent, target_logits, draft_logits, temperature, method, stream=None, merged_parent=None):
    """Acceptance rate of the solver `method` at every internal node (see include/mpv.h): returns
    (alpha float32 [B,N], counters) as CUDA tensors; leaves get 0.  merged_parent (numpy int32 [B,N]
    on the host, one parent array per tree) calls mpv_acceptance_rates_merged."""
    import torch
    from .trees import tree_depth
    B, N, V = target_logits.shape
    for t, name in ((target_logits, "target_logits"), (draft_logits, "draft_logits")):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous CUDA tensor")
    if draft_logits.shape != target_logits.shape or draft_logits.dtype != target_logits.dtype:
        raise ValueError("target and draft logits must have the same shape and dtype")
    dev = target_logits.device
    max_depth = max(1, tree_depth(list(parent)) if len(parent) == N and N > 0 else 1)
    prob = _make_problem(B, N, V, method, _dtype_id(target_logits), temperature, max_depth, parent)
    lib = load_library()
    need = ctypes.c_size_t(0)
    rc = lib.mpv_workspace_bytes(ctypes.byref(prob), ctypes.byref(need))
    if rc != 0:
        raise MpvError(rc, "mpv_workspace_bytes")
    workspace = torch.empty(max(need.value, 256), dtype=torch.uint8, device=dev)
    alpha = torch.empty(B, N, dtype=torch.float32, device=dev)
    counters = torch.empty(8, dtype=torch.int32, device=dev)
    if merged_parent is not None:
        import numpy as np
        rows = np.ascontiguousarray(np.asarray(merged_parent), dtype=np.int32)
        if rows.shape != (B, N):
            raise ValueError("merged_parent must be [B,N]")
        rc = lib.mpv_acceptance_rates_merged(ctypes.byref(prob), rows.ctypes.data, ctypes.c_void_p(target_logits.data_ptr()),
                                             ctypes.c_void_p(draft_logits.data_ptr()), ctypes.c_void_p(workspace.data_ptr()),
                                             ctypes.c_size_t(workspace.numel()), ctypes.c_void_p(alpha.data_ptr()),
                                             ctypes.c_void_p(counters.data_ptr()), _stream_ptr(stream))
        if rc != 0:
            raise MpvError(rc, "mpv_acceptance_rates_merged")
        return alpha, counters
    rc = lib.mpv_acceptance_rates(ctypes.byref(prob), ctypes.c_void_p(target_logits.data_ptr()),
                                  ctypes.c_void_p(draft_logits.data_ptr()), ctypes.c_void_p(workspace.data_ptr()),
                                  ctypes.c_size_t(workspace.numel()), ctypes.c_void_p(alpha.data_ptr()),
                                  ctypes.c_void_p(counters.data_ptr()), _stream_ptr(stream))
    if rc != 0:
        raise MpvError(rc, "mpv_acceptance_rates")
    return alpha, counters


def mpv_nucleus_mask(logits, temperature, top_p, out=None, inplace=False, stream=None):
    """Nucleus (top-p) transform of every row of a CUDA tensor [..., V] (see include/mpv.h): tokens
    outside the nucleus get the logit -inf.  Returns (masked, threshold[...], kept[...]); with
    inplace=True `masked` is `logits` itself."""
    import torch
    if not logits.is_cuda or not logits.is_contiguous() or logits.dim() < 1:
        raise ValueError("logits must be a contiguous CUDA tensor")
    V = logits.shape[-1]
    rows = logits.numel() // V if V else 0
    if inplace:
        out = logits
    elif out is None:
        out = torch.empty_like(logits)
    lead = tuple(logits.shape[:-1])
    thr = torch.empty(lead, dtype=torch.float32, device=logits.device)
    kept = torch.empty(lead, dtype=torch.int32, device=logits.device)
    rc = load_library().mpv_nucleus_mask(ctypes.c_void_p(logits.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                                         _dtype_id(logits), rows, V, float(temperature), float(top_p),
                                         ctypes.c_void_p(thr.data_ptr()), ctypes.c_void_p(kept.data_ptr()),
                                         _stream_ptr(stream))
    if rc != 0:
        raise MpvError(rc, "mpv_nucleus_mask")
    return out, thr, kept


def mpv_row_stats(logits, temperature, out=None, stream=None):
    """(max, ln sum exp((z-max)/T)) of every row of a [rows, V] CUDA tensor."""
    import torch
    if not logits.is_cuda or not logits.is_contiguous() or logits.dim() != 2:
        raise ValueError("logits must be a contiguous 2-D CUDA tensor")
    rows, V = logits.shape
    if out is None:
        out = torch.empty(rows, 2, dtype=torch.float32, device=logits.device)
    rc = load_library().mpv_row_stats(ctypes.c_void_p(logits.data_ptr()), _dtype_id(logits), rows, V,
                                      float(temperature), ctypes.c_void_p(out.data_ptr()), _stream_ptr(stream))
    if rc != 0:
        raise MpvError(rc, "mpv_row_stats")
    return out


def mpv_fill_uniforms(seed, count, out=None, device="cuda", stream=None):
    """count counter-based uniforms in [0,1) from `seed` (see include/mpv.h)."""
    import torch
    if out is None:
        out = torch.empty(count, dtype=torch.float32, device=device)
    rc = load_library().mpv_fill_uniforms(ctypes.c_uint64(seed & (2 ** 64 - 1)), int(count),
                                          ctypes.c_void_p(out.data_ptr()), _stream_ptr(stream))
    if rc != 0:
        raise MpvError(rc, "mpv_fill_uniforms")
    return out


MPV_KERNEL_NAMES = {0: "init", 1: "node_task", 2: "debug_stats"}


def mpv_timing_enable(max_launches):
    """Bracket every kernel of the following mpv_verify calls with HIP events
    (0 turns it off)."""
    rc = load_library().mpv_timing_enable(int(max_launches))
    if rc != 0:
        raise MpvError(rc, "mpv_timing_enable")


def mpv_timing_read(capacity):
    """After synchronising: list of (kernel_id, milliseconds) of the recorded launches."""
    ms = (ctypes.c_float * capacity)()
    ids = (ctypes.c_int32 * capacity)()
    n = ctypes.c_int32(0)
    rc = load_library().mpv_timing_read(ms, ids, capacity, ctypes.byref(n))
    if rc != 0:
        raise MpvError(rc, "mpv_timing_read")
    return [(int(ids[i]), float(ms[i])) for i in range(n.value)]
