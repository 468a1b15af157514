"""ctypes binding of libdfa.so: same names as the C ABI in include/dfa.h.

Argument marshalling only.  Tensors are torch tensors on the GPU (torch is used for
device memory and streams); data pointers, element strides and the current HIP stream are
passed to the library, which runs every step of the path in its own kernels.  There is no
fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os

from .build import LIB_PATH

DFA_BF16, DFA_F32 = 0, 1
DFA_MAX_BRANCHES = 8
DFA_ERR_WORKSPACE = -8

# include/dfa.h (the operator) and include/dfa_bench.h (measurement aids)
EXPORTS = [
    "dfa_version", "dfa_error_string", "dfa_index_map", "dfa_index_map_device", "dfa_workspace_bytes", "dfa_forward",
    "dfa_forward_static",
    "dfa_forward_branch", "dfa_merge", "dfa_gather", "dfa_scatter", "dfa_plan_describe", "dfa_plan_describe_forward",
    "dfa_release_plans", "dfa_linear", "dfa_encoder_stack", "dfa_backward",
]
BENCH_EXPORTS = ["dfa_forward_timed", "dfa_mfma_peak", "dfa_dense_unfused", "dfa_dense_unfused_workspace_bytes"]


class Branch(ctypes.Structure):
    _fields_ = [("w", ctypes.c_int32), ("r", ctypes.c_int32)]


class Strides(ctypes.Structure):
    _fields_ = [("b", ctypes.c_int64), ("n", ctypes.c_int64), ("h", ctypes.c_int64)]


class DfaError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {error_string(code)} (code {code})")


_lib = None
_i32p = ctypes.POINTER(ctypes.c_int32)


def _one_hip_runtime():
    """The stream handles torch hands out are only valid in the HIP runtime torch itself uses:
    refuse to run if loading libdfa.so pulled in a second copy of libamdhip64."""
    try:
        maps = open("/proc/self/maps").read()
    except OSError:
        return
    paths = {ln.split()[-1] for ln in maps.splitlines() if "libamdhip64" in ln}
    if len(paths) > 1:
        raise RuntimeError(f"two HIP runtimes loaded: {sorted(paths)}")


def lib():
    """Loads libdfa.so (after torch, so that both share one HIP runtime)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        import torch  # noqa: F401  (brings in libamdhip64 first)
        L = ctypes.CDLL(LIB_PATH)
        _one_hip_runtime()
        L.dfa_error_string.restype = ctypes.c_char_p
        L.dfa_error_string.argtypes = [ctypes.c_int]
        vp, i32, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float
        L.dfa_index_map.argtypes = [i32, i32, Branch, _i32p, _i32p]
        L.dfa_index_map_device.argtypes = [i32, i32, Branch, _i32p, vp, vp]
        fwd = [vp, vp, vp, Strides, Strides, Strides, i32, i32, i32, i32, ctypes.c_int, f32,
               ctypes.POINTER(Branch), i32, _i32p, vp, vp, vp, ctypes.c_size_t, vp]
        L.dfa_workspace_bytes.argtypes = [i32, i32, i32, i32, ctypes.c_int, ctypes.POINTER(Branch), i32, _i32p]
        L.dfa_forward.argtypes = fwd
        L.dfa_forward_static.argtypes = fwd[:-3] + [vp]
        L.dfa_forward_timed.argtypes = fwd + [i32, ctypes.POINTER(f32)]
        L.dfa_forward_branch.argtypes = [vp, vp, vp, Strides, Strides, Strides, i32, i32, i32, i32,
                                         ctypes.c_int, f32, Branch, _i32p, vp, vp, vp]
        L.dfa_merge.argtypes = [vp, vp, i32, i32, i32, i32, i32, ctypes.c_int, vp, vp, vp]
        L.dfa_gather.argtypes = [vp, Strides, i32, i32, i32, i32, ctypes.c_int, Branch, _i32p, vp, vp]
        L.dfa_scatter.argtypes = [vp, i32, i32, i32, i32, ctypes.c_int, Branch, _i32p, vp, vp]
        L.dfa_plan_describe.argtypes = [i32, i32, i32, ctypes.POINTER(Branch), i32, _i32p,
                                        _i32p, _i32p, _i32p, _i32p, _i32p, _i32p, _i32p, _i32p]
        L.dfa_plan_describe_forward.argtypes = [i32, i32, i32, ctypes.POINTER(Branch), i32, _i32p,
                                                _i32p, _i32p, _i32p, _i32p, _i32p, _i32p, _i32p, _i32p, _i32p]
        i64 = ctypes.c_int64
        L.dfa_linear.argtypes = [vp, vp, vp, i64, i32, i32, i64, i64, i64, vp]
        L.dfa_encoder_stack.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, f32, ctypes.POINTER(Branch), i32,
                                        _i32p, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.dfa_backward.argtypes = [vp, vp, vp, vp, vp, vp, Strides, Strides, Strides, i32, i32, i32, i32, ctypes.c_int,
                                   f32, ctypes.POINTER(Branch), i32, _i32p, vp, vp, vp, vp, vp]
        L.dfa_mfma_peak.argtypes = [i32, ctypes.POINTER(f32), ctypes.POINTER(f32)]
        L.dfa_dense_unfused_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.dfa_dense_unfused.argtypes = [vp, vp, vp, Strides, Strides, Strides, i32, i32, i32, i32, f32, vp, vp, vp,
                                        ctypes.c_size_t, vp]
        for name in EXPORTS + BENCH_EXPORTS:
            if name not in ("dfa_error_string", "dfa_workspace_bytes", "dfa_dense_unfused_workspace_bytes"):
                getattr(L, name).restype = ctypes.c_int
        L.dfa_workspace_bytes.restype = ctypes.c_size_t
        L.dfa_dense_unfused_workspace_bytes.restype = ctypes.c_size_t
        _lib = L
    return _lib


def error_string(code: int) -> str:
    return lib().dfa_error_string(int(code)).decode()


def version() -> int:
    return lib().dfa_version()


def _check(rc, where):
    if rc != 0:
        raise DfaError(rc, where)


def _branches(branches):
    arr = (Branch * len(branches))(*[Branch(int(w), int(r)) for (w, r) in branches])
    return arr, len(branches)


def _i32_array(values):
    """Flattens nested ints into a C int32 array; None -> NULL."""
    if values is None:
        return None
    flat = []
    for row in values:
        if isinstance(row, (list, tuple)) or hasattr(row, "__iter__"):
            flat.extend(int(x) for x in row)
        else:
            flat.append(int(row))
    return (ctypes.c_int32 * len(flat))(*flat)


def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return DFA_BF16
    if t.dtype == torch.float32:
        return DFA_F32
    raise DfaError(-4, "dtype")


def _strides(t):
    """Element strides (b, n, h) of a [B, N, H, D] view whose last dim is contiguous."""
    if t.dim() != 4 or t.stride(3) != 1:
        raise DfaError(-5, "tensor must be [B, N, H, D] with contiguous D")
    return Strides(t.stride(0), t.stride(1), t.stride(2))


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _gpu(t, name):
    if not t.is_cuda:
        raise RuntimeError(f"{name} must live in GPU memory")


def index_map(N, H, w, r, head_offsets=None):
    """Host indexer: list of H lists with the kept token positions of one branch (Eq. 1)."""
    out = (ctypes.c_int32 * (H * (N // max(r, 1))))()
    _check(lib().dfa_index_map(N, H, Branch(w, r), _i32_array(head_offsets), out), "dfa_index_map")
    per = N // r
    return [list(out[h * per:(h + 1) * per]) for h in range(H)]


def index_map_device(N, H, w, r, head_offsets=None):
    """Device indexer: int32 tensor [H, N // r] on the GPU."""
    import torch
    out = torch.empty((H, N // r), dtype=torch.int32, device="cuda")
    _check(lib().dfa_index_map_device(N, H, Branch(w, r), _i32_array(head_offsets),
                                      ctypes.c_void_p(out.data_ptr()), _stream()), "dfa_index_map_device")
    return out


_ws_bytes = {}


def workspace_bytes(B, H, N, D, dtype_code, branches, head_offsets=None):
    """Bytes of workspace dfa_forward uses for this shape on the current device (0 = none)."""
    offs = _i32_array(head_offsets)
    key = (B, H, N, D, dtype_code, tuple(tuple(b) for b in branches), tuple(offs) if offs is not None else None)
    if key not in _ws_bytes:
        br, nb = _branches(branches)
        _ws_bytes[key] = int(lib().dfa_workspace_bytes(B, H, N, D, dtype_code, br, nb, offs))
    return _ws_bytes[key]


def _workspace(workspace, q, branches, head_offsets):
    """(pointer, bytes, keep-alive) of the workspace argument: a uint8 tensor, None (NULL: unsplit launch)
    or "auto" (a fresh tensor of the size the library asks for)."""
    import torch
    if isinstance(workspace, str) and workspace == "auto":
        B, N, H, D = q.shape
        need = workspace_bytes(B, H, N, D, _dtype_code(q), branches, head_offsets)
        workspace = torch.empty((need,), dtype=torch.uint8, device=q.device) if need else None
    if workspace is None:
        return ctypes.c_void_p(None), ctypes.c_size_t(0), None
    _gpu(workspace, "workspace")
    return ctypes.c_void_p(workspace.data_ptr()), ctypes.c_size_t(workspace.numel() * workspace.element_size()), workspace


def _fwd_args(q, k, v, branches, scale, head_offsets, out, lse, workspace):
    for t, nm in ((q, "q"), (k, "k"), (v, "v"), (out, "out")):
        _gpu(t, nm)
    B, N, H, D = q.shape
    br, nb = _branches(branches)
    ws_ptr, ws_bytes, keep = _workspace(workspace, q, branches, head_offsets)
    return [ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(k.data_ptr()), ctypes.c_void_p(v.data_ptr()),
            _strides(q), _strides(k), _strides(v), B, H, N, D, _dtype_code(q), ctypes.c_float(scale),
            br, nb, _i32_array(head_offsets), ctypes.c_void_p(out.data_ptr()),
            ctypes.c_void_p(lse.data_ptr() if lse is not None else None), ws_ptr, ws_bytes, _stream()], keep


def forward(q, k, v, branches, scale, head_offsets=None, out=None, lse=None, want_lse=True, workspace="auto"):
    """Fused dilated attention.  q, k, v [B, N, H, D] (may be strided views) -> (out, lse).
    workspace: uint8 GPU tensor of workspace_bytes(...), None for no workspace, "auto" to allocate one."""
    import torch
    B, N, H, D = q.shape
    if out is None:
        out = torch.empty((B, N, H, D), dtype=q.dtype, device=q.device)
    if lse is None and want_lse:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    args, keep = _fwd_args(q, k, v, branches, scale, head_offsets, out, lse, workspace)
    _check(lib().dfa_forward(*args), "dfa_forward")
    if keep is not None and hasattr(keep, "record_stream"):
        keep.record_stream(torch.cuda.current_stream())     # the launch reads it after this function returns
    return out, lse


def forward_static(q, k, v, branches, scale, head_offsets=None, out=None, lse=None):
    """dfa_forward_static: the forward pass through the library's static scratch array (no device allocation
    inside the library; `out` and `lse` are the caller's)."""
    import torch
    B, N, H, D = q.shape
    if out is None:
        out = torch.empty((B, N, H, D), dtype=q.dtype, device=q.device)
    if lse is None:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    args, _ = _fwd_args(q, k, v, branches, scale, head_offsets, out, lse, None)
    _check(lib().dfa_forward_static(*(args[:-3] + args[-1:])), "dfa_forward_static")
    return out, lse


def forward_timed(q, k, v, branches, scale, iters, head_offsets=None, out=None, lse=None, workspace="auto"):
    """Mean milliseconds per dfa_forward launch over `iters` launches (HIP events on the stream)."""
    import torch
    B, N, H, D = q.shape
    if out is None:
        out = torch.empty((B, N, H, D), dtype=q.dtype, device=q.device)
    if lse is None:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    ms = ctypes.c_float(0.0)
    args, keep = _fwd_args(q, k, v, branches, scale, head_offsets, out, lse, workspace)
    _check(lib().dfa_forward_timed(*(args + [int(iters), ctypes.byref(ms)])), "dfa_forward_timed")
    del keep            # the call synchronises the stream
    return ms.value


def forward_branch(q, k, v, w, r, scale, head_offsets=None, out_b=None, lse_b=None):
    """One unmerged branch: (out_b fp32 [B,N,H,D] zero on rows not kept, lse_b fp32 [B,H,N] -inf there)."""
    import torch
    for t, nm in ((q, "q"), (k, "k"), (v, "v")):
        _gpu(t, nm)
    B, N, H, D = q.shape
    if out_b is None:
        out_b = torch.empty((B, N, H, D), dtype=torch.float32, device=q.device)
    if lse_b is None:
        lse_b = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    _check(lib().dfa_forward_branch(
        ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(k.data_ptr()), ctypes.c_void_p(v.data_ptr()),
        _strides(q), _strides(k), _strides(v), B, H, N, D, _dtype_code(q), ctypes.c_float(scale),
        Branch(w, r), _i32_array(head_offsets), ctypes.c_void_p(out_b.data_ptr()),
        ctypes.c_void_p(lse_b.data_ptr()), _stream()), "dfa_forward_branch")
    return out_b, lse_b


def merge(out_b, lse_b, dtype, out=None, lse=None):
    """LSE merge of stacked branch results: out_b fp32 [nb,B,N,H,D], lse_b fp32 [nb,B,H,N]."""
    import torch
    _gpu(out_b, "out_b")
    _gpu(lse_b, "lse_b")
    nb, B, N, H, D = out_b.shape
    if out is None:
        out = torch.empty((B, N, H, D), dtype=dtype, device=out_b.device)
    if lse is None:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=out_b.device)
    code = DFA_BF16 if dtype == torch.bfloat16 else DFA_F32
    _check(lib().dfa_merge(ctypes.c_void_p(out_b.data_ptr()), ctypes.c_void_p(lse_b.data_ptr()), nb, B, H, N, D,
                           code, ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(lse.data_ptr()), _stream()),
           "dfa_merge")
    return out, lse


def gather(x, w, r, head_offsets=None, out=None):
    """Kept rows of x [B, N, H, D] -> dense [B, H, N // r, D] (Eq. 1)."""
    import torch
    _gpu(x, "x")
    B, N, H, D = x.shape
    xg = out if out is not None else torch.empty((B, H, N // r, D), dtype=x.dtype, device=x.device)
    _check(lib().dfa_gather(ctypes.c_void_p(x.data_ptr()), _strides(x), B, H, N, D, _dtype_code(x), Branch(w, r),
                            _i32_array(head_offsets), ctypes.c_void_p(xg.data_ptr()), _stream()), "dfa_gather")
    return xg


def scatter(og, N, w, r, head_offsets=None, out=None):
    """Dense [B, H, N // r, D] back to token positions [B, N, H, D], zero elsewhere (Eq. 3)."""
    import torch
    _gpu(og, "og")
    B, H, _, D = og.shape
    if out is None:
        out = torch.empty((B, N, H, D), dtype=og.dtype, device=og.device)
    _check(lib().dfa_scatter(ctypes.c_void_p(og.data_ptr()), B, H, N, D, _dtype_code(og), Branch(w, r),
                             _i32_array(head_offsets), ctypes.c_void_p(out.data_ptr()), _stream()), "dfa_scatter")
    return out


def linear(x, w, out=None):
    """y = x . w^T (bf16): x [..., K] with contiguous rows, w [N, K]; one weight row per output feature."""
    import torch
    _gpu(x, "x")
    _gpu(w, "w")
    K = x.shape[-1]
    M = x.numel() // K
    Nf = w.shape[0]
    if x.dtype != torch.bfloat16 or w.dtype != torch.bfloat16:
        raise TypeError("linear: bf16 tensors expected")
    if not x.is_contiguous() or w.stride(1) != 1 or w.shape[1] != K:
        raise ValueError("linear: x must be contiguous and w [N, K] with contiguous rows")
    y = out if out is not None else torch.empty(x.shape[:-1] + (Nf,), dtype=torch.bfloat16, device=x.device)
    _check(lib().dfa_linear(ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(w.data_ptr()), ctypes.c_void_p(y.data_ptr()),
                            M, Nf, K, K, w.stride(0), y.stride(-2) if y.dim() > 1 else Nf, _stream()), "dfa_linear")
    return y


def encoder_stack(x, w_qkv, w_o, H, branches, scale, head_offsets=None, buffers=None, workspace="auto"):
    """`layers` attention layers back to back: x [B, N, E] bf16, w_qkv [layers, 3E, E], w_o [layers, E, E].

    Returns (y [B, N, E], qkv of the last layer [B, N, 3, H, D], attention output of the last layer
    [B, N, H, D]).  `buffers` = (qkv, attn, y) tensors to reuse; `workspace` as in forward()."""
    import torch
    for t, nm in ((x, "x"), (w_qkv, "w_qkv"), (w_o, "w_o")):
        _gpu(t, nm)
        if t.dtype != torch.bfloat16 or not t.is_contiguous():
            raise TypeError(f"encoder_stack: {nm} must be a contiguous bf16 tensor")
    B, N, E = x.shape
    layers = w_qkv.shape[0]
    D = E // H
    if tuple(w_qkv.shape) != (layers, 3 * E, E) or tuple(w_o.shape) != (layers, E, E) or H * D != E:
        raise ValueError("encoder_stack: weight shapes do not match x")
    if buffers is None:
        buffers = (torch.empty((B, N, 3, H, D), dtype=torch.bfloat16, device=x.device),
                   torch.empty((B, N, H, D), dtype=torch.bfloat16, device=x.device),
                   torch.empty((B, N, E), dtype=torch.bfloat16, device=x.device))
    qkv, attn, y = buffers
    br, nb = _branches(branches)
    vp = ctypes.c_void_p
    ws_ptr, ws_bytes, keep = _workspace(workspace, qkv[:, :, 0], branches, head_offsets)
    _check(lib().dfa_encoder_stack(vp(x.data_ptr()), vp(w_qkv.data_ptr()), vp(w_o.data_ptr()), layers, B, H, N, D,
                                   ctypes.c_float(scale), br, nb, _i32_array(head_offsets),
                                   vp(qkv.data_ptr()), vp(attn.data_ptr()), vp(y.data_ptr()), ws_ptr, ws_bytes,
                                   _stream()),
           "dfa_encoder_stack")
    if keep is not None:
        keep.record_stream(torch.cuda.current_stream())
    return y, qkv, attn


def backward(q, k, v, out, lse, dout, branches, scale, head_offsets=None):
    """(dq, dk, dv) of dfa_forward for a gradient dout of its output; all [B, N, H, D] of q's dtype."""
    import torch
    for t, nm in ((q, "q"), (k, "k"), (v, "v"), (out, "out"), (lse, "lse"), (dout, "dout")):
        _gpu(t, nm)
    B, N, H, D = q.shape
    if not (out.is_contiguous() and dout.is_contiguous() and lse.is_contiguous()):
        raise ValueError("backward: out, dout and lse must be contiguous")
    if out.dtype != q.dtype or dout.dtype != q.dtype or lse.dtype != torch.float32:
        raise TypeError("backward: out and dout must have q's dtype, lse fp32")
    br, nb = _branches(branches)
    dq, dk, dv = (torch.empty((B, N, H, D), dtype=q.dtype, device=q.device) for _ in range(3))
    delta = torch.empty((2, B, H, N), dtype=torch.float32, device=q.device)
    vp = ctypes.c_void_p
    _check(lib().dfa_backward(vp(q.data_ptr()), vp(k.data_ptr()), vp(v.data_ptr()), vp(out.data_ptr()),
                              vp(lse.data_ptr()), vp(dout.data_ptr()), _strides(q), _strides(k), _strides(v),
                              B, H, N, D, _dtype_code(q), ctypes.c_float(scale), br, nb, _i32_array(head_offsets),
                              vp(delta.data_ptr()), vp(dq.data_ptr()), vp(dk.data_ptr()), vp(dv.data_ptr()), _stream()),
           "dfa_backward")
    return dq, dk, dv


def dense_unfused(q, k, v, scale, out=None, lse=None, workspace=None):
    """Dense attention over all N tokens with the scores materialised in memory (the size sweep's comparison path)."""
    import torch
    for t, nm in ((q, "q"), (k, "k"), (v, "v")):
        _gpu(t, nm)
    B, N, H, D = q.shape
    if q.dtype != torch.bfloat16:
        raise DfaError(-4, "dense_unfused takes bf16 tensors")
    if out is None:
        out = torch.empty((B, N, H, D), dtype=q.dtype, device=q.device)
    if lse is None:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    need = int(lib().dfa_dense_unfused_workspace_bytes(B, H, N, D))
    if workspace is None:
        workspace = torch.empty((max(need, 16),), dtype=torch.uint8, device=q.device)
    vp = ctypes.c_void_p
    _check(lib().dfa_dense_unfused(vp(q.data_ptr()), vp(k.data_ptr()), vp(v.data_ptr()), _strides(q), _strides(k), _strides(v),
                                   B, H, N, D, ctypes.c_float(scale), vp(out.data_ptr()), vp(lse.data_ptr()),
                                   vp(workspace.data_ptr()), ctypes.c_size_t(workspace.numel()), _stream()), "dfa_dense_unfused")
    workspace.record_stream(torch.cuda.current_stream())
    return out, lse


def mfma_peak(random_operands=True):
    """(TFLOP/s, shader MHz) of an MFMA-only loop on the whole chip; synchronises."""
    t, m = ctypes.c_float(0.0), ctypes.c_float(0.0)
    _check(lib().dfa_mfma_peak(1 if random_operands else 0, ctypes.byref(t), ctypes.byref(m)), "dfa_mfma_peak")
    return t.value, m.value


def plan_describe(B, H, N, branches, head_offsets=None):
    """Host view of the launch plan: dict of numpy int32 arrays (tiles, rows, segs, items)."""
    import numpy as np
    br, nb = _branches(branches)
    off = _i32_array(head_offsets)
    cnt = [ctypes.c_int32(0) for _ in range(4)]
    refs = [ctypes.byref(c) for c in cnt]
    _check(lib().dfa_plan_describe(B, H, N, br, nb, off, *refs, None, None, None, None), "dfa_plan_describe")
    nt, nr, ns, ni = (c.value for c in cnt)
    tiles = np.zeros((nt, 6), dtype=np.int32)
    rows = np.zeros((nr,), dtype=np.int32)
    segs = np.zeros((max(ns, 1), 4), dtype=np.int32)
    items = np.zeros((ni, 2), dtype=np.int32)
    p = lambda a: a.ctypes.data_as(_i32p)
    _check(lib().dfa_plan_describe(B, H, N, br, nb, off, *refs, p(tiles), p(rows), p(segs), p(items)),
           "dfa_plan_describe")
    return dict(tiles=tiles, rows=rows, segs=segs[:ns], items=items)


def plan_describe_forward(B, H, N, branches, head_offsets=None):
    """Host view of the plan the bf16 forward launches (row groups packed into tiles): as plan_describe, plus
    block_mult [n_segs][8], the multiplicity of each progression for the rows of each 32-row block of its tile."""
    import numpy as np
    br, nb = _branches(branches)
    off = _i32_array(head_offsets)
    cnt = [ctypes.c_int32(0) for _ in range(4)]
    refs = [ctypes.byref(c) for c in cnt]
    _check(lib().dfa_plan_describe_forward(B, H, N, br, nb, off, *refs, None, None, None, None, None),
           "dfa_plan_describe_forward")
    nt, nr, ns, ni = (c.value for c in cnt)
    tiles = np.zeros((nt, 6), dtype=np.int32)
    rows = np.zeros((nr,), dtype=np.int32)
    segs = np.zeros((max(ns, 1), 4), dtype=np.int32)
    block_mult = np.zeros((max(ns, 1), 8), dtype=np.int32)
    items = np.zeros((ni, 2), dtype=np.int32)
    p = lambda a: a.ctypes.data_as(_i32p)
    _check(lib().dfa_plan_describe_forward(B, H, N, br, nb, off, *refs, p(tiles), p(rows), p(segs), p(block_mult), p(items)),
           "dfa_plan_describe_forward")
    return dict(tiles=tiles, rows=rows, segs=segs[:ns], block_mult=block_mult[:ns], items=items)


def release_plans():
    _check(lib().dfa_release_plans(), "dfa_release_plans")
