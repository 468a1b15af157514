"""ctypes front end of the fp64 C oracle (oracle/dfa_oracle.c).

TEST INFRASTRUCTURE ONLY.  Nothing here is used by the GPU library; the two
share no code.  Arrays are numpy fp64, q/k/v/out in [B, N, H, D], lse in
[B, H, N].  Operation definitions: SAM-Lightening section 3.1, Eq. 1-3; the
per-head start offset and the multi-branch log-sum-exp merge come from the
workload definition (the paper describes a single (w, r) with offset 0).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dfa_oracle.c")
_LIB = os.path.join(_HERE, "libdfa_oracle.so")
_lib = None

_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O3, OpenMP over the independent (b, h) units)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        for name in ("dfa_oracle_index_map", "dfa_oracle_branch", "dfa_oracle_segment_probs",
                     "dfa_oracle_merge", "dfa_oracle_forward", "dfa_oracle_forward_rows",
                     "dfa_oracle_num_threads", "dfa_oracle_backward"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _d(a):
    return a.ctypes.data_as(_dp)


def _i(a):
    return a.ctypes.data_as(_ip) if a is not None else None


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _offsets(head_offsets, nb, H):
    if head_offsets is None:
        return None
    o = np.ascontiguousarray(head_offsets, dtype=np.int32)
    assert o.shape == (nb, H), "head_offsets must be [n_branches, H]"
    return o


def num_threads() -> int:
    return _load().dfa_oracle_num_threads()


def index_map(N, H, w, r, head_offsets=None):
    """Kept token positions of one branch: int32 [H, N // r], segment-major then j (Eq. 1)."""
    off = None if head_offsets is None else np.ascontiguousarray(head_offsets, dtype=np.int32)
    idx = np.empty((H, N // r), dtype=np.int32)
    rc = _load().dfa_oracle_index_map(N, H, w, r, _i(off), _i(idx))
    if rc != 0:
        raise ValueError("dfa_oracle_index_map: bad arguments")
    return idx


def branch(q, k, v, w, r, scale, head_offsets=None):
    """One unmerged branch: (out_b [B,N,H,D] zero on rows not kept, lse_b [B,H,N] -inf there)."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, N, H, D = q.shape
    off = None if head_offsets is None else np.ascontiguousarray(head_offsets, dtype=np.int32)
    out = np.empty((B, N, H, D), dtype=np.float64)
    lse = np.empty((B, H, N), dtype=np.float64)
    rc = _load().dfa_oracle_branch(_d(q), _d(k), _d(v), B, H, N, D, ctypes.c_double(scale),
                                   w, r, _i(off), _d(out), _d(lse))
    if rc != 0:
        raise ValueError("dfa_oracle_branch: bad arguments")
    return out, lse


def segment_probs(q, k, v, w, r, scale, offset, b, h, seg):
    """Softmax matrix [w/r, w/r] of one sparsified segment (Eq. 2 before the product with V)."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, N, H, D = q.shape
    p = np.empty((w // r, w // r), dtype=np.float64)
    rc = _load().dfa_oracle_segment_probs(_d(q), _d(k), _d(v), B, H, N, D, ctypes.c_double(scale),
                                          w, r, offset, b, h, seg, _d(p))
    if rc != 0:
        raise ValueError("dfa_oracle_segment_probs: bad arguments")
    return p


def merge(out_b, lse_b):
    """LSE merge.  out_b [nb, rows, D], lse_b [nb, rows] -> (out [rows, D], lse [rows])."""
    out_b, lse_b = _f64(out_b), _f64(lse_b)
    nb, rows, D = out_b.shape
    assert lse_b.shape == (nb, rows)
    out = np.empty((rows, D), dtype=np.float64)
    lse = np.empty((rows,), dtype=np.float64)
    rc = _load().dfa_oracle_merge(nb, ctypes.c_size_t(rows), D, _d(out_b), _d(lse_b), _d(out), _d(lse))
    if rc != 0:
        raise ValueError("dfa_oracle_merge: bad arguments")
    return out, lse


def forward(q, k, v, branches, scale, head_offsets=None, return_branches=False):
    """Whole operator: (out [B,N,H,D], lse [B,H,N]) and optionally the per-branch results."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, N, H, D = q.shape
    nb = len(branches)
    w = np.array([b[0] for b in branches], dtype=np.int32)
    r = np.array([b[1] for b in branches], dtype=np.int32)
    off = _offsets(head_offsets, nb, H)
    out = np.empty((B, N, H, D), dtype=np.float64)
    lse = np.empty((B, H, N), dtype=np.float64)
    bo = np.empty((nb, B, N, H, D), dtype=np.float64) if return_branches else None
    bl = np.empty((nb, B, H, N), dtype=np.float64) if return_branches else None
    rc = _load().dfa_oracle_forward(_d(q), _d(k), _d(v), B, H, N, D, ctypes.c_double(scale), nb,
                                    _i(w), _i(r), _i(off), _d(out), _d(lse),
                                    _d(bo) if bo is not None else None,
                                    _d(bl) if bl is not None else None)
    if rc != 0:
        raise ValueError("dfa_oracle_forward: bad arguments")
    return (out, lse, bo, bl) if return_branches else (out, lse)


def forward_rows(q, k, v, branches, scale, bhn, head_offsets=None):
    """Operator output for sampled rows only.  bhn int [n, 3] of (b, h, n) -> (out [n, D], lse [n])."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, N, H, D = q.shape
    nb = len(branches)
    w = np.array([b[0] for b in branches], dtype=np.int32)
    r = np.array([b[1] for b in branches], dtype=np.int32)
    off = _offsets(head_offsets, nb, H)
    bhn = np.ascontiguousarray(bhn, dtype=np.int32)
    n = bhn.shape[0]
    out = np.empty((n, D), dtype=np.float64)
    lse = np.empty((n,), dtype=np.float64)
    rc = _load().dfa_oracle_forward_rows(_d(q), _d(k), _d(v), B, H, N, D, ctypes.c_double(scale), nb,
                                         _i(w), _i(r), _i(off), n, _i(bhn), _d(out), _d(lse))
    if rc != 0:
        raise ValueError("dfa_oracle_forward_rows: bad arguments")
    return out, lse


def backward(q, k, v, dout, branches, scale, head_offsets=None):
    """(dq, dk, dv) for a gradient dout of the merged output; all [B, N, H, D] fp64."""
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    B, N, H, D = q.shape
    nb = len(branches)
    w = np.ascontiguousarray([b[0] for b in branches], dtype=np.int32)
    r = np.ascontiguousarray([b[1] for b in branches], dtype=np.int32)
    offs = _offsets(head_offsets, nb, H)
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    rc = _load().dfa_oracle_backward(_d(q), _d(k), _d(v), _d(dout), B, H, N, D, ctypes.c_double(scale), nb,
                                     _i(w), _i(r), _i(offs), _d(dq), _d(dk), _d(dv))
    if rc != 0:
        raise ValueError("dfa_oracle_backward: bad arguments")
    return dq, dk, dv


# ---------------------------------------------------------------------------------------------
# The steps either side of the operator inside one encoder layer (the "encoder attention
# stack" workload: QKV projection 768 -> 2304, dilated attention, output projection 768 -> 768;
# no bias, residual or normalisation).  The paper names these projections only as part of the
# ViT encoder's self-attention blocks (section 3.1); the feature order of the fused QKV
# output is this build's reading: feature f = t*E + h*D + d with t = 0, 1, 2 for q, k, v.

def linear(x, w):
    """y = x . w^T in fp64: x [..., K], w [N, K] (one weight row per output feature) -> [..., N]."""
    x, w = _f64(x), _f64(w)
    assert x.shape[-1] == w.shape[1]
    return np.matmul(x, w.T)


def attention_layer(x, w_qkv, w_o, H, branches, scale, head_offsets=None):
    """One layer of the stack: x [B, N, E] -> (y [B, N, E], qkv [B, N, 3, H, D], attn [B, N, H, D]).

    qkv = x . w_qkv^T split as [3][H][D]; attn = dilated attention of (q, k, v); y = attn . w_o^T.
    """
    x = _f64(x)
    B, N, E = x.shape
    D = E // H
    assert w_qkv.shape == (3 * E, E) and w_o.shape == (E, E) and H * D == E
    qkv = linear(x, w_qkv).reshape(B, N, 3, H, D)
    attn, _ = forward(qkv[:, :, 0], qkv[:, :, 1], qkv[:, :, 2], branches, scale, head_offsets)
    y = linear(attn.reshape(B, N, E), w_o)
    return y, qkv, attn
