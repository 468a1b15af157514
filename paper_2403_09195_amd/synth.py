"""Seeded synthetic inputs for the dilated-flash-attention workloads.

Every element is a pure function of (seed, tensor id, linear index): a
counter-based splitmix64 stream feeds a Box-Muller transform in fp64 and the
result is rounded once to the requested storage type.  The module holds no
attention arithmetic; it only makes numbers.  Both the CPU oracle's tests and
the GPU path's tests draw their tensors from here so that they see bit-identical
inputs.

The paper evaluates on natural images pushed through trained weights (section
4.1); neither is available, and the operator's cost depends on shapes only, so
iid N(0,1) tensors with the paper's shapes (1024x1024 image, patch 16 ->
64x64 = 4096 tokens, bfloat16 as in section 4.1) stand in for them.
"""
from __future__ import annotations

import os

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)

TENSOR_Q, TENSOR_K, TENSOR_V, TENSOR_X = 0, 1, 2, 3
BASE_SEED = 20240309


def _mix(z: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on an array of uint64 counters (wrapping arithmetic)."""
    with np.errstate(over="ignore"):
        z = z + _GAMMA
        z = (z ^ (z >> np.uint64(30))) * _C1
        z = (z ^ (z >> np.uint64(27))) * _C2
        return z ^ (z >> np.uint64(31))


def _stream_key(seed: int, tensor_id: int) -> np.uint64:
    a = _mix(np.array([seed & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64))
    b = _mix(np.array([(tensor_id * 0x1000003) & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64) ^ a)
    return b[0]


def _normal_chunk(key, first, count, out):
    idx = np.arange(first, first + count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        c = key + idx * np.uint64(2)
    b1 = _mix(c)
    b2 = _mix(c + np.uint64(1))
    # 53-bit uniforms; u1 in (0,1] so the logarithm is finite
    u1 = ((b1 >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)
    u2 = (b2 >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
    out[:] = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def normal_f64(seed: int, tensor_id: int, count: int, start: int = 0) -> np.ndarray:
    """`count` iid N(0,1) draws in fp64: elements start .. start+count-1 of the stream.

    Chunks are filled by a few threads; the values do not depend on the chunking."""
    key = _stream_key(seed, tensor_id)
    out = np.empty(count, dtype=np.float64)
    chunk = 1 << 20
    spans = [(lo, min(count, lo + chunk)) for lo in range(0, count, chunk)]
    if len(spans) <= 1:
        for lo, hi in spans:
            _normal_chunk(key, start + lo, hi - lo, out[lo:hi])
        return out
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        list(ex.map(lambda s: _normal_chunk(key, start + s[0], s[1] - s[0], out[s[0]:s[1]]), spans))
    return out


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (round to nearest, ties to even); returns the 16-bit patterns."""
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = bits + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to fp64."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def tensor(seed: int, tensor_id: int, shape, dtype: str, std: float = 1.0):
    """One synthetic tensor.

    dtype "bf16": returns (bits uint16 array, fp64 array holding exactly the
    bf16 values).  dtype "f32": returns (float32 array, its exact fp64 widening).
    """
    n = int(np.prod(shape))
    x = normal_f64(seed, tensor_id, n) * std
    if dtype == "bf16":
        bits = f32_to_bf16_bits(x.astype(np.float32)).reshape(shape)
        return bits, bf16_bits_to_f64(bits)
    if dtype == "f32":
        f = x.astype(np.float32).reshape(shape)
        return f, f.astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


def qkv(seed: int, B: int, N: int, H: int, D: int, dtype: str):
    """Q, K, V of layout [B, N, H, D]; returns ((q,k,v) storage arrays, (q,k,v) fp64)."""
    shape = (B, N, H, D)
    st, ex = [], []
    for tid in (TENSOR_Q, TENSOR_K, TENSOR_V):
        s, e = tensor(seed, tid, shape, dtype)
        st.append(s)
        ex.append(e)
    return tuple(st), tuple(ex)


# The workloads of the task definition, as (name -> parameters).  Head offset is
# h mod r unless "offsets" is given.
CONFIGS = {
    "tiny": dict(B=1, H=1, N=256, D=64, dtype="f32", branches=[(64, 2)], seed=BASE_SEED + 1),
    "sam": dict(B=1, H=12, N=4096, D=64, dtype="bf16",
                branches=[(1024, 1), (2048, 2), (4096, 4)], seed=BASE_SEED + 2),
    "throughput": dict(B=16, H=12, N=4096, D=64, dtype="bf16",
                       branches=[(1024, 1), (2048, 2), (4096, 4)], seed=BASE_SEED + 3),
    "stack_layer": dict(B=8, H=12, N=4096, D=64, dtype="bf16",
                        branches=[(1024, 1), (2048, 2), (4096, 4)], seed=BASE_SEED + 4),
    "highres": dict(B=2, H=12, N=16384, D=64, dtype="bf16",
                    branches=[(2048, 1), (4096, 2), (8192, 4), (16384, 8)], seed=BASE_SEED + 5),
}


def useful_flops(B: int, H: int, N: int, D: int, branches) -> int:
    """4*D flops per kept (query, key) pair: N*w/r^2 pairs per branch per (b, h)."""
    pairs = sum(N * w // (r * r) for (w, r) in branches)
    return 4 * D * pairs * B * H
