"""Helpers of the GPU parity tests: seeded inputs -> device tensors, results -> fp64 numpy."""
import numpy as np


def to_device(storage):
    """uint16 bf16 bit patterns or float32 array -> torch tensor on the GPU."""
    import torch
    if storage.dtype == np.uint16:
        return torch.from_numpy(storage.view(np.int16).copy()).view(torch.bfloat16).cuda()
    return torch.from_numpy(storage.copy()).cuda()


def to_f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def make_qkv(seed, B, N, H, D, dtype):
    from paper_2403_09195_amd import synth
    st, ex = synth.qkv(seed, B, N, H, D, dtype)
    return tuple(to_device(s) for s in st), ex


def error_stats(got, ref):
    d = np.abs(got - ref)
    return float(d.max()), float(d.mean())


# lse of the bf16 path.  The workload definition gives no bar for it; this one follows from the arithmetic: the
# kernel's denominator is the sum of the numerators after their rounding to bf16 (the values the second
# product uses, added up on the matrix cores), each off by at most 2^-8 relative (half a unit of an 8-bit
# significand), so the sum is off by at most 2^-8 relative and lse by -ln(1 - 2^-8) = 3.914e-3, reached only
# when a single key carries the row and sits badly between two bf16 values; rows whose weight is spread over
# many keys see the roundings average out (3e-4 at the throughput workload).  The rest of the bar covers the
# fp32 rounding of lse itself.
BF16_LSE = 3.95e-3


def check_lse(got, ref, atol, rtol=0.0):
    """-inf must match exactly; finite values within atol + rtol*|ref|."""
    inf_ref = np.isneginf(ref)
    assert np.array_equal(np.isneginf(got), inf_ref)
    fin = ~inf_ref
    assert np.all(np.isfinite(got[fin]))
    err = np.abs(got[fin] - ref[fin])
    assert np.all(err <= atol + rtol * np.abs(ref[fin])), float(err.max())
    return float(err.max()) if fin.any() else 0.0
