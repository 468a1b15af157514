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


def check_lse(got, ref, atol, rtol=0.0):
    """-inf must match exactly; finite values within atol + rtol*|ref|."""
    inf_ref = np.isneginf(ref)
    assert np.array_equal(np.isneginf(got), inf_ref)
    fin = ~inf_ref
    assert np.all(np.isfinite(got[fin]))
    err = np.abs(got[fin] - ref[fin])
    assert np.all(err <= atol + rtol * np.abs(ref[fin])), float(err.max())
    return float(err.max()) if fin.any() else 0.0
