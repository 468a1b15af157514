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


# ---------------------------------------------------------------------------------------------- lse of the bf16 path
# The workload definition gives no bar for lse; these follow from the arithmetic.  The kernel's denominator is the
# sum of the numerators after their rounding to bf16 (the values the second product uses, added up in fp32 on the
# matrix cores).  Every numerator is off by at most 2^-8 relative (half a unit of an 8-bit significand).
#
# Worst case, any input: the sum is off by at most 2^-8 relative, lse by -ln(1 - 2^-8) = 3.914e-3.  It is reached
# when one badly placed key carries the row, or when all numerators of a row are equal and round the same way.
BF16_LSE = 3.95e-3
#
# Rows whose weight is spread over keys with unrelated scores: the roundings are independent, each with a relative
# standard deviation of at most 2^-8 / sqrt(3) (uniform within half a unit in the last place, i.e. within 2^-8 of a
# value just above a power of two, where the relative error is largest), so the relative error of the sum has standard deviation at most
# 2^-8 / sqrt(3) * sqrt(sum_j (m_j w_j)^2), w_j the softmax weight of key j and m_j the number of branches that pair
# it with the row (a key that several branches keep is one numerator m_j e^s_j, rounded once).  With
# Z = sum_j m_j e^(s_j) = e^lse and Z2 = sum_j m_j e^(2 s_j) = e^lse2, where lse2 is the operator's own lse at twice the
# scale (the oracle gives it), sum_j (m_j w_j)^2 <= max_j m_j * Z2 / Z^2 <= nb * exp(lse2 - 2 lse).  The bar per row is six
# such standard deviations (788 000 rows are compared in the largest test; 6 sigma is exceeded once in 5e8), never
# more than the worst case, plus the rounding of lse itself to fp32 and of the logarithm (4e-6 * max(1, |lse|)).
BF16_LSE_SIGMAS = 6.0


def bf16_lse_bar(l_ref, l_ref2, nb):
    """Per-row bar for |lse - l_ref| of the bf16 path on inputs with unrelated scores (see above).
    l_ref, l_ref2: the oracle's lse at the call's scale and at twice that scale; nb: number of branches."""
    with np.errstate(invalid="ignore", over="ignore"):
        spread = np.sqrt(nb * np.exp(l_ref2 - 2.0 * l_ref))          # >= sqrt(sum_j (m_j w_j)^2); nan where lse = -inf
    spread = np.where(np.isfinite(spread), np.minimum(spread, 1.0), 1.0)
    bar = BF16_LSE_SIGMAS * 2.0 ** -8 / np.sqrt(3.0) * spread
    return np.minimum(bar, BF16_LSE) + 4e-6 * np.maximum(1.0, np.abs(np.where(np.isfinite(l_ref), l_ref, 0.0)))


def check_lse(got, ref, atol, rtol=0.0):
    """-inf must match exactly; finite values within atol + rtol*|ref| (atol a number or an array of ref's shape)."""
    inf_ref = np.isneginf(ref)
    assert np.array_equal(np.isneginf(got), inf_ref)
    fin = ~inf_ref
    assert np.all(np.isfinite(got[fin]))
    err = np.abs(got[fin] - ref[fin])
    bar = (np.broadcast_to(atol, ref.shape)[fin] if np.ndim(atol) else atol) + rtol * np.abs(ref[fin])
    assert np.all(err <= bar), (float(err.max()), float(np.max(err / bar)))
    return float(err.max()) if fin.any() else 0.0


def check_lse_bf16(got, oracle, ex, branches, scale, l_ref, head_offsets=None):
    """lse of the bf16 path against the per-row bar (inputs with unrelated scores: random data).  Returns the largest
    error and the largest error as a fraction of its row's bar."""
    _, l_ref2 = oracle.forward(*ex, branches, 2.0 * scale, head_offsets=head_offsets)
    bar = bf16_lse_bar(l_ref, l_ref2, len(branches))
    mx = check_lse(got, l_ref, atol=bar)
    fin = np.isfinite(l_ref)
    frac = float(np.max(np.abs(got[fin] - l_ref[fin]) / bar[fin])) if fin.any() else 0.0
    return mx, frac
