"""The bf16 bars for lse used by the GPU parity tests (gpu_util.BF16_LSE, the worst case, and gpu_util.bf16_lse_bar,
the per-row bar for inputs with unrelated scores) are derived from the kernel's arithmetic, not
given by the workload definition.  This file checks the derivation on the CPU, without the oracle and without
the kernels: softmax numerators rounded to bf16 (nearest even) before they are summed move the logarithm of the
sum by at most -ln(1 - 2^-8), the bound is approached by rows that one badly placed key carries, and rows
whose weight is spread over many keys stay far below it."""
import numpy as np

from gpu_util import BF16_LSE, bf16_lse_bar


def _round_bf16(x):
    """fp32 -> bf16 -> fp32, round to nearest even (finite positive inputs)."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32)
    r = ((u.astype(np.uint64) + 0x7FFF + ((u >> 16) & 1)) >> 16 << 16).astype(np.uint32)
    return r.view(np.float32)


def _lse_shift(p):
    """|ln sum(bf16(p)) - ln sum(p)| per row, sums in fp64."""
    exact = p.astype(np.float64).sum(axis=-1)
    rounded = _round_bf16(p).astype(np.float64).sum(axis=-1)
    return np.abs(np.log(rounded) - np.log(exact))


def test_rounding_helper_is_bf16_nearest_even():
    # 1 + 2^-8 lies half way between 1 and 1 + 2^-7: ties go to the even significand (1.0); just above goes up
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 3 * 2.0 ** -8, 0.3], dtype=np.float32)
    got = _round_bf16(x)
    assert got[0] == 1.0 and got[1] == 1.0 and got[2] == np.float32(1.0 + 2.0 ** -7)
    assert got[3] == np.float32(1.0 + 2.0 ** -6)          # tie between 1 + 2^-7 (odd) and 1 + 2^-6 (even)
    assert abs(got[4] - 0.3) <= 0.3 * 2.0 ** -8 and (got.view(np.uint32) & 0xFFFF == 0).all()


def test_bound_holds_and_is_nearly_reached():
    rng = np.random.default_rng(5)
    bound = -np.log1p(-2.0 ** -8)
    assert bound < BF16_LSE < 1.02 * bound
    # numerators as the kernel holds them: 2^x with x anywhere below the rebase threshold of 2^8
    for nkeys in (1, 2, 3, 8, 64, 1024):
        p = np.exp2(rng.uniform(-30.0, 8.0, size=(20000, nkeys))).astype(np.float32)
        assert _lse_shift(p).max() <= bound
    # worst case: one key, its numerator just above a power of two and just below the rounding tie
    p = np.array([[np.float32(1.0 + 2.0 ** -8 - 2.0 ** -20)], [np.float32(2.0 ** 5 * (1.0 + 2.0 ** -8 - 2.0 ** -20))]])
    worst = _lse_shift(p)
    assert np.all(worst > 0.99 * 2.0 ** -8) and np.all(worst <= bound)


def test_spread_rows_stay_far_below_the_bound():
    rng = np.random.default_rng(6)
    # scores of the workloads: N(0, 1) scaled logits, 1024 to 3072 keys per row
    for nkeys in (1024, 3072):
        s = rng.standard_normal((2000, nkeys))
        p = np.exp2((s - 4.0) * np.log2(np.e)).astype(np.float32)
        assert _lse_shift(p).max() <= 5e-4


def test_per_row_bar_covers_independent_roundings_and_is_not_slack():
    """Rows of n keys with N(0, sigma^2) scaled scores, numerators rounded to bf16 before the sum: the shift of lse
    stays below the per-row bar (six standard deviations of the summed roundings, capped by the worst case) on every
    row, and the largest shift seen is a good part of the bar - the bar is not a loose one."""
    rng = np.random.default_rng(7)
    worst_frac = {}
    for nkeys in (1, 2, 5, 32, 256, 1024, 3072):
        for sigma in (0.5, 1.0, 1.5, 8.0):
            s = sigma * rng.standard_normal((4000, nkeys))
            # numerators as the kernel holds them: against a reference exponent somewhere below the row maximum
            ref = s.max(axis=-1, keepdims=True) - rng.uniform(0.0, 5.0, size=(4000, 1))
            p = np.exp(s - ref).astype(np.float32)
            lse = np.log(np.exp(s - ref).sum(axis=-1)) + ref[:, 0]
            lse2 = np.log(np.exp(2.0 * (s - ref)).sum(axis=-1)) + 2.0 * ref[:, 0]
            bar = bf16_lse_bar(lse, lse2, 1) - 4e-6 * np.maximum(1.0, np.abs(lse))      # the rounding part alone
            shift = _lse_shift(p)
            assert np.all(shift <= bar), (nkeys, sigma, float((shift / bar).max()))
            worst_frac[(nkeys, sigma)] = float((shift / bar).max())
    # 4000 rows reach about 3.5 standard deviations, and a rounding is on average smaller than the bound on it
    assert 0.25 <= worst_frac[(1024, 1.0)] <= 0.7 and 0.25 <= worst_frac[(3072, 1.5)] <= 0.7
    # the throughput workload's rows (1024 to 3072 keys, sigma about 1, three branches): bars around 1e-3 where the
    # worst case is 3.9e-3
    s = rng.standard_normal((16, 1024))
    bar = bf16_lse_bar(np.log(np.exp(s).sum(-1)), np.log(np.exp(2 * s).sum(-1)), 3)
    assert 5e-4 <= bar.min() and bar.max() <= 2e-3


def test_per_row_bar_does_not_cover_equal_numerators():
    """What the per-row bar assumes: unrelated scores.  Rows whose numerators are all equal round the same way and may
    move lse by up to the worst case; tests on such inputs (all-zero queries) use BF16_LSE."""
    p = np.full((1, 1024), np.float32(1.0 + 2.0 ** -8 - 2.0 ** -20))
    lse = np.log(p.astype(np.float64).sum(-1))
    lse2 = np.log((p.astype(np.float64) ** 2).sum(-1))
    assert _lse_shift(p)[0] > bf16_lse_bar(lse, lse2, 1)[0] and _lse_shift(p)[0] <= BF16_LSE
