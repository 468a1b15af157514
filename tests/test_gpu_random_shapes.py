"""Seeded random valid problems (sizes, branch sets, head offsets, ragged partitions) through the
forward and backward entry points against the oracle: shapes nobody picked by hand."""
import numpy as np
import pytest

from gpu_util import check_lse, error_stats, make_qkv, to_device, to_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2403_09195_amd import binding
    binding.lib()
    return binding


def _problem(seed):
    rng = np.random.default_rng(1000 + seed)
    Bsz, H = int(rng.integers(1, 4)), int(rng.integers(1, 6))
    N = int(rng.integers(40, 1400))
    nb = int(rng.integers(1, 5))
    branches, offs = [], []
    for _ in range(nb):
        r = int(rng.integers(1, 7))
        w = int(rng.integers(max(r, 8), 2 * N))                 # any segment length, also beyond N
        branches.append((w, r))
        offs.append([int(rng.integers(0, r)) for _ in range(H)])
    return Bsz, N, H, branches, (offs if seed % 2 else None)


@pytest.mark.parametrize("seed", range(12))
def test_random_problem_forward_and_backward(B, oracle, seed):
    from paper_2403_09195_amd import synth
    Bsz, N, H, branches, offs = _problem(seed)
    print(f"[random {seed}] B={Bsz} N={N} H={H} branches={branches} offsets={offs}", flush=True)
    for dtype in ("bf16", "f32"):
        (q, k, v), ex = make_qkv(2000 + seed, Bsz, N, H, 64, dtype)
        out, lse = B.forward(q, k, v, branches, 0.125, head_offsets=offs)
        o_ref, l_ref = oracle.forward(*ex, branches, 0.125, head_offsets=offs)
        mx, mean = error_stats(to_f64(out), o_ref)
        if dtype == "bf16":
            check_lse(to_f64(lse), l_ref, atol=2e-3)
            assert mx <= 2e-2 and mean <= 2e-3
        else:
            check_lse(to_f64(lse), l_ref, atol=1e-5, rtol=1e-5)
            assert mx <= 1e-5
        dead = np.isneginf(l_ref).transpose(0, 2, 1)
        assert np.all(to_f64(out)[dead] == 0.0)
        st, ge = synth.tensor(2000 + seed, 7, (Bsz, N, H, 64), dtype)
        g = to_device(st)
        dq, dk, dv = B.backward(q, k, v, out, lse, g, branches, 0.125, head_offsets=offs)
        refs = oracle.backward(*ex, ge, branches, 0.125, head_offsets=offs)
        for name, got, ref in zip(("dq", "dk", "dv"), (dq, dk, dv), refs):
            d = np.abs(to_f64(got) - ref)
            if dtype == "f32":
                assert d.max() <= 2e-5 * max(1.0, np.abs(ref).max()), name
            else:
                # Rows differ widely here (a row with a short list has a sharp softmax and large gradients, one
                # with long lists small ones), so each row is held to its own size: per element
                # |err| <= 2^-8 |g| + 3e-2 rms(row), and the mean error of a row <= 2^-7 rms(row) + 1e-5: a row with a
                # dozen keys averages nothing, so the bf16 roundings of P, dS, the forward's out (through delta) and
                # the result, 2^-9 each, add up (measured worst 0.0044 rms(row), on 13-key rows).
                row_rms = np.sqrt(np.mean(ref ** 2, axis=-1, keepdims=True))
                assert np.all(d <= 2.0 ** -8 * np.abs(ref) + 3e-2 * row_rms + 1e-5), name
                assert np.all(d.mean(axis=-1, keepdims=True) <= 2.0 ** -7 * row_rms + 1e-5), name
            assert np.all(to_f64(got)[dead] == 0.0)
