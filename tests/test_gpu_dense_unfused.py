"""The size sweep's comparison path (dense attention with the score matrix held in memory, section 4.3's
"FlashAttention off") against the oracle's dense case w = N, r = 1, and against the fused kernel on the same
inputs.  Bars: outputs as everywhere (max-abs 2e-2, mean-abs 2e-3); lse: the scores pass through memory as
bf16, so a scaled score below 8 in magnitude is off by at most half a unit of an 8-bit significand, 2^-6, and
lse by no more than its worst score."""
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


@pytest.mark.parametrize("Bsz,N,H", [(2, 256, 3), (1, 512, 2), (2, 1024, 6), (1, 4096, 2)])
def test_dense_unfused_matches_the_oracle(B, oracle, Bsz, N, H):
    (q, k, v), ex = make_qkv(700 + N, Bsz, N, H, 64, "bf16")
    out, lse = B.dense_unfused(q, k, v, 0.125)
    o_ref, l_ref = oracle.forward(*ex, [(N, 1)], 0.125)
    assert float(np.abs(0.125 * np.einsum("bnhd,bmhd->bhnm", ex[0], ex[1])).max()) < 8.0      # what the lse bar assumes
    mx, mean = error_stats(to_f64(out), o_ref)
    le = check_lse(to_f64(lse), l_ref, atol=2.0 ** -6 + 1e-5)
    print(f"[dense unfused N={N}] out max-abs {mx:.3e} mean-abs {mean:.3e} lse max-abs {le:.3e}", flush=True)
    assert mx <= 2e-2 and mean <= 2e-3
    # the fused kernel on the same problem agrees with it to the same bars
    fo, fl = B.forward(q, k, v, [(N, 1)], 0.125)
    mx2, mean2 = error_stats(to_f64(out), to_f64(fo))
    assert mx2 <= 2e-2 and mean2 <= 2e-3


def test_dense_unfused_reads_strided_views_and_checks_its_arguments(B, oracle):
    import torch
    from paper_2403_09195_amd import synth
    Bsz, N, H, D = 2, 256, 2, 64
    st, ex = synth.tensor(710, 3, (Bsz, N, 3, H, D), "bf16")
    packed = to_device(st)
    out, lse = B.dense_unfused(packed[:, :, 0], packed[:, :, 1], packed[:, :, 2], 0.125)
    o_ref, l_ref = oracle.forward(ex[:, :, 0], ex[:, :, 1], ex[:, :, 2], [(N, 1)], 0.125)
    mx, mean = error_stats(to_f64(out), o_ref)
    assert mx <= 2e-2 and mean <= 2e-3
    check_lse(to_f64(lse), l_ref, atol=2.0 ** -6 + 1e-5)
    q = packed[:, :, 0]
    with pytest.raises(B.DfaError) as e:                       # rows that are no whole 256-row tiles
        B.dense_unfused(q[:, :200], q[:, :200], q[:, :200], 0.125)
    assert e.value.code == -2
    with pytest.raises(B.DfaError) as e:
        B.dense_unfused(q, q, q, 0.125, workspace=torch.empty((1024,), dtype=torch.uint8, device="cuda"))
    assert e.value.code == B.DFA_ERR_WORKSPACE
