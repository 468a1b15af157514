"""dfa_forward_static, the entry point for callers that cannot allocate device memory: it runs the kernels of
dfa_forward on a static device array (launch plan + partial results of a split launch) and must give the results
of dfa_forward with a workspace, bit for bit, call after call, also when the shape shrinks or changes between
calls (the array keeps the previous call's contents).  Through the C ABI."""
import numpy as np
import pytest

from gpu_util import check_lse_bf16, error_stats, make_qkv, to_f64

pytestmark = pytest.mark.gpu

SAM_BRANCHES = [(1024, 1), (2048, 2), (4096, 4)]


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2403_09195_amd import binding
    binding.lib()
    return binding


def _same(a, b):
    return bool((a[0] == b[0]).all()) and bool((a[1] == b[1]).all())


def test_static_scratch_matches_dfa_forward_on_consecutive_calls(B, oracle):
    import torch
    # 1: a single image, the launch whose key walks are split over several workgroups per tile (plan and partial results in the scratch)
    (q, k, v), ex = make_qkv(950, 1, 4096, 12, 64, "bf16")
    assert B.workspace_bytes(1, 12, 4096, 64, B.DFA_BF16, SAM_BRANCHES) > 0
    ref1 = B.forward(q, k, v, SAM_BRANCHES, 0.125)
    got1 = B.forward_static(q, k, v, SAM_BRANCHES, 0.125)
    torch.cuda.synchronize()
    assert _same(got1, ref1)
    o_ref, l_ref = oracle.forward(*ex, SAM_BRANCHES, 0.125)
    mx, mean = error_stats(to_f64(got1[0]), o_ref)
    assert mx <= 2e-2 and mean <= 2e-3
    check_lse_bf16(to_f64(got1[1]), oracle, ex, SAM_BRANCHES, 0.125, l_ref)

    # 2: straight after it a smaller input (also split: half the tokens, fewer heads, ragged tiles of 250 rows)
    small_br = [(500, 1), (1000, 2), (2000, 4)]
    (q2, k2, v2), ex2 = make_qkv(951, 1, 2000, 5, 64, "bf16")
    assert B.workspace_bytes(1, 5, 2000, 64, B.DFA_BF16, small_br) > 0
    got2 = B.forward_static(q2, k2, v2, small_br, 0.125)
    ref2 = B.forward(q2, k2, v2, small_br, 0.125)
    torch.cuda.synchronize()
    assert _same(got2, ref2)
    o2, l2 = oracle.forward(*ex2, small_br, 0.125)
    mx, mean = error_stats(to_f64(got2[0]), o2)
    assert mx <= 2e-2 and mean <= 2e-3
    check_lse_bf16(to_f64(got2[1]), oracle, ex2, small_br, 0.125, l2)

    # 3: the first shape again on other data (the plan is copied in anew), twice (the second call only enqueues),
    # into the caller's own output tensors
    (q3, k3, v3), _ = make_qkv(952, 1, 4096, 12, 64, "bf16")
    ref3 = B.forward(q3, k3, v3, SAM_BRANCHES, 0.125)
    out = torch.full_like(ref3[0], float("nan"))
    lse = torch.full_like(ref3[1], float("nan"))
    for _ in range(2):
        got3 = B.forward_static(q3, k3, v3, SAM_BRANCHES, 0.125, out=out, lse=lse)
        torch.cuda.synchronize()
        assert got3[0] is out and _same(got3, ref3)
        out.fill_(float("nan")); lse.fill_(float("nan"))

    # 4: a launch that is not split (a batch that fills the chip) and the fp32 path, rows kept by no branch included
    (q4, k4, v4), _ = make_qkv(953, 16, 1024, 12, 64, "bf16")
    br4 = [(256, 1), (512, 2), (1024, 4)]
    assert B.workspace_bytes(16, 12, 1024, 64, B.DFA_BF16, br4) == 0
    assert _same(B.forward_static(q4, k4, v4, br4, 0.125), B.forward(q4, k4, v4, br4, 0.125))
    (q5, k5, v5), _ = make_qkv(954, 1, 256, 1, 64, "f32")
    got5, ref5 = B.forward_static(q5, k5, v5, [(64, 2)], 0.125), B.forward(q5, k5, v5, [(64, 2)], 0.125)
    assert bool((got5[0] == ref5[0]).all()) and bool((got5[1] == ref5[1]).all())
    assert bool(torch.isneginf(got5[1][0, 0, 1::2]).all())


def test_static_scratch_rejects_what_does_not_fit(B):
    """Segments of a single row make one workgroup per row: 32 images x 12 heads x 4096 rows = 1 572 864 launch items
    of 32 bytes, beyond the 40 MiB array.  Refused with DFA_ERR_WORKSPACE (dfa_forward takes the same problem), and
    the scratch goes on working afterwards.  Real tensors throughout: nothing here depends on the refusal."""
    import torch
    Bsz, N, H = 32, 4096, 12
    plan = B.plan_describe(Bsz, H, N, [(1, 1)])
    assert 32 * len(plan["items"]) > 40 << 20
    q = torch.randn((Bsz, N, H, 64), device="cuda", dtype=torch.float32).bfloat16()
    with pytest.raises(B.DfaError) as e:
        B.forward_static(q, q, q, [(1, 1)], 0.125)
    assert e.value.code == B.DFA_ERR_WORKSPACE
    out, lse = B.forward(q, q, q, [(1, 1)], 0.125)          # every row attends itself alone: out = v
    assert bool((out == q).all())
    (q, k, v), _ = make_qkv(955, 1, 512, 2, 64, "bf16")
    assert _same(B.forward_static(q, k, v, [(128, 1), (512, 4)], 0.125), B.forward(q, k, v, [(128, 1), (512, 4)], 0.125))
