"""The caller-owned workspace of dfa_forward (room for the partial results of a launch whose tiles are
walked by several workgroups each): calls of one shape that overlap on two streams, each with a workspace of its
own, give the results of serial calls; without a workspace the unsplit launch agrees to rounding; too small a
workspace is refused.  All through the C ABI."""
import ctypes

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


def test_two_streams_one_shape_each_with_its_own_workspace(B, oracle):
    import torch
    Bsz, N, H, D = 1, 4096, 12, 64
    need = B.workspace_bytes(Bsz, H, N, D, B.DFA_BF16, SAM_BRANCHES)
    assert need == 512 * 256 * (64 * 2 + 8)                       # this shape is split: one block of partial results per workgroup slot
    inputs = [make_qkv(900 + i, Bsz, N, H, D, "bf16") for i in range(2)]
    serial = []
    for (q, k, v), _ in inputs:
        ws = torch.empty((need,), dtype=torch.uint8, device="cuda")
        serial.append(B.forward(q, k, v, SAM_BRANCHES, 0.125, workspace=ws))
    torch.cuda.synchronize()
    # against the oracle once
    o_ref, l_ref = oracle.forward(*inputs[0][1], SAM_BRANCHES, 0.125)
    mx, mean = error_stats(to_f64(serial[0][0]), o_ref)
    assert mx <= 2e-2 and mean <= 2e-3
    check_lse_bf16(to_f64(serial[0][1]), oracle, inputs[0][1], SAM_BRANCHES, 0.125, l_ref)

    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    spaces = [torch.empty((need,), dtype=torch.uint8, device="cuda") for _ in range(2)]
    outs = [[], []]
    torch.cuda.synchronize()
    for rep in range(8):                                    # interleaved enqueues: the launches of the two streams overlap
        for i, st in enumerate(streams):
            with torch.cuda.stream(st):
                (q, k, v), _ = inputs[i]
                outs[i].append(B.forward(q, k, v, SAM_BRANCHES, 0.125, workspace=spaces[i]))
    torch.cuda.synchronize()
    for i in range(2):
        for out, lse in outs[i]:
            assert bool((out == serial[i][0]).all()) and bool((lse == serial[i][1]).all())


def test_no_workspace_runs_unsplit_and_small_workspace_is_refused(B, oracle):
    import torch
    Bsz, N, H, D = 1, 4096, 12, 64
    (q, k, v), ex = make_qkv(902, Bsz, N, H, D, "bf16")
    need = B.workspace_bytes(Bsz, H, N, D, B.DFA_BF16, SAM_BRANCHES)
    out_s, lse_s = B.forward(q, k, v, SAM_BRANCHES, 0.125)                     # "auto": split
    out_u, lse_u = B.forward(q, k, v, SAM_BRANCHES, 0.125, workspace=None)     # unsplit
    o_ref, l_ref = oracle.forward(*ex, SAM_BRANCHES, 0.125)
    for out, lse in ((out_s, lse_s), (out_u, lse_u)):
        mx, mean = error_stats(to_f64(out), o_ref)
        assert mx <= 2e-2 and mean <= 2e-3
        check_lse_bf16(to_f64(lse), oracle, ex, SAM_BRANCHES, 0.125, l_ref)
    small = torch.empty((need - 256,), dtype=torch.uint8, device="cuda")
    with pytest.raises(B.DfaError) as e:
        B.forward(q, k, v, SAM_BRANCHES, 0.125, workspace=small)
    assert e.value.code == B.DFA_ERR_WORKSPACE
    # a shape that needs none ignores whatever is passed
    (q2, k2, v2), _ = make_qkv(903, 4, 512, 2, D, "bf16")
    a = B.forward(q2, k2, v2, [(128, 1)], 0.125, workspace=small)
    b = B.forward(q2, k2, v2, [(128, 1)], 0.125, workspace=None)
    assert bool((a[0] == b[0]).all()) and bool((a[1] == b[1]).all())


def test_plan_cache_keeps_working_past_its_bound(B, oracle):
    """More shapes than the cache holds (64): the oldest plans are dropped and rebuilt on demand."""
    (q, k, v), ex = make_qkv(904, 1, 70 * 64, 1, 64, "bf16")
    first = None
    for n in range(1, 71):
        N = 64 * n
        out, lse = B.forward(q[:, :N], k[:, :N], v[:, :N], [(64, 1)], 0.125)
        if n == 1:
            first = (out.clone(), lse.clone())
    out, lse = B.forward(q[:, :64], k[:, :64], v[:, :64], [(64, 1)], 0.125)    # dropped by now, built again
    assert bool((out == first[0]).all()) and bool((lse == first[1]).all())
    o_ref, l_ref = oracle.forward(ex[0][:, :64], ex[1][:, :64], ex[2][:, :64], [(64, 1)], 0.125)
    mx, mean = error_stats(to_f64(out), o_ref)
    assert mx <= 2e-2 and mean <= 2e-3
