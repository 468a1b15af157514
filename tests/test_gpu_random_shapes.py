"""Seeded random valid problems (sizes, branch sets, head offsets, ragged partitions) through the
forward and backward entry points against the oracle: shapes nobody picked by hand."""
import numpy as np
import pytest

import helpers
from gpu_util import check_lse, check_lse_bf16, error_stats, make_qkv, to_device, to_f64

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


@pytest.mark.parametrize("seed", range(24))
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
            check_lse_bf16(to_f64(lse), oracle, ex, branches, 0.125, l_ref, offs)     # per-row bar
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
        # size of the terms each gradient element is a sum of (dense numpy, independent of oracle and kernels)
        bounds = helpers.multiset_attention_backward(*ex, ge, 0.125, branches, offs)[3:]
        for name, got, ref, absum in zip(("dq", "dk", "dv"), (dq, dk, dv), refs, bounds):
            d = np.abs(to_f64(got) - ref)
            if dtype == "f32":
                assert d.max() <= 2e-5 * max(1.0, np.abs(ref).max()), name
            else:
                # A gradient element is a sum of terms that each carry bf16 roundings of relative size eps = 2^-9:
                # P or dS rounded for the second product, delta taken from the rounded forward output, and the
                # result's own rounding.  Rows differ widely in size (short lists: sharp softmax, large terms) and
                # sums cancel, so the bar is the forward bound eps * sum|terms| of each element, not a fraction
                # of the result: |err| <= 2^-8 |g| + 4 eps sum|terms| per element (worst seen over 132 seeds: 1.5 eps),
                # 4 eps on a row's mean (worst 1.7), and eps on the mean over the tensor, where the roundings
                # average out (worst 0.42).  Elements with no term at all must come out as zero.
                eps = 2.0 ** -9
                assert np.all(d <= 2.0 ** -8 * np.abs(ref) + 4 * eps * absum + 1e-6), name
                assert np.all(d.mean(axis=-1) <= 4 * eps * absum.mean(axis=-1) + 1e-6), name
                assert d.mean() <= eps * absum.mean() + 1e-7, name
            assert np.all(to_f64(got)[dead] == 0.0)


def _many_branch_problem(seed):
    """Up to eight branches on a few thousand tokens; every third problem with nested power-of-two rates and
    segment lengths (the workloads' pattern: many shared keys), the others with arbitrary ones."""
    rng = np.random.default_rng(7000 + seed)
    H = int(rng.integers(1, 4))
    N = int(rng.integers(300, 5000))
    nb = int(rng.integers(2, 9))
    nested = seed % 3 == 0
    branches, offs = [], []
    for _ in range(nb):
        r = int(rng.choice([1, 2, 4, 8, 16])) if nested else int(rng.choice([1, 2, 3, 4, 6, 8, 12, 16]))
        w = int(rng.choice([64, 128, 256, 512, 1024, 2048, 4096])) if nested else int(rng.integers(max(r, 16), 2 * N))
        branches.append((w, r))
        offs.append([int(rng.integers(0, r)) for _ in range(H)])
    return N, H, branches, (None if nested or seed % 2 == 0 else offs)


@pytest.mark.parametrize("seed", range(12))
def test_random_problem_with_many_branches_forward(B, oracle, seed):
    """Keys kept by up to eight branches at once: the plans of these problems carry multiplicities up to 8."""
    N, H, branches, offs = _many_branch_problem(seed)
    print(f"[many branches {seed}] N={N} H={H} branches={branches} offsets={offs}", flush=True)
    for dtype in ("bf16", "f32"):
        (q, k, v), ex = make_qkv(3000 + seed, 1, N, H, 64, dtype)
        out, lse = B.forward(q, k, v, branches, 0.125, head_offsets=offs)
        o_ref, l_ref = oracle.forward(*ex, branches, 0.125, head_offsets=offs)
        mx, mean = error_stats(to_f64(out), o_ref)
        if dtype == "bf16":
            check_lse_bf16(to_f64(lse), oracle, ex, branches, 0.125, l_ref, offs)     # per-row bar
            assert mx <= 2e-2 and mean <= 2e-3
        else:
            check_lse(to_f64(lse), l_ref, atol=1e-5, rtol=1e-5)
            assert mx <= 1e-5
        assert np.all(to_f64(out)[np.isneginf(l_ref).transpose(0, 2, 1)] == 0.0)


def _small_group_problem(seed):
    """Problems whose row groups are smaller than a tile and share keys: the workloads' nested family scaled to small
    images, and sets of narrow windows with arbitrary rates and offsets."""
    rng = np.random.default_rng(9000 + seed)
    Bsz, H = int(rng.integers(1, 4)), int(rng.integers(1, 5))
    if seed % 2 == 0:
        N = int(rng.choice([128, 256, 384, 512, 768, 1024, 1536, 2048]))
        nb = int(rng.integers(2, 5))
        branches = [(max(N >> (nb - 1 - x), 1 << x), 1 << x) for x in range(nb)]
        return Bsz, N, H, branches, None
    N = int(rng.integers(64, 1500))
    branches = [(int(rng.choice([16, 32, 48, 64, 100, 128, 200, 256])), int(rng.integers(1, 5))) for _ in range(int(rng.integers(2, 6)))]
    offs = [[int(rng.integers(0, r)) for _ in range(H)] for (_, r) in branches]
    return Bsz, N, H, branches, offs


@pytest.mark.parametrize("seed", range(40))
def test_random_problem_with_small_row_groups_bf16(B, oracle, seed):
    """Plans that pack several row groups into a tile (and, for single images, split the walks): out within the rounding
    of its bf16 result and of its numerators, lse within the row's bar; every seventh problem at scale = 1."""
    Bsz, N, H, branches, offs = _small_group_problem(seed)
    scale = 1.0 if seed % 7 == 0 else 0.125
    plan = B.plan_describe_forward(Bsz, H, N, branches, offs)
    packed = bool((plan["block_mult"] == 0).any())
    split = B.workspace_bytes(Bsz, H, N, 64, B.DFA_BF16, branches, offs) > 0
    print(f"[small groups {seed}] B={Bsz} N={N} H={H} branches={branches} offsets={offs} scale={scale} packed={packed} split={split}", flush=True)
    (q, k, v), ex = make_qkv(4000 + seed, Bsz, N, H, 64, "bf16")
    out, lse = B.forward(q, k, v, branches, scale, head_offsets=offs)
    o_ref, l_ref = oracle.forward(*ex, branches, scale, head_offsets=offs)
    check_lse_bf16(to_f64(lse), oracle, ex, branches, scale, l_ref, offs)
    d = np.abs(to_f64(out) - o_ref)
    assert np.all(d <= 2.0 ** -7 * np.maximum(1.0, np.abs(o_ref)))
    assert np.all(to_f64(out)[np.isneginf(l_ref).transpose(0, 2, 1)] == 0.0)


@pytest.mark.parametrize("seed", [3, 17, 22, 41, 59])
def test_random_problem_with_sharp_softmax_bf16(B, oracle, seed):
    """scale = 1 (Eq. 2 as printed): scores of standard deviation 8, so one or two keys carry most rows.  That is
    where the rounding of a single numerator shows in the denominator: lse must stay inside the derived bar, and
    out, whose values reach 4 here, inside the rounding of its own bf16 result plus that of its few numerators."""
    Bsz, N, H, branches, offs = _problem(seed)
    print(f"[sharp {seed}] B={Bsz} N={N} H={H} branches={branches} offsets={offs}", flush=True)
    (q, k, v), ex = make_qkv(2000 + seed, Bsz, N, H, 64, "bf16")
    out, lse = B.forward(q, k, v, branches, 1.0, head_offsets=offs)
    o_ref, l_ref = oracle.forward(*ex, branches, 1.0, head_offsets=offs)
    # few keys carry a row here: the per-row bar is at or near the worst case for most rows
    le, _ = check_lse_bf16(to_f64(lse), oracle, ex, branches, 1.0, l_ref, offs)
    d = np.abs(to_f64(out) - o_ref)
    print(f"[sharp {seed}] lse max-abs {le:.3e} out max-abs {d.max():.3e}", flush=True)
    assert np.all(d <= 2.0 ** -7 * np.maximum(1.0, np.abs(o_ref)))
    assert np.all(to_f64(out)[np.isneginf(l_ref).transpose(0, 2, 1)] == 0.0)
