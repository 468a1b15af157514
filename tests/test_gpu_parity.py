"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the same
seeded inputs.  Bars: index maps and byte movement bit-exact; bf16 outputs max-abs <= 2e-2 and
mean-abs <= 2e-3; fp32 outputs max-abs <= 1e-5; lse (no bar given by the workload definition):
bf16 per row from the arithmetic (gpu_util.bf16_lse_bar: about 1e-3 on the workloads' rows, never more than the
worst case 3.95e-3, which alone applies to inputs with equal or hand-made scores), fp32 1e-5 * max(1, |lse|),
with -inf matching exactly."""
import numpy as np
import pytest

from gpu_util import BF16_LSE, check_lse, check_lse_bf16, error_stats, make_qkv, to_device, to_f64

pytestmark = pytest.mark.gpu

BF16_MAX, BF16_MEAN, F32_MAX = 2e-2, 2e-3, 1e-5


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2403_09195_amd import binding
    binding.lib()
    return binding


def _check_bf16(out, lse, o_ref, l_ref, tag="", rows=None):
    """rows = (oracle, ex, branches, scale, head_offsets) of a problem on random data: lse is then held to the
    per-row bar; without it to the worst-case bar."""
    mx, mean = error_stats(to_f64(out), o_ref)
    if rows is None:
        le, frac = check_lse(to_f64(lse), l_ref, atol=BF16_LSE), float("nan")
    else:
        le, frac = check_lse_bf16(to_f64(lse), rows[0], rows[1], rows[2], rows[3], l_ref, rows[4])
    print(f"[{tag}] bf16 out max-abs {mx:.3e} mean-abs {mean:.3e} lse max-abs {le:.3e} (at most {frac:.2f} of a row's bar)", flush=True)
    assert mx <= BF16_MAX and mean <= BF16_MEAN
    return mx, mean


def _check_f32(out, lse, o_ref, l_ref, tag="", tol=F32_MAX):
    mx, mean = error_stats(to_f64(out), o_ref)
    le = check_lse(to_f64(lse), l_ref, atol=tol, rtol=1e-5)
    print(f"[{tag}] f32 out max-abs {mx:.3e} mean-abs {mean:.3e} lse max-abs {le:.3e}", flush=True)
    assert mx <= tol
    return mx


# ---------------------------------------------------------------- indexer, gather, placement
@pytest.mark.parametrize("N,H,w,r,offs", [
    (256, 1, 64, 2, None), (4096, 12, 1024, 1, None), (4096, 12, 2048, 2, None),
    (4096, 12, 4096, 4, None), (16384, 12, 16384, 8, None), (360, 5, 120, 3, [2, 0, 1, 1, 2]),
    (64, 3, 64, 64, None), (7, 2, 7, 1, None),
])
def test_device_index_map_bit_exact(B, oracle, N, H, w, r, offs):
    got = B.index_map_device(N, H, w, r, offs).cpu().numpy()
    ref = oracle.index_map(N, H, w, r, offs)
    assert got.dtype == np.int32 and np.array_equal(got, ref)
    assert np.array_equal(np.array(B.index_map(N, H, w, r, offs), dtype=np.int32), ref)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("N,H,w,r,offs", [(512, 5, 128, 4, None), (360, 3, 120, 3, [2, 0, 1]), (256, 2, 256, 1, None)])
def test_gather_and_placement_bit_exact(B, oracle, dtype, N, H, w, r, offs):
    from paper_2403_09195_amd import synth
    Bsz, D = 3, 64
    st, _ = synth.tensor(77, 3, (Bsz, N, H, D), dtype)
    x = to_device(st)
    idx = oracle.index_map(N, H, w, r, offs)                       # [H, N/r]
    xg = B.gather(x, w, r, offs)
    import torch
    raw = lambda t: t.cpu().view(dtype=torch.int16 if dtype == "bf16" else torch.int32).numpy()
    host = st.view(np.int16) if dtype == "bf16" else st.view(np.int32)
    ref_g = np.stack([host[:, idx[h], h, :] for h in range(H)], axis=1)     # [B, H, N/r, D]
    assert np.array_equal(raw(xg), ref_g)
    back = B.scatter(xg, N, w, r, offs)
    ref_s = np.zeros_like(host)
    for h in range(H):
        ref_s[:, idx[h], h, :] = host[:, idx[h], h, :]
    assert np.array_equal(raw(back), ref_s)


def test_gather_reads_strided_views(B, oracle):
    import torch
    from paper_2403_09195_amd import synth
    Bsz, N, H, D, w, r = 2, 256, 4, 64, 64, 2
    st, _ = synth.tensor(78, 3, (Bsz, N, 3, H, D), "bf16")
    packed = to_device(st)
    k_view = packed[:, :, 1]                                         # [B, N, H, D], strided
    idx = oracle.index_map(N, H, w, r)
    got = B.gather(k_view, w, r).cpu().view(dtype=torch.int16).numpy()
    host = st.view(np.int16)[:, :, 1]
    assert np.array_equal(got, np.stack([host[:, idx[h], h, :] for h in range(H)], axis=1))


# ---------------------------------------------------------------- fp32 path
def test_tiny_config_fp32(B, oracle):
    from paper_2403_09195_amd import synth
    c = synth.CONFIGS["tiny"]
    (q, k, v), ex = make_qkv(c["seed"], c["B"], c["N"], c["H"], c["D"], "f32")
    out, lse = B.forward(q, k, v, c["branches"], 0.125)
    o_ref, l_ref = oracle.forward(*ex, c["branches"], 0.125)
    _check_f32(out, lse, o_ref, l_ref, "tiny")
    odd = to_f64(out)[0, 1::2, 0]
    assert np.all(odd == 0.0) and np.all(np.isneginf(to_f64(lse)[0, 0, 1::2]))   # rows kept by nothing
    out2, lse2 = B.forward(q, k, v, c["branches"], 0.125)
    assert bool((out2 == out).all()) and bool((lse2 == lse).all())             # deterministic


@pytest.mark.parametrize("scale", [0.125, 1.0])
def test_fp32_multi_branch_ragged(B, oracle, scale):
    # key lists of 40 and 100 keys (ragged 64-key tiles), 300-row groups (ragged 256-row tiles)
    Bsz, N, H, D = 2, 1200, 3, 64
    branches = [(120, 3), (600, 2), (1200, 12)]
    offs = [[2, 0, 1], [1, 1, 0], [5, 11, 0]]
    (q, k, v), ex = make_qkv(101, Bsz, N, H, D, "f32")
    out, lse = B.forward(q, k, v, branches, scale, head_offsets=offs)
    o_ref, l_ref = oracle.forward(*ex, branches, scale, head_offsets=offs)
    # scale = 1 is the literal Eq. 2 (logits 8x larger: sigma 8, row maxima 30-40); the same 1e-5 bar
    _check_f32(out, lse, o_ref, l_ref, f"f32 ragged s={scale}")


# ---------------------------------------------------------------- bf16 path
def test_bf16_small_multi_tile(B, oracle):
    Bsz, N, H, D = 2, 1024, 5, 64
    branches = [(256, 1), (512, 2), (1024, 4)]
    (q, k, v), ex = make_qkv(102, Bsz, N, H, D, "bf16")
    out, lse = B.forward(q, k, v, branches, 0.125)
    o_ref, l_ref = oracle.forward(*ex, branches, 0.125)
    _check_bf16(out, lse, o_ref, l_ref, "bf16 small", rows=(oracle, ex, branches, 0.125, None))
    out2, lse2 = B.forward(q, k, v, branches, 0.125)
    assert bool((out2 == out).all()) and bool((lse2 == lse).all())


@pytest.mark.parametrize("Bsz,N,H,branches,split", [
    (2, 256, 6, [(64, 1), (128, 2), (256, 4)], False),       # 256^2 image: groups of 32, 16, 16 rows, filler slots between them
    (3, 1024, 12, [(256, 1), (512, 2), (1024, 4)], False),   # 512^2 image: groups of 128, 64, 64 rows fill a tile exactly
    (1, 2048, 4, [(512, 1), (1024, 2), (2048, 4)], True),    # two groups of 128 rows share a tile whose walk is split over workgroups
    (2, 600, 3, [(100, 1), (300, 2), (600, 3), (50, 1)], False),   # ragged groups, rates 2 and 3
])
def test_bf16_tiles_that_pack_several_row_groups(B, oracle, Bsz, N, H, branches, split):
    """Row groups that fill only part of a tile share one (each on waves of its own, the tile walking the union of
    their key lists, a wave masking the progressions its rows do not attend to): results as from the definition."""
    plan = B.plan_describe_forward(Bsz, H, N, branches)
    plain = B.plan_describe(Bsz, H, N, branches)
    assert len(plan["tiles"]) < len(plain["tiles"]) and int((plan["block_mult"] == 0).sum()) > 0
    assert (B.workspace_bytes(Bsz, H, N, 64, B.DFA_BF16, branches) > 0) == split
    (q, k, v), ex = make_qkv(110 + N, Bsz, N, H, 64, "bf16")
    out, lse = B.forward(q, k, v, branches, 0.125)
    o_ref, l_ref = oracle.forward(*ex, branches, 0.125)
    _check_bf16(out, lse, o_ref, l_ref, f"bf16 packed N={N}", rows=(oracle, ex, branches, 0.125, None))
    if split:
        out_u, lse_u = B.forward(q, k, v, branches, 0.125, workspace=None)      # the same tiles walked whole
        _check_bf16(out_u, lse_u, o_ref, l_ref, f"bf16 packed unsplit N={N}", rows=(oracle, ex, branches, 0.125, None))


def test_bf16_packed_plan_of_many_workgroups(B, oracle):
    """A long launch of packed tiles (several rounds of the chip's workgroup slots): 4096 (b, h) units of a 256^2
    image, 8192 workgroups of six row groups each."""
    Bsz, N, H = 128, 256, 32
    branches = [(64, 1), (128, 2), (256, 4)]
    plan = B.plan_describe_forward(Bsz, H, N, branches)
    assert int((plan["items"][:, 0] >= 0).sum()) == 8192 and int((plan["block_mult"] == 0).sum()) > 0
    (q, k, v), ex = make_qkv(140, Bsz, N, H, 64, "bf16")
    out, lse = B.forward(q, k, v, branches, 0.125)
    o_ref, l_ref = oracle.forward(*ex, branches, 0.125)
    _check_bf16(out, lse, o_ref, l_ref, "bf16 packed, long launch", rows=(oracle, ex, branches, 0.125, None))


def test_bf16_ragged_tiles_explicit_offsets_and_uncovered_rows(B, oracle):
    Bsz, N, H, D = 2, 1200, 3, 64
    branches = [(120, 3), (600, 2), (1200, 12)]
    offs = [[2, 0, 1], [1, 1, 0], [5, 11, 0]]
    (q, k, v), ex = make_qkv(103, Bsz, N, H, D, "bf16")
    out, lse = B.forward(q, k, v, branches, 0.125, head_offsets=offs)
    o_ref, l_ref = oracle.forward(*ex, branches, 0.125, head_offsets=offs)
    _check_bf16(out, lse, o_ref, l_ref, "bf16 ragged", rows=(oracle, ex, branches, 0.125, offs))
    dead = np.isneginf(l_ref).transpose(0, 2, 1)                     # [B, N, H]
    assert dead.any() and np.all(to_f64(out)[dead] == 0.0)


def test_bf16_dense_special_case_and_single_head(B, oracle):
    # w = N, r = 1: plain softmax attention
    (q, k, v), ex = make_qkv(104, 1, 320, 1, 64, "bf16")
    out, lse = B.forward(q, k, v, [(320, 1)], 0.125)
    o_ref, l_ref = oracle.forward(*ex, [(320, 1)], 0.125)
    _check_bf16(out, lse, o_ref, l_ref, "bf16 dense", rows=(oracle, ex, [(320, 1)], 0.125, None))


def test_bf16_eight_branches_and_no_lse(B, oracle):
    Bsz, N, H, D = 1, 512, 4, 64
    branches = [(64, 1), (128, 2), (256, 4), (512, 8), (512, 1), (256, 2), (128, 4), (64, 8)]
    (q, k, v), ex = make_qkv(105, Bsz, N, H, D, "bf16")
    out, lse = B.forward(q, k, v, branches, 0.125)
    o_ref, l_ref = oracle.forward(*ex, branches, 0.125)
    _check_bf16(out, lse, o_ref, l_ref, "bf16 8 branches", rows=(oracle, ex, branches, 0.125, None))
    out2, none = B.forward(q, k, v, branches, 0.125, want_lse=False)
    assert none is None and bool((out2 == out).all())


@pytest.mark.parametrize("count,r", [(1, 1), (2, 1), (31, 1), (32, 1), (33, 1), (63, 2), (64, 1), (65, 3),
                                     (95, 1), (96, 2), (97, 1), (128, 1), (129, 2), (257, 1)])
def test_bf16_key_counts_around_the_pipeline_beats(B, oracle, count, r):
    """Segments of `count` kept keys: one key (a row attends only itself), and counts just below,
    at and above the 32-key beat and the 64-key stage of the kernel's pipeline, with a second,
    coarser branch on top so that two key lists of ragged length are walked back to back."""
    w = count * r
    N, H = 4 * w, 3
    branches = [(w, r), (2 * w, 2 * r)]
    (q, k, v), ex = make_qkv(300 + count, 2, N, H, 64, "bf16")
    out, lse = B.forward(q, k, v, branches, 0.125)
    o_ref, l_ref = oracle.forward(*ex, branches, 0.125)
    _check_bf16(out, lse, o_ref, l_ref, f"bf16 count {count} r {r}", rows=(oracle, ex, branches, 0.125, None))
    out1, lse1 = B.forward(q, k, v, branches[:1], 0.125)
    o1, l1 = oracle.forward(*ex, branches[:1], 0.125)
    _check_bf16(out1, lse1, o1, l1, f"bf16 count {count} r {r}, one branch", rows=(oracle, ex, branches[:1], 0.125, None))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("N,branches,offs", [
    (1000, [(300, 1), (128, 3), (2048, 7)], None),                 # w does not divide N, r does not divide w, w > N
    (1025, [(1024, 1), (512, 2)], None),                           # a last part of a single token
    (777, [(100, 4), (250, 5), (777, 9)], [[3, 0], [4, 2], [8, 1]]),
])
def test_ragged_partitions(B, oracle, dtype, N, branches, offs):
    """Shapes the paper's equal-length parts do not cover: short last part, one part for w > N,
    every r-th row of a part from the head's start when r does not divide w."""
    H = 2
    (q, k, v), ex = make_qkv(320 + N, 2, N, H, 64, dtype)
    out, lse = B.forward(q, k, v, branches, 0.125, head_offsets=offs)
    o_ref, l_ref = oracle.forward(*ex, branches, 0.125, head_offsets=offs)
    if dtype == "bf16":
        _check_bf16(out, lse, o_ref, l_ref, f"ragged N={N}", rows=(oracle, ex, branches, 0.125, offs))
    else:
        _check_f32(out, lse, o_ref, l_ref, f"ragged N={N}")
    dead = np.isneginf(l_ref).transpose(0, 2, 1)
    assert np.all(to_f64(out)[dead] == 0.0)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("N,branches,offs", [
    (512, [(256, 2), (256, 2), (512, 1)], None),                   # one branch twice: its keys count double
    (768, [(192, 2), (384, 3), (768, 1)], None),                   # rates 2 and 3: shared keys every 6th row
    (1024, [(256, 1), (512, 2), (1024, 4), (1024, 8)], None),      # nested rates, multiplicities 1 to 4
    (640, [(128, 4), (320, 2), (640, 4)], [[1, 1], [1, 1], [1, 3]]),   # explicit offsets: two branches share keys in one head only
])
def test_keys_kept_by_several_branches(B, oracle, dtype, N, branches, offs):
    """Branch sets whose key lists overlap: the launch plan visits a shared key once and weights it by
    the number of branches that keep it; the oracle visits it once per branch."""
    H = 2
    plan = B.plan_describe(2, H, N, branches, offs)
    assert int(plan["segs"][:, 3].max()) >= 2                      # the case does exercise a multiplicity
    (q, k, v), ex = make_qkv(340 + N, 2, N, H, 64, dtype)
    out, lse = B.forward(q, k, v, branches, 0.125, head_offsets=offs)
    o_ref, l_ref = oracle.forward(*ex, branches, 0.125, head_offsets=offs)
    if dtype == "bf16":
        _check_bf16(out, lse, o_ref, l_ref, f"shared keys N={N}", rows=(oracle, ex, branches, 0.125, offs))
    else:
        _check_f32(out, lse, o_ref, l_ref, f"shared keys N={N}")


def test_bf16_reference_exponent_moves_when_logits_keep_growing(B, oracle):
    """Keys ordered so that logits grow along every key list (and jump between lists): the
    reference exponent of the online softmax has to move many times, also late in the walk,
    and the accumulator is rescaled each time.  Keys with falling logits follow in the second
    head, where it must never move after the first block."""
    import torch
    from paper_2403_09195_amd import synth
    Bsz, N, H, D = 1, 1024, 2, 64
    branches = [(512, 1), (1024, 2)]
    st, ex = synth.qkv(301, Bsz, N, H, D, "bf16")
    q, k, v = (np.array(a, dtype=np.float64) for a in ex)
    q[:] = np.abs(q)                                   # q.k grows with the ramp applied to k below
    ramp = np.linspace(0.2, 6.0, N)[None, :, None, None]
    k = np.abs(k) * ramp
    k[:, :, 1] = k[:, ::-1, 1]                         # head 1: falling
    def to_bf16(a):
        t = torch.from_numpy(a.astype(np.float32)).bfloat16()
        return t.cuda(), t.float().numpy().astype(np.float64)
    (qd, qe), (kd, ke), (vd, ve) = to_bf16(q), to_bf16(k), to_bf16(v)
    out, lse = B.forward(qd, kd, vd, branches, 0.125)
    o_ref, l_ref = oracle.forward(qe, ke, ve, branches, 0.125)
    assert l_ref.max() > 40.0                          # far beyond what one fixed exponent could carry in bf16 sums
    mx, mean = error_stats(to_f64(out), o_ref)
    le = check_lse(to_f64(lse), l_ref, atol=0.0, rtol=1e-4)
    print(f"[growing logits] out max-abs {mx:.3e} mean-abs {mean:.3e} lse rel {le:.3e}", flush=True)
    assert mx <= BF16_MAX and mean <= BF16_MEAN


def test_bf16_side_stream_and_plan_release(B, oracle):
    """The launch goes to the caller's stream; a released plan cache is rebuilt on the next call."""
    import torch
    Bsz, N, H, D = 2, 768, 3, 64
    branches = [(256, 1), (768, 3)]
    (q, k, v), ex = make_qkv(302, Bsz, N, H, D, "bf16")
    out0, lse0 = B.forward(q, k, v, branches, 0.125)
    o_ref, l_ref = oracle.forward(*ex, branches, 0.125)
    _check_bf16(out0, lse0, o_ref, l_ref, "default stream", rows=(oracle, ex, branches, 0.125, None))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        out1, lse1 = B.forward(q, k, v, branches, 0.125)
    side.synchronize()
    assert bool((out1 == out0).all()) and bool((lse1 == lse0).all())
    torch.cuda.synchronize()
    B.release_plans()
    out2, lse2 = B.forward(q, k, v, branches, 0.125)
    assert bool((out2 == out0).all()) and bool((lse2 == lse0).all())
    # another shape in between, then the first one again (two cached plans)
    (q3, k3, v3), ex3 = make_qkv(303, 1, 256, 2, D, "bf16")
    out3, lse3 = B.forward(q3, k3, v3, [(128, 2)], 0.125)
    o3, l3 = oracle.forward(*ex3, [(128, 2)], 0.125)
    _check_bf16(out3, lse3, o3, l3, "second shape", rows=(oracle, ex3, [(128, 2)], 0.125, None))
    out4, _ = B.forward(q, k, v, branches, 0.125)
    assert bool((out4 == out0).all())


@pytest.mark.parametrize("Bsz,N,H", [(4, 1024, 6), (1, 2048, 3)])
def test_forward_and_backward_replay_from_a_captured_graph(B, Bsz, N, H):
    """Once a shape's plan exists the calls only enqueue kernels, so they can be captured in a HIP graph: the
    graph is replayed on fresh inputs, with eager work and synchronisations in between, and every replay must
    equal the eager call on the same inputs bit for bit (the second shape takes the split launch and its merge)."""
    import torch
    from paper_2403_09195_amd import synth
    branches = [(N // 4, 1), (N // 2, 2), (N, 4)]
    mk = lambda seed: make_qkv(seed, Bsz, N, H, 64, "bf16")[0]
    q, k, v = mk(900)
    g = to_device(synth.tensor(900, 7, (Bsz, N, H, 64), "bf16")[0])
    out, lse = B.forward(q, k, v, branches, 0.125)                     # builds the plan
    dq, dk, dv = B.backward(q, k, v, out, lse, g, branches, 0.125)
    need = B.workspace_bytes(Bsz, H, N, 64, B.DFA_BF16, branches)
    assert (need > 0) == (Bsz == 1)
    ws = torch.empty((max(need, 16),), dtype=torch.uint8, device="cuda")   # the caller's workspace: allocated before the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.forward(q, k, v, branches, 0.125, out=out, lse=lse, workspace=ws)
        grads = B.backward(q, k, v, out, lse, g, branches, 0.125)
    for rep in range(3):
        nq, nk, nv = mk(901 + rep)
        q.copy_(nq); k.copy_(nk); v.copy_(nv)
        out.zero_(); lse.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        e_out, e_lse = B.forward(nq, nk, nv, branches, 0.125)
        e_grads = B.backward(nq, nk, nv, e_out, e_lse, g, branches, 0.125)
        torch.cuda.synchronize()
        assert bool((out == e_out).all()) and bool((lse == e_lse).all()), rep
        for a, b in zip(grads, e_grads):
            assert bool((a == b).all()), rep


def test_bf16_reads_packed_qkv_through_strides(B, oracle):
    import torch
    from paper_2403_09195_amd import synth
    Bsz, N, H, D = 2, 512, 3, 64
    branches = [(128, 1), (256, 2), (512, 4)]
    st, ex = synth.tensor(106, 3, (Bsz, N, 3, H, D), "bf16")
    packed = to_device(st)
    out, lse = B.forward(packed[:, :, 0], packed[:, :, 1], packed[:, :, 2], branches, 0.125)
    o_ref, l_ref = oracle.forward(ex[:, :, 0], ex[:, :, 1], ex[:, :, 2], branches, 0.125)
    _check_bf16(out, lse, o_ref, l_ref, "bf16 packed qkv", rows=(oracle, (ex[:, :, 0], ex[:, :, 1], ex[:, :, 2]), branches, 0.125, None))


def test_bf16_sam_scale_config_full(B, oracle):
    from paper_2403_09195_amd import synth
    c = synth.CONFIGS["sam"]
    (q, k, v), ex = make_qkv(c["seed"], c["B"], c["N"], c["H"], c["D"], "bf16")
    out, lse = B.forward(q, k, v, c["branches"], 0.125)
    o_ref, l_ref = oracle.forward(*ex, c["branches"], 0.125)
    _check_bf16(out, lse, o_ref, l_ref, "sam-scale B=1", rows=(oracle, ex, c["branches"], 0.125, None))


@pytest.mark.parametrize("name", ["throughput", "highres"])
def test_bf16_full_size_configs_element_by_element(B, oracle, name):
    """The full-size launches (the first is the one the benchmark times) against the oracle on the same inputs,
    every element of out and lse: the oracle needs a few seconds for them on the machine's host cores."""
    from paper_2403_09195_amd import synth
    c = synth.CONFIGS[name]
    (q, k, v), ex = make_qkv(c["seed"], c["B"], c["N"], c["H"], c["D"], "bf16")
    out, lse = B.forward(q, k, v, c["branches"], 0.125)
    o_ref, l_ref = oracle.forward(*ex, c["branches"], 0.125)
    _check_bf16(out, lse, o_ref, l_ref, f"{name}, every element", rows=(oracle, ex, c["branches"], 0.125, None))


def _branch_membership(N, H, branches):
    """kept[x][h, n]: branch x keeps row n of head h (offset h mod r); seg[x][n]: its segment of that branch."""
    n = np.arange(N)
    kept = [np.stack([(n % w) % r == h % r for h in range(H)]) for (w, r) in branches]
    seg = [n // w for (w, r) in branches]
    return kept, seg


def test_bf16_full_size_zero_queries_closed_form_on_every_row(B):
    """Every row of the full-size launch, not a sample: with q = 0 all numerators of a row are equal, so lse is
    the logarithm of the row's key count (each key once per branch that pairs it with the row) and out the
    mean of those V rows - both computed here in numpy from segment sums, without the oracle."""
    import torch
    from paper_2403_09195_amd import synth
    c = synth.CONFIGS["throughput"]
    Bsz, N, H, D, branches = c["B"], c["N"], c["H"], c["D"], c["branches"]
    (q, k, v), ex = make_qkv(c["seed"], Bsz, N, H, D, "bf16")
    out, lse = B.forward(torch.zeros_like(q), k, v, branches, 0.125)
    vv = ex[2]                                                   # [B, N, H, D] fp64
    kept, seg = _branch_membership(N, H, branches)
    num = np.zeros((Bsz, N, H, D))
    cnt = np.zeros((H, N))
    for x, (w, r) in enumerate(branches):
        for h in range(H):
            m = kept[x][h]
            sums = np.add.reduceat(np.where(m[None, :, None], vv[:, :, h, :], 0.0), np.arange(0, N, w), axis=1)
            num[:, m, h, :] += sums[:, seg[x][m], :]
            cnt[h, m] += w // r
    ref = num / cnt.T[None, :, :, None]
    got, got_l = to_f64(out), to_f64(lse)
    # Rows of one branch: every numerator is exactly 1.  Rows of several branches: numerators m / m_max for keys
    # held by m branches (1/3, 2/3, 1), and equal numerators all round the same way - the correlated case of
    # the bound behind BF16_LSE (1.5e-3 here).
    l_err = np.abs(got_l - np.log(cnt)[None])
    one_branch = np.broadcast_to((cnt == branches[0][0] // branches[0][1])[None], l_err.shape)
    assert l_err[one_branch].max() <= 1e-5 and l_err.max() <= BF16_LSE
    d = np.abs(got - ref)
    print(f"[zero q, every row] out max-abs {d.max():.3e} mean-abs {d.mean():.3e}", flush=True)
    assert d.max() <= BF16_MAX and d.mean() <= BF16_MEAN


@pytest.mark.parametrize("name", ["throughput", "highres"])
def test_bf16_full_size_constant_v_comes_back_exactly(B, name):
    """out is the weighted mean of V rows under the weights the kernel actually uses (the denominator is the sum
    of the same rounded numerators that enter the second product), so a V whose rows are all one vector of
    bf16 values must come back as exactly that vector on every row, whatever q and k are."""
    import torch
    from paper_2403_09195_amd import synth
    c = synth.CONFIGS[name]
    Bsz, N, H, D, branches = c["B"], c["N"], c["H"], c["D"], c["branches"]
    (q, k, v), _ = make_qkv(c["seed"], Bsz, N, H, D, "bf16")
    row = v[0, 0].clone()                                        # [H, D]: one vector per head
    vc = row[None, None].expand(Bsz, N, H, D).contiguous()
    out, _ = B.forward(q, k, vc, branches, 0.125)
    assert bool((out == vc).all())


@pytest.mark.parametrize("name,b_t,t", [("throughput", 3, 1234), ("highres", 1, 9000)])
def test_bf16_full_size_locality_on_every_row(B, name, b_t, t):
    """Changing the K and V rows of one token changes exactly the rows that hold that token as a key (same
    segment of a branch that keeps both, Eq. 1) and leaves every other row of the full-size launch as it was,
    bit for bit: a gather that reached outside a row's key lists, or missed a part of them, shows here."""
    import torch
    from paper_2403_09195_amd import synth
    c = synth.CONFIGS[name]
    Bsz, N, H, D, branches = c["B"], c["N"], c["H"], c["D"], c["branches"]
    (q, k, v), _ = make_qkv(c["seed"], Bsz, N, H, D, "bf16")
    out0, lse0 = B.forward(q, k, v, branches, 0.125)
    k2, v2 = k.clone(), v.clone()
    k2[b_t, t] = -k[b_t, t]
    v2[b_t, t] = v[b_t, t] + 1.0
    out1, lse1 = B.forward(q, k2, v2, branches, 0.125)
    torch.cuda.synchronize()
    kept, seg = _branch_membership(N, H, branches)
    touched = np.zeros((H, N), dtype=bool)
    for x in range(len(branches)):
        for h in range(H):
            if kept[x][h][t]:
                touched[h] |= kept[x][h] & (seg[x] == seg[x][t])
    changed = ((out0 != out1).any(dim=-1).permute(0, 2, 1) | (lse0 != lse1)).cpu().numpy()      # [B, H, N]
    expect = np.zeros((Bsz, H, N), dtype=bool)
    expect[b_t] = touched
    assert not (changed & ~expect).any()
    assert changed[expect].mean() >= 0.99
    print(f"[locality {name}] rows holding the token: {int(expect.sum())}, changed: {int(changed.sum())}", flush=True)


# ---------------------------------------------------------------- stage entry points
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_unmerged_branches_and_standalone_merge(B, oracle, dtype):
    import torch
    Bsz, N, H, D = 2, 512, 3, 64
    branches = [(128, 1), (256, 2), (512, 4)]
    (q, k, v), ex = make_qkv(107, Bsz, N, H, D, dtype)
    o_ref, l_ref, bo_ref, bl_ref = oracle.forward(*ex, branches, 0.125, return_branches=True)
    outs, lses = [], []
    for x, (w, r) in enumerate(branches):
        ob, lb = B.forward_branch(q, k, v, w, r, 0.125)
        assert ob.dtype == torch.float32
        mx, mean = error_stats(to_f64(ob), bo_ref[x])
        if dtype == "bf16":
            check_lse_bf16(to_f64(lb), oracle, ex, [(w, r)], 0.125, bl_ref[x])
        else:
            check_lse(to_f64(lb), bl_ref[x], atol=1e-5, rtol=1e-5)
        assert mx <= (BF16_MAX if dtype == "bf16" else F32_MAX)
        dead = np.isneginf(bl_ref[x]).transpose(0, 2, 1)
        assert np.all(to_f64(ob)[dead] == 0.0)
        outs.append(ob)
        lses.append(lb)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    out, lse = B.merge(torch.stack(outs), torch.stack(lses), tdt)
    if dtype == "bf16":
        _check_bf16(out, lse, o_ref, l_ref, "branch+merge bf16", rows=(oracle, ex, branches, 0.125, None))
    else:
        _check_f32(out, lse, o_ref, l_ref, "branch+merge f32")
    # the merge kernel alone, on the oracle's own fp64 branch results rounded to fp32
    ob32 = torch.from_numpy(bo_ref.astype(np.float32)).cuda()
    lb32 = torch.from_numpy(bl_ref.astype(np.float32)).cuda()
    out_m, lse_m = B.merge(ob32, lb32, torch.float32)
    mx, _ = error_stats(to_f64(out_m), o_ref)
    check_lse(to_f64(lse_m), l_ref, atol=1e-5, rtol=1e-5)
    assert mx <= F32_MAX


def test_bf16_tensors_beyond_two_gigabytes(B):
    """344 images: every tensor passes 2^31 bytes, so any 32-bit byte or element offset in the kernels
    or the plan would show.  The first, a middle and the last pair of images must come out bit for bit as
    when the pair is run on its own (each tile's arithmetic does not depend on the launch around it; a
    pair, because a single image is a launch of few workgroups, which takes the split path); the same
    for the gradients."""
    import torch
    Bsz, N, H, D = 344, 4096, 12, 64
    branches = [(1024, 1), (2048, 2), (4096, 4)]
    gen = torch.Generator(device="cuda").manual_seed(9)
    q, k, v, g = (torch.randn((Bsz, N, H, D), device="cuda", dtype=torch.float32, generator=gen).bfloat16()
                  for _ in range(4))
    assert q.numel() * 2 > 2 ** 31
    out, lse = B.forward(q, k, v, branches, 0.125)
    dq, dk, dv = B.backward(q, k, v, out, lse, g, branches, 0.125)
    torch.cuda.synchronize()
    for b in (0, 171, Bsz - 2):
        sl = slice(b, b + 2)
        o1, l1 = B.forward(q[sl], k[sl], v[sl], branches, 0.125)
        assert bool((o1 == out[sl]).all()) and bool((l1 == lse[sl]).all()), b
        g1 = B.backward(q[sl], k[sl], v[sl], o1, l1, g[sl].contiguous(), branches, 0.125)
        for got, full in zip(g1, (dq, dk, dv)):
            assert bool((got == full[sl]).all()), b
    assert bool(torch.isfinite(out[-1].float()).all())


def test_mfma_only_loop_reports_a_plausible_ceiling(B):
    for random_operands in (False, True):
        tflops, mhz = B.mfma_peak(random_operands)
        assert 800.0 < tflops < 2600.0 and 1000.0 < mhz < 2600.0, (tflops, mhz)
