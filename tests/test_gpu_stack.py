"""GPU parity of the projections and of the encoder attention stack (QKV projection, dilated
attention, output projection per layer) against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest

from gpu_util import error_stats, to_device, to_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2403_09195_amd import binding
    binding.lib()
    return binding


def _bf16(seed, tid, shape, std=1.0):
    from paper_2403_09195_amd import synth
    bits, exact = synth.tensor(seed, tid, shape, "bf16", std=std)
    return to_device(bits), exact


def _linear_bar(x_exact, w_exact, y_ref):
    """Error bar of one bf16 projection with fp32 accumulation: the result is rounded once to
    bf16 (half an ulp, at most 2^-8 relative, reached just above a power of two) and the fp32 sum of
    K products is off by at most K * 2^-24 * sum |x_k w_k| (far less in practice)."""
    K = x_exact.shape[-1]
    mag = np.matmul(np.abs(x_exact), np.abs(w_exact).T)
    return 2.0 ** -8 * np.abs(y_ref) + K * 2.0 ** -24 * mag + 1e-30


# (36864, 1024) is large enough for the 256-feature tile to be chosen; (28672, 2048) has 112 such tiles per die,
# three full rounds and a half-full one, whose 16 tiles are cut into 128-feature halves; the others run the
# 128-feature tile throughout
@pytest.mark.parametrize("M,N,K", [(256, 128, 64), (512, 256, 128), (768, 384, 192), (1024, 2304, 768), (512, 768, 768),
                                   (36864, 1024, 128), (28672, 2048, 64)])
def test_linear_against_fp64_matmul(B, oracle, M, N, K):
    x, xe = _bf16(401, 3, (M, K))
    w, we = _bf16(401, 10, (N, K), std=0.02)
    y = B.linear(x, w)
    ref = oracle.linear(xe, we)
    err = np.abs(to_f64(y) - ref)
    bar = _linear_bar(xe, we, ref)
    print(f"[linear {M}x{N}x{K}] max err {err.max():.3e}, worst err/bar {float((err / bar).max()):.3f}", flush=True)
    assert np.all(err <= bar)


def test_linear_identity_and_row_selection(B):
    """w = I copies x bit for bit; a weight matrix with a single 1 per row permutes features: any
    wrong row, column or k mapping in the tiling shows as a misplaced element."""
    import torch
    M, K = 512, 256
    x, _ = _bf16(402, 3, (M, K))
    eye = torch.eye(K, dtype=torch.bfloat16, device="cuda")
    assert bool((B.linear(x, eye) == x).all())
    perm = torch.randperm(K, generator=torch.Generator().manual_seed(5)).cuda()
    y = B.linear(x, eye[perm])                     # output feature n reads input feature perm[n]
    assert bool((y == x[:, perm]).all())
    # a strided weight view (rows of a wider matrix) and a preallocated output
    wide = torch.zeros((K, 2 * K), dtype=torch.bfloat16, device="cuda")
    wide[:, :K] = eye[perm]
    out = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    assert B.linear(x, wide[:, :K], out=out) is out and bool((out == x[:, perm]).all())


def test_linear_rejects_bad_shapes(B):
    import torch
    x = torch.zeros((256, 64), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((128, 64), dtype=torch.bfloat16, device="cuda")
    B.linear(x, w)
    for bad_x, bad_w in ((torch.zeros((384, 64), dtype=torch.bfloat16, device="cuda"), w),
                         (x, torch.zeros((100, 64), dtype=torch.bfloat16, device="cuda")),
                         (torch.zeros((256, 96), dtype=torch.bfloat16, device="cuda"),
                          torch.zeros((128, 96), dtype=torch.bfloat16, device="cuda"))):
        with pytest.raises(B.DfaError) as e:
            B.linear(bad_x, bad_w)
        assert e.value.code == -2


def _stack_inputs(seed, Bsz, N, H, D, layers):
    E = H * D
    x, xe = _bf16(seed, 3, (Bsz, N, E))
    wq, wqe, wo, woe = [], [], [], []
    for l in range(layers):
        a, ae = _bf16(seed, 10 + 2 * l, (3 * E, E), std=0.02)
        b, be = _bf16(seed, 11 + 2 * l, (E, E), std=0.02)
        wq.append(a); wqe.append(ae); wo.append(b); woe.append(be)
    import torch
    return x, xe, torch.stack(wq), np.stack(wqe), torch.stack(wo), np.stack(woe)


def _rel(got, ref):
    """max-abs and mean-abs error relative to the RMS of the reference (activations shrink from
    layer to layer in this stack, which has no residual or normalisation, so absolute bars mean nothing)."""
    rms = float(np.sqrt(np.mean(ref ** 2)))
    d = np.abs(got - ref)
    return float(d.max()) / rms, float(d.mean()) / rms


@pytest.mark.parametrize("Bsz,N,H,branches", [
    (2, 512, 4, [(128, 1), (256, 2), (512, 4)]),
    (8, 4096, 12, [(1024, 1), (2048, 2), (4096, 4)]),        # a layer of the stack workload at its full size
])
def test_one_layer_each_step_against_the_oracle(B, oracle, Bsz, N, H, branches):
    """One layer, checked step by step, every element: the oracle is fed the GPU's own (bf16) input of each
    step, so every step is held to its own bar: projections to the rounding bar above, attention to the
    operator's bars scaled by the size of its values."""
    D = 64
    E = H * D
    x, xe, wq, wqe, wo, woe = _stack_inputs(410, Bsz, N, H, D, 1)
    y, qkv, attn = B.encoder_stack(x, wq, wo, H, branches, 0.125)
    qkv_g, attn_g, y_g = to_f64(qkv), to_f64(attn), to_f64(y)
    # step 1: QKV projection
    ref = oracle.linear(xe, wqe[0]).reshape(Bsz, N, 3, H, D)
    assert np.all(np.abs(qkv_g - ref) <= _linear_bar(xe, wqe[0], ref.reshape(Bsz, N, 3 * E)).reshape(ref.shape))
    # step 2: attention on the GPU's qkv; values are ~ v / sqrt(keys), so the bars scale with the value RMS
    a_ref, _ = oracle.forward(qkv_g[:, :, 0], qkv_g[:, :, 1], qkv_g[:, :, 2], branches, 0.125)
    mx, mean = _rel(attn_g, a_ref)
    print(f"[layer] attention rel max {mx:.3e} mean {mean:.3e}", flush=True)
    assert mx <= 2e-2 and mean <= 2e-3
    # step 3: output projection on the GPU's attention output
    ae = attn_g.reshape(Bsz, N, E)
    ref = oracle.linear(ae, woe[0])
    assert np.all(np.abs(y_g - ref) <= _linear_bar(ae, woe[0], ref))
    # and the whole layer against the oracle's unrounded layer
    y_ref, _, _ = oracle.attention_layer(xe, wqe[0], woe[0], H, branches, 0.125)
    mx, mean = _rel(y_g, y_ref)
    print(f"[layer] whole layer rel max {mx:.3e} mean {mean:.3e}", flush=True)
    assert mx <= 5e-2 and mean <= 5e-3


def test_three_layer_stack_end_to_end(B, oracle):
    """Three layers end to end against the unrounded oracle: the drift of three bf16 roundings per
    layer, reported relative to the RMS of the result and held to a loose bar; the workspace
    variant must give the same bits."""
    import torch
    Bsz, N, H, D, layers = 1, 512, 2, 64, 3
    E = H * D
    branches = [(256, 1), (512, 2)]
    x, xe, wq, wqe, wo, woe = _stack_inputs(411, Bsz, N, H, D, layers)
    y, qkv, attn = B.encoder_stack(x, wq, wo, H, branches, 0.125)
    ref = xe
    for l in range(layers):
        ref, _, _ = oracle.attention_layer(ref, wqe[l], woe[l], H, branches, 0.125)
    mx, mean = _rel(to_f64(y), ref)
    print(f"[stack x{layers}] rel max {mx:.3e} mean {mean:.3e}, result rms {np.sqrt(np.mean(ref ** 2)):.3e}", flush=True)
    assert mx <= 0.15 and mean <= 2e-2
    ws = (torch.empty_like(qkv), torch.empty_like(attn), torch.empty_like(y))
    y2, _, _ = B.encoder_stack(x, wq, wo, H, branches, 0.125, buffers=ws)
    assert y2 is ws[2] and bool((y2 == y).all())


def test_full_size_layer_with_identity_projections_is_the_operator(B):
    """The stack workload's shapes (8 images, 4096 tokens, 12 heads): with W_qkv = [I; I; I] and W_o = I the
    projections copy their input exactly (one product by 1 per output, the rest by 0), so the layer must equal
    dfa_forward on x taken as q, k and v, bit for bit - the packed, strided q / k / v views and the [B, N, H*D]
    hand-over between the three launches, at the size the benchmark runs."""
    import torch
    from paper_2403_09195_amd import synth
    c = synth.CONFIGS["stack_layer"]
    Bsz, N, H, D, branches = c["B"], c["N"], c["H"], c["D"], c["branches"]
    E = H * D
    x = to_device(synth.tensor(c["seed"], 3, (Bsz, N, E), "bf16")[0])
    eye = torch.eye(E, dtype=torch.bfloat16, device=x.device)
    wq = torch.cat([eye, eye, eye], dim=0)[None].contiguous()
    wo = eye[None].contiguous()
    y, qkv, attn = B.encoder_stack(x, wq, wo, H, branches, 0.125)
    xh = x.view(Bsz, N, H, D)
    out, _ = B.forward(xh, xh, xh, branches, 0.125)
    torch.cuda.synchronize()
    for t in range(3):
        assert bool((qkv[:, :, t] == xh).all())
    assert bool((attn == out).all())
    assert bool((y.view(Bsz, N, H, D) == out).all())
