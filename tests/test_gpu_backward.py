"""GPU parity of the backward entry point against the fp64 oracle (itself pinned by central
differences of the forward).  The GPU backward is given the GPU forward's own out and lse."""
import numpy as np
import pytest

import helpers
from gpu_util import make_qkv, to_device, to_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2403_09195_amd import binding
    binding.lib()
    return binding


def _dout(seed, shape, dtype):
    from paper_2403_09195_amd import synth
    st, ex = synth.tensor(seed, 7, shape, dtype)
    return to_device(st), ex


def _report(tag, got, ref):
    """Returns (worst excess over the final bf16 rounding, mean-abs error), both relative to the rms."""
    rms = float(np.sqrt(np.mean(ref ** 2)))
    d = np.abs(got - ref)
    excess = float((d - 2.0 ** -8 * np.abs(ref)).max())
    print(f"[{tag}] max-abs {d.max():.3e} mean-abs {d.mean():.3e} (gradient rms {rms:.3e}), "
          f"beyond the result's own rounding {excess:.3e}", flush=True)
    return excess / rms, float(d.mean()) / rms


CASES = [
    (2, 256, 3, [(64, 2)], None),                                   # uncovered rows
    (1, 512, 4, [(128, 1), (256, 2), (512, 4)], None),              # the workload's branch pattern, scaled down
    (2, 300, 2, [(100, 3), (77, 1), (512, 5)], [[2, 0], [0, 0], [4, 1]]),   # ragged parts, explicit offsets
    (1, 768, 2, [(192, 2), (384, 3), (768, 1), (768, 1)], None),            # shared keys of multiplicity up to 4
]


@pytest.mark.parametrize("Bsz,N,H,branches,offs", CASES)
def test_backward_fp32(B, oracle, Bsz, N, H, branches, offs):
    """fp32 path: sums of up to a few thousand fp32 products per gradient element; held to 2e-5 of the
    largest gradient magnitude (measured about 1e-6)."""
    (q, k, v), ex = make_qkv(500 + N, Bsz, N, H, 64, "f32")
    g, ge = _dout(500 + N, (Bsz, N, H, 64), "f32")
    out, lse = B.forward(q, k, v, branches, 0.125, head_offsets=offs)
    dq, dk, dv = B.backward(q, k, v, out, lse, g, branches, 0.125, head_offsets=offs)
    rq, rk, rv = oracle.backward(*ex, ge, branches, 0.125, head_offsets=offs)
    for name, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        err = np.abs(to_f64(got) - ref)
        print(f"[f32 {name}] max-abs {err.max():.3e}, largest gradient {np.abs(ref).max():.3e}", flush=True)
        assert err.max() <= 2e-5 * max(1.0, np.abs(ref).max())
    _, l_ref = oracle.forward(*ex, branches, 0.125, head_offsets=offs)
    dead = np.isneginf(l_ref).transpose(0, 2, 1)
    for got in (dq, dk, dv):
        assert np.all(to_f64(got)[dead] == 0.0)


@pytest.mark.parametrize("Bsz,N,H,branches,offs", CASES)
def test_backward_bf16(B, oracle, Bsz, N, H, branches, offs):
    """bf16 path (matrix cores): P and dS are rounded to bf16 before their second products, as the
    forward rounds P (each term off by up to 2^-9 of itself, random in sign), delta = dout . out is
    taken from the bf16-rounded forward output, and every gradient is rounded to bf16 (up to 2^-8 of
    its own size).  Bar, the forward's figures taken relative to the gradient's rms:
    |err| <= 2^-8 |g| + 3e-2 rms(g) per element (the largest of some 10^5 random rounding errors whose
    typical size is 1.5e-3 rms(g): the measured worst is 2.1e-2), mean-abs <= 2e-3 rms(g)."""
    (q, k, v), ex = make_qkv(600 + N, Bsz, N, H, 64, "bf16")
    g, ge = _dout(600 + N, (Bsz, N, H, 64), "bf16")
    out, lse = B.forward(q, k, v, branches, 0.125, head_offsets=offs)
    dq, dk, dv = B.backward(q, k, v, out, lse, g, branches, 0.125, head_offsets=offs)
    rq, rk, rv = oracle.backward(*ex, ge, branches, 0.125, head_offsets=offs)
    for name, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        mx, mean = _report(f"bf16 {name}", to_f64(got), ref)
        assert mx <= 3e-2 and mean <= 2e-3


def test_backward_reads_strided_inputs_and_rejects_bad_arguments(B, oracle):
    import torch
    from paper_2403_09195_amd import synth
    Bsz, N, H, D = 1, 256, 2, 64
    branches = [(128, 1), (256, 2)]
    st, ex = synth.tensor(701, 3, (Bsz, N, 3, H, D), "f32")
    packed = to_device(st)
    q, k, v = packed[:, :, 0], packed[:, :, 1], packed[:, :, 2]
    g, ge = _dout(701, (Bsz, N, H, D), "f32")
    out, lse = B.forward(q, k, v, branches, 0.125)
    dq, dk, dv = B.backward(q, k, v, out, lse, g, branches, 0.125)
    rq, rk, rv = oracle.backward(ex[:, :, 0], ex[:, :, 1], ex[:, :, 2], ge, branches, 0.125)
    for got, ref in ((dq, rq), (dk, rk), (dv, rv)):
        assert np.abs(to_f64(got) - ref).max() <= 2e-5 * max(1.0, np.abs(ref).max())
    with pytest.raises(B.DfaError) as e:
        B.backward(q, k, v, out, lse, g, [(128, 0)], 0.125)
    assert e.value.code == -2
    with pytest.raises(TypeError):
        B.backward(q, k, v, out.bfloat16(), lse, g, branches, 0.125)


def test_backward_bf16_sam_scale_config(B, oracle):
    """The SAM-scale workload (one 1024^2 image, 12 heads, three branches) in full."""
    from paper_2403_09195_amd import synth
    c = synth.CONFIGS["sam"]
    (q, k, v), ex = make_qkv(c["seed"], c["B"], c["N"], c["H"], c["D"], "bf16")
    g, ge = _dout(c["seed"], (c["B"], c["N"], c["H"], c["D"]), "bf16")
    out, lse = B.forward(q, k, v, c["branches"], 0.125)
    dq, dk, dv = B.backward(q, k, v, out, lse, g, c["branches"], 0.125)
    rq, rk, rv = oracle.backward(*ex, ge, c["branches"], 0.125)
    for name, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        mx, mean = _report(f"sam bf16 {name}", to_f64(got), ref)
        assert mx <= 3e-2 and mean <= 2e-3


def test_backward_bf16_full_size_element_by_element(B, oracle):
    """The launch the backward benchmark times (16 images, 12 heads, 4096 tokens) against the oracle on the same
    inputs, every element of the three gradients (the oracle needs some ten seconds on the machine's host cores)."""
    import torch
    from paper_2403_09195_amd import synth
    c = synth.CONFIGS["throughput"]
    (q, k, v), ex = make_qkv(c["seed"], c["B"], c["N"], c["H"], c["D"], "bf16")
    g, ge = _dout(c["seed"], (c["B"], c["N"], c["H"], c["D"]), "bf16")
    out, lse = B.forward(q, k, v, c["branches"], 0.125)
    dq, dk, dv = B.backward(q, k, v, out, lse, g, c["branches"], 0.125)
    torch.cuda.synchronize()
    refs = oracle.backward(*ex, ge, c["branches"], 0.125)
    got = [to_f64(t) for t in (dq, dk, dv)]
    # Three (b, h) units through the chain rule written with dense matrices in numpy (independent of oracle and
    # kernels): the size of the terms every gradient element is a sum of.
    units = [(0, 0), (7, 5), (15, 11)]
    eps = 2.0 ** -9
    spread = []                                       # per tensor: largest / rms of the root-sum-of-squares of an element's terms
    for (b, h) in units:
        sl = tuple(np.ascontiguousarray(a[b:b + 1, :, h:h + 1]) for a in ex)
        offs = [[h % r] for (_, r) in c["branches"]]
        dense = helpers.multiset_attention_backward(*sl, np.ascontiguousarray(ge[b:b + 1, :, h:h + 1]), 0.125, c["branches"], offs,
                                                    want_sq=True)
        for i, name in enumerate(("dq", "dk", "dv")):
            ref_u, abs_u, sq_u = refs[i][b, :, h], dense[3 + i][0, :, 0], dense[6 + i][0, :, 0]
            assert np.abs(dense[i][0, :, 0] - ref_u).max() <= 1e-9 * max(1.0, np.abs(ref_u).max())   # same gradients as the oracle's
            # every element of the unit: off by no more than its own bf16 rounding and what roundings of 2^-9 in P, dS,
            # the forward output inside delta and the result add up to over the terms at worst
            d = np.abs(got[i][b, :, h] - ref_u)
            assert np.all(d <= 2.0 ** -8 * np.abs(ref_u) + 4 * eps * abs_u), (name, b, h)
            spread.append((name, float(sq_u.max() / np.sqrt(np.mean(sq_u ** 2)))))
    for i, name in enumerate(("dq", "dk", "dv")):
        mx, mean = _report(f"throughput, every element, {name}", got[i], refs[i])
        # Every element of the launch.  The mean error is held to 2e-3 of the gradient's rms, as in the small cases.
        # The largest of the n = 5 * 10^7 errors of a tensor: an error is a sum of many independent roundings, so it
        # is normal with a standard deviation proportional to the root-sum-of-squares of the element's terms;
        # the rms error over the tensor is at most 1.25 x the mean bar (normal: rms = 1.2533 x mean-abs), the
        # element with the largest terms stands `rho` above the rms (taken from the dense chain rule on the three
        # units above, with a quarter on top for the units not looked at), and the largest of n normal draws is
        # sqrt(2 ln 2n) standard deviations out.
        rho = 1.25 * max(r for nm, r in spread if nm == name)
        z = float(np.sqrt(2.0 * np.log(2.0 * refs[i].size)))
        bar = z * rho * 1.2533 * 2e-3
        print(f"[throughput, {name}] largest error beyond the result's rounding {mx:.3e} of the rms; bar {bar:.3e} "
              f"(z = {z:.2f}, rho = {rho:.2f})", flush=True)
        assert mean <= 2e-3 and mx <= bar


def test_backward_bf16_full_size_locality_on_every_row(B):
    """Changing dout of one token changes dq of that token only, and dk / dv of exactly the tokens it holds as
    keys (same segment of a branch that keeps both, Eq. 1); every other row of the three full-size gradients
    stays as it was, bit for bit."""
    import torch
    from paper_2403_09195_amd import synth
    c = synth.CONFIGS["throughput"]
    Bsz, N, H, D, branches = c["B"], c["N"], c["H"], c["D"], c["branches"]
    (q, k, v), _ = make_qkv(c["seed"], Bsz, N, H, D, "bf16")
    g, _ = _dout(c["seed"], (Bsz, N, H, D), "bf16")
    out, lse = B.forward(q, k, v, branches, 0.125)
    first = [x.clone() for x in B.backward(q, k, v, out, lse, g, branches, 0.125)]
    b_t, t = 5, 2049
    g2 = g.clone()
    g2[b_t, t] = -g[b_t, t] + 0.5
    second = B.backward(q, k, v, out, lse, g2, branches, 0.125)
    torch.cuda.synchronize()
    n = np.arange(N)
    keys_of_t = np.zeros((H, N), dtype=bool)
    for (w, r) in branches:
        for h in range(H):
            kept = (n % w) % r == h % r
            if kept[t]:
                keys_of_t[h] |= kept & (n // w == t // w)
    changed = [(a != b).any(dim=-1).permute(0, 2, 1).cpu().numpy() for a, b in zip(first, second)]   # [B, H, N] each
    only_t = np.zeros((Bsz, H, N), dtype=bool)
    only_t[b_t, :, t] = True
    keys = np.zeros((Bsz, H, N), dtype=bool)
    keys[b_t] = keys_of_t
    assert np.array_equal(changed[0], only_t)
    for name, ch in zip(("dk", "dv"), changed[1:]):
        assert not (ch & ~keys).any(), name
        assert ch[keys].mean() >= 0.99, name
    print(f"[backward locality] keys of the token: {int(keys.sum())}; dk rows changed {int(changed[1].sum())}, "
          f"dv rows changed {int(changed[2].sum())}", flush=True)


@pytest.mark.parametrize("count", [1, 31, 33, 64, 65, 129])
def test_backward_bf16_list_lengths_around_the_block_sizes(B, oracle, count):
    """Lists of `count` rows: one row (P = 1, dq = dk = 0, dv = dout), and lengths just below, at and
    above the 32-row block and the 64-row stage the kernels walk in."""
    w, r = 2 * count, 2
    N, H = 3 * w, 2
    branches = [(w, r), (N, 1)]
    (q, k, v), ex = make_qkv(800 + count, 1, N, H, 64, "bf16")
    g, ge = _dout(800 + count, (1, N, H, 64), "bf16")
    for br in (branches[:1], branches):
        out, lse = B.forward(q, k, v, br, 0.125)
        dq, dk, dv = B.backward(q, k, v, out, lse, g, br, 0.125)
        rq, rk, rv = oracle.backward(*ex, ge, br, 0.125)
        for name, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
            # a gradient that is exactly zero (a single row per list: dq = dk = 0) comes out as fp32 round-off
            # of dout . v - dout . out, about 1e-7 of dout's size; the floor stands for that
            rms = max(float(np.sqrt(np.mean(ref ** 2))), 1e-4)
            d = np.abs(to_f64(got) - ref)
            # with a handful of rows per list nothing averages the bf16 roundings of P, dS and the result
            # (2^-9 each): the mean bar is 2^-8 of the rms here instead of the workload's 2e-3
            assert float((d - 2.0 ** -8 * np.abs(ref)).max()) <= 3e-2 * rms and float(d.mean()) <= 2.0 ** -8 * rms, (name, len(br))
