"""Independent numpy references used to pin the oracle (none of them calls the oracle)."""
import numpy as np


def dense_softmax_attention(q, k, v, scale):
    """Textbook softmax(scale * q k^T) v for one head: q,k,v [n, D] -> (out [n, D], lse [n])."""
    s = scale * (q @ k.T)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    l = e.sum(axis=1, keepdims=True)
    return (e / l) @ v, (m + np.log(l))[:, 0]


def multiplicity_matrix(N, h, branches, head_offsets=None):
    """mult[n, j] = number of branches in which query n attends key j (same segment, both kept)."""
    n = np.arange(N)
    mult = np.zeros((N, N), dtype=np.int64)
    for x, (w, r) in enumerate(branches):
        o = (h % r) if head_offsets is None else int(head_offsets[x][h])
        pos = n - (n // w) * w - o                  # position inside the part, counted from the head's start
        kept = (pos >= 0) & (pos % r == 0)
        same_seg = (n[:, None] // w) == (n[None, :] // w)
        mult += (same_seg & kept[:, None] & kept[None, :]).astype(np.int64)
    return mult


def multiset_attention(q, k, v, scale, branches, head_offsets=None):
    """Brute force: softmax attention of every query over the multiset union of its branches' key sets.

    q, k, v [B, N, H, D] fp64 -> (out [B, N, H, D], lse [B, H, N]).  Rows with no key: (0, -inf).
    """
    B, N, H, D = q.shape
    out = np.zeros((B, N, H, D))
    lse = np.full((B, H, N), -np.inf)
    for h in range(H):
        mult = multiplicity_matrix(N, h, branches, head_offsets)
        has = mult.sum(axis=1) > 0
        for b in range(B):
            s = scale * (q[b, :, h] @ k[b, :, h].T)
            with np.errstate(divide="ignore"):
                t = np.where(mult > 0, s + np.log(np.maximum(mult, 1)), -np.inf)
            m = np.where(has, t.max(axis=1), 0.0)
            e = np.exp(t - m[:, None])
            l = e.sum(axis=1)
            o = (e @ v[b, :, h]) / np.where(has, l, 1.0)[:, None]
            out[b, :, h] = np.where(has[:, None], o, 0.0)
            with np.errstate(divide="ignore"):
                lse[b, h] = np.where(has, m + np.log(np.where(has, l, 1.0)), -np.inf)
    return out, lse


def randn(rng, *shape):
    return rng.standard_normal(shape)


def multiset_attention_backward(q, k, v, dout, scale, branches, head_offsets=None, want_sq=False):
    """Chain rule on the multiset softmax, written with dense matrices per (b, h):
      P = mult * exp(scale q k^T - lse),  out = P v,  delta = rowsum(dout * out),  dP = dout v^T,
      dS = P * (dP - delta),  dq = scale dS k,  dk = scale dS^T q,  dv = P^T dout.
    Returns (dq, dk, dv, dq_abs, dk_abs, dv_abs), all [B, N, H, D] fp64.  The *_abs arrays are the same sums
    over absolute values of their terms, with |dP - delta| bounded by |dP| + rowsum(|dout * out|): what a
    rounding error of relative size eps in every term can at most add up to is eps times them.
    want_sq: three more arrays, the root of the sum of the squared terms of every element (what independent
    rounding errors of the terms add up to, in standard deviations per unit of their own)."""
    B, N, H, D = q.shape
    res = [np.zeros((B, N, H, D)) for _ in range(9 if want_sq else 6)]
    for h in range(H):
        mult = multiplicity_matrix(N, h, branches, head_offsets).astype(np.float64)
        has = mult.sum(axis=1) > 0
        for b in range(B):
            qh, kh, vh, gh = q[b, :, h], k[b, :, h], v[b, :, h], dout[b, :, h]
            s = scale * (qh @ kh.T)
            m = np.where(has, np.where(mult > 0, s, -np.inf).max(axis=1, initial=-np.inf), 0.0)
            e = mult * np.exp(np.minimum(s - m[:, None], 700.0) * (mult > 0))
            l = e.sum(axis=1)
            P = e / np.where(has, l, 1.0)[:, None]
            out = P @ vh
            delta = (gh * out).sum(axis=1)
            delta_abs = np.abs(gh * out).sum(axis=1)
            dP = gh @ vh.T
            dS = P * (dP - delta[:, None])
            W = P * (np.abs(dP) + delta_abs[:, None])
            res[0][b, :, h] = scale * (dS @ kh)
            res[1][b, :, h] = scale * (dS.T @ qh)
            res[2][b, :, h] = P.T @ gh
            res[3][b, :, h] = scale * (W @ np.abs(kh))
            res[4][b, :, h] = scale * (W.T @ np.abs(qh))
            res[5][b, :, h] = P.T @ np.abs(gh)
            if want_sq:
                res[6][b, :, h] = scale * np.sqrt((dS ** 2) @ (kh ** 2))
                res[7][b, :, h] = scale * np.sqrt((dS ** 2).T @ (qh ** 2))
                res[8][b, :, h] = np.sqrt((P ** 2).T @ (gh ** 2))
    return tuple(res)
