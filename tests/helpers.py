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
