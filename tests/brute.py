"""Independent float64 re-statements of attention used ONLY to pin the oracle.

Nothing here is shared with ``oracle/`` or with the GPU library.  The head expansion is the
repeat-interleave that the paper's "KV Group Sharing" workaround performs (appendix, official
implementation of KV group sharing): every K (V) head is duplicated n_q/n_k (n_q/n_v) times in
place, after which each query head has a K and a V of its own and ordinary multi-head attention
applies.
"""
import numpy as np


def bf16_bits_to_f64(a):
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def expand_heads(x, n_rep):
    """[B, n, T, d] -> [B, n*n_rep, T, d], each head repeated n_rep times consecutively."""
    B, n, T, d = x.shape
    return np.broadcast_to(x[:, :, None, :, :], (B, n, n_rep, T, d)).reshape(B, n * n_rep, T, d)


def mha_decode(q, k, v, scale):
    """q [B,H,d], k [B,H,T,d], v [B,H,T,dv] -> o [B,H,dv], lse [B,H]; one head each, einsum."""
    s = np.einsum("bhc,bhjc->bhj", q, k) * scale
    m = s.max(axis=-1, keepdims=True)
    p = np.exp(s - m)
    l = p.sum(axis=-1, keepdims=True)
    o = np.einsum("bhj,bhje->bhe", p / l, v)
    return o, (m + np.log(l))[..., 0]


def diffqkv_decode_by_expansion(q, k, v, scale, seqlens=None):
    q, k, v = bf16_bits_to_f64(q), bf16_bits_to_f64(k), bf16_bits_to_f64(v)
    B, n_q, _ = q.shape
    n_k, n_v = k.shape[1], v.shape[1]
    ke, ve = expand_heads(k, n_q // n_k), expand_heads(v, n_q // n_v)
    if seqlens is None:
        return mha_decode(q, ke, ve, scale)
    outs, lses = [], []
    for b in range(B):
        t = int(seqlens[b])
        o, l = mha_decode(q[b : b + 1], ke[b : b + 1, :, :t], ve[b : b + 1, :, :t], scale)
        outs.append(o)
        lses.append(l)
    return np.concatenate(outs), np.concatenate(lses)


def enumerate_decode(q, k, v, scale):
    """Pure-Python loops with explicit integer head indices (tiny shapes only)."""
    import math

    q, k, v = bf16_bits_to_f64(q), bf16_bits_to_f64(k), bf16_bits_to_f64(v)
    B, n_q, d = q.shape
    n_k, T = k.shape[1], k.shape[2]
    n_v, dv = v.shape[1], v.shape[3]
    out = np.zeros((B, n_q, dv))
    for b in range(B):
        for h in range(n_q):
            kh = h // (n_q // n_k)
            vh = h // (n_q // n_v)
            scores = [scale * sum(q[b, h, c] * k[b, kh, j, c] for c in range(d)) for j in range(T)]
            z = sum(math.exp(x) for x in scores)
            for e in range(dv):
                out[b, h, e] = sum(math.exp(scores[j]) / z * v[b, vh, j, e] for j in range(T))
    return out


def gather_paged(pool, block_table, seqlens, T_cap):
    """[n_pages, n, P, d] pool -> contiguous [B, n, T_cap, d] (zeros beyond each T_b)."""
    n_pages, n, P, d = pool.shape
    B = block_table.shape[0]
    out = np.zeros((B, n, T_cap, d), dtype=pool.dtype)
    for b in range(B):
        for j in range(int(seqlens[b])):
            out[b, :, j, :] = pool[block_table[b, j // P], :, j % P, :]
    return out
