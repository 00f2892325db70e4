"""Pins for the float64 oracle: checks against things the paper and the mathematics fix, none of
which call back into the oracle's own formula.  CPU only."""
import itertools
import math

import numpy as np
import pytest
import torch

import brute
import oracle
from paper_2501_13629_amd import inputs

TOL = 1e-12


def rnd(shape, seed, dtype=np.float32):
    rng = np.random.default_rng(seed)
    return rng.standard_normal(shape).astype(dtype)


def to_bf16_bits(x):
    return inputs.as_numpy(torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16))


def rel_close(a, b, tol=TOL):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape
    denom = np.maximum(1.0, np.abs(b))
    assert np.max(np.abs(a - b) / denom) <= tol, np.max(np.abs(a - b) / denom)


HEADS = [(4, 1, 2), (8, 2, 4), (6, 3, 6), (6, 2, 1), (8, 8, 8), (4, 1, 1), (12, 2, 6), (8, 4, 2)]


# P1: a context of one token returns V exactly (softmax over one element is 1).
@pytest.mark.parametrize("n_q,n_k,n_v", HEADS)
def test_context_of_one_returns_v(n_q, n_k, n_v):
    q, k, v = rnd((3, n_q, 16), 1), rnd((3, n_k, 1, 16), 2), rnd((3, n_v, 1, 8), 3)
    out, lse = oracle.decode(q, k, v)
    g = n_q // n_v
    for h in range(n_q):
        assert np.array_equal(out[:, h, :], v[:, h // g, 0, :].astype(np.float64))
    # lse of a single score is the score itself
    s = np.einsum("bhc,bhc->bh", q.astype(np.float64), np.repeat(k[:, :, 0], n_q // n_k, axis=1).astype(np.float64))
    rel_close(lse, s * oracle.default_scale(16))


# P2: weights sum to one => constant V rows come back unchanged, whatever Q and K are.
def test_constant_v_returns_constant():
    q, k = rnd((2, 8, 32), 4), rnd((2, 2, 37, 32), 5)
    c = rnd((2, 4, 1, 16), 6)
    v = np.ascontiguousarray(np.broadcast_to(c, (2, 4, 37, 16)))
    out, _ = oracle.decode(q, k, v)
    for h in range(8):
        rel_close(out[:, h], c[:, h // 2, 0].astype(np.float64), 1e-14)


# P3: the paper's own second definition -- expand K (or V) by repeat-interleave and run ordinary
# attention per query head (appendix, KV group sharing).  Pins the head map for n_k<n_v and n_k>n_v.
@pytest.mark.parametrize("n_q,n_k,n_v", HEADS)
@pytest.mark.parametrize("bf16", [False, True])
def test_equals_attention_on_expanded_heads(n_q, n_k, n_v, bf16):
    q, k, v = rnd((2, n_q, 24), 7), rnd((2, n_k, 29, 24), 8), rnd((2, n_v, 29, 40), 9)
    if bf16:
        q, k, v = to_bf16_bits(q), to_bf16_bits(k), to_bf16_bits(v)
    scale = 0.37
    out, lse = oracle.decode(q, k, v, scale=scale)
    ro, rl = brute.diffqkv_decode_by_expansion(q, k, v, scale)
    rel_close(out, ro)
    rel_close(lse, rl)


# P4: n_k = n_v is grouped-query attention, n_k = n_v = n_q multi-head, n_k = n_v = 1 multi-query
# (appendix "Comparison with Existing Attention Mechanisms"): compare with a library routine.
@pytest.mark.parametrize("n_q,n_kv", [(8, 8), (8, 2), (8, 1), (6, 3)])
def test_reduces_to_library_attention(n_q, n_kv):
    B, T, d = 2, 33, 16
    q, k, v = rnd((B, n_q, d), 10), rnd((B, n_kv, T, d), 11), rnd((B, n_kv, T, d), 12)
    out, _ = oracle.decode(q, k, v)
    tq = torch.from_numpy(q).double()[:, :, None, :]
    tk = torch.from_numpy(k).double().repeat_interleave(n_q // n_kv, dim=1)
    tv = torch.from_numpy(v).double().repeat_interleave(n_q // n_kv, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=oracle.default_scale(d))
    rel_close(out, ref[:, :, 0, :].numpy(), 1e-11)


# P5: brute-force enumeration with explicit integer head indices on every divisor pair.
def test_brute_force_tiny_shapes():
    for n_q in (1, 2, 4, 6):
        divs = [x for x in range(1, n_q + 1) if n_q % x == 0]
        for n_k, n_v in itertools.product(divs, divs):
            for T in (1, 2, 5):
                q, k, v = rnd((2, n_q, 4), 13 + T), rnd((2, n_k, T, 4), 14 + n_k), rnd((2, n_v, T, 3), 15 + n_v)
                out, _ = oracle.decode(q, k, v, scale=0.5)
                rel_close(out, brute.enumerate_decode(q, k, v, 0.5))


# P6: q = 0 gives uniform weights: the output is the arithmetic mean of the V rows.
def test_zero_query_gives_mean_of_v():
    q = np.zeros((2, 4, 8), np.float32)
    k, v = rnd((2, 1, 50, 8), 16), rnd((2, 2, 50, 8), 17)
    out, lse = oracle.decode(q, k, v)
    for h in range(4):
        rel_close(out[:, h], v[:, h // 2].astype(np.float64).mean(axis=1))
    rel_close(lse, np.full((2, 4), math.log(50.0)))


# P7: adding the same vector u to every K row shifts every score of a head by q.u: no change.
def test_score_shift_invariance():
    q, k, v = rnd((1, 4, 8), 18), rnd((1, 2, 20, 8), 19), rnd((1, 4, 20, 8), 20)
    u = rnd((1, 2, 1, 8), 21)
    a, la = oracle.decode(q, k, v)
    b, lb = oracle.decode(q, (k.astype(np.float64) + u).astype(np.float32), v)
    # the shifted K is re-rounded to fp32, so agreement is to fp32 rounding of the scores only
    assert np.max(np.abs(a - b)) < 5e-6
    shift = np.einsum("bhc,bhc->bh", q.astype(np.float64), np.repeat(u[:, :, 0], 2, axis=1)) * oracle.default_scale(8)
    assert np.max(np.abs((lb - la) - shift)) < 5e-6


# P8: the result does not depend on the order of the cached tokens => a paged cache with any page
# permutation equals the contiguous cache it represents.
@pytest.mark.parametrize("P", [1, 4, 16])
def test_paged_equals_contiguous(P):
    cfg = inputs.config("paged_ragged", B=3, n_q=8, n_k=2, n_v=4, d_qk=16, d_v=16, page_size=P,
                        seqlens=[1, 37, 64])
    d = inputs.make_paged(cfg)
    q, kp, vp = (inputs.as_numpy(d[x]) for x in ("q", "k_pool", "v_pool"))
    bt, sl = d["block_table"].numpy(), d["seqlens"].numpy()
    out, lse = oracle.decode_paged(q, kp, vp, bt, sl)
    kc, vc = brute.gather_paged(kp, bt, sl, 64), brute.gather_paged(vp, bt, sl, 64)
    ro, rl = brute.diffqkv_decode_by_expansion(q, kc, vc, oracle.default_scale(16), seqlens=sl)
    rel_close(out, ro)
    rel_close(lse, rl)
    # and joint permutation of the rows of a contiguous cache changes nothing
    perm = np.random.default_rng(0).permutation(37)
    o1, _ = oracle.decode(q[1:2], kc[1:2, :, :37], vc[1:2, :, :37])
    o2, _ = oracle.decode(q[1:2], np.ascontiguousarray(kc[1:2, :, perm]), np.ascontiguousarray(vc[1:2, :, perm]))
    rel_close(o1, o2, 1e-13)


# P9: splitting the context and merging the parts by log-sum-exp is the whole.
def test_split_merge_identity():
    q, k, v = rnd((1, 4, 8), 22), rnd((1, 2, 23, 8), 23), rnd((1, 2, 23, 8), 24)
    full, lfull = oracle.decode(q, k, v)
    for cuts in ([5], [1, 22], [7, 7, 15], [23]):
        edges = [0] + list(np.cumsum(cuts)) if sum(cuts) == 23 else [0] + cuts + [23]
        edges = sorted(set(min(e, 23) for e in edges))
        parts = [oracle.decode(q, np.ascontiguousarray(k[:, :, a:b]), np.ascontiguousarray(v[:, :, a:b]))
                 for a, b in zip(edges[:-1], edges[1:])]
        for h in range(4):
            o, l = oracle.lse_merge(np.stack([p[0][0, h] for p in parts]), np.array([p[1][0, h] for p in parts]))
            rel_close(o, full[0, h])
            assert abs(l - lfull[0, h]) < 1e-12
    # an empty part (lse = -inf) contributes nothing
    o, l = oracle.lse_merge(np.stack([full[0, 0], np.full(8, 123.0)]), np.array([lfull[0, 0], -np.inf]))
    rel_close(o, full[0, 0])


# P10: causal prefill row i is decode over the first i+1 cache rows; the last row is decode at T=S.
# With S_k > S_q the mask is aligned to the newest token.
@pytest.mark.parametrize("S_q,S_k", [(9, 9), (4, 11)])
def test_prefill_rows_are_decodes(S_q, S_k):
    B, n_q, n_k, n_v, d = 2, 4, 1, 2, 8
    q, k, v = rnd((B, n_q, S_q, d), 25), rnd((B, n_k, S_k, d), 26), rnd((B, n_v, S_k, d), 27)
    out, lse = oracle.prefill(q, k, v, causal=True)
    for i in range(S_q):
        t = i + 1 + S_k - S_q
        ro, rl = brute.diffqkv_decode_by_expansion(np.ascontiguousarray(q[:, :, i]), k[:, :, :t], v[:, :, :t],
                                                   oracle.default_scale(d))
        rel_close(out[:, :, i], ro)
        rel_close(lse[:, :, i], rl)
    # row subset selection returns the same rows
    sub, _ = oracle.prefill(q, k, v, causal=True, rows=[S_q - 1, 0])
    assert np.array_equal(sub[:, :, 0], out[:, :, S_q - 1]) and np.array_equal(sub[:, :, 1], out[:, :, 0])
    # non-causal: every row sees every key
    nc, _ = oracle.prefill(q, k, v, causal=False)
    ro, _ = brute.diffqkv_decode_by_expansion(np.ascontiguousarray(q[:, :, 0]), k, v, oracle.default_scale(d))
    rel_close(nc[:, :, 0], ro)


# P11: orthogonal K rows with a large scale make the softmax one-hot: the output tends to V[j].
def test_one_hot_limit():
    d, T = 8, 8
    k = (np.eye(T, d, dtype=np.float32) * 1.0)[None, None]
    v = rnd((1, 1, T, 5), 28)
    for j in range(T):
        q = np.zeros((1, 2, d), np.float32)
        q[0, :, j] = 1.0
        out, _ = oracle.decode(q, k, v, scale=60.0)
        assert np.max(np.abs(out[0, 0] - v[0, 0, j])) < 1e-9
        assert np.max(np.abs(out[0, 1] - v[0, 0, j])) < 1e-9


# P12: head locality -- K head k' only reaches query heads [k' g_k, (k'+1) g_k); same for V with g_v.
def test_head_locality():
    n_q, n_k, n_v = 12, 2, 6
    q, k, v = rnd((1, n_q, 8), 29), rnd((1, n_k, 10, 8), 30), rnd((1, n_v, 10, 8), 31)
    base, _ = oracle.decode(q, k, v)
    for kh in range(n_k):
        k2 = k.copy()
        k2[:, kh] += 1.0
        changed = np.any(oracle.decode(q, k2, v)[0] != base, axis=-1)[0]
        assert list(np.nonzero(changed)[0]) == list(range(kh * 6, (kh + 1) * 6))
    for vh in range(n_v):
        v2 = v.copy()
        v2[:, vh] += 1.0
        changed = np.any(oracle.decode(q, k, v2)[0] != base, axis=-1)[0]
        assert list(np.nonzero(changed)[0]) == list(range(vh * 2, (vh + 1) * 2))


# strides: a token-major cache (b, s, n, d), as in the paper's cost model, read through strides
def test_token_major_strides():
    q, k, v = rnd((2, 4, 8), 32), rnd((2, 9, 2, 8), 33), rnd((2, 9, 4, 8), 34)
    a, _ = oracle.decode(q, k.transpose(0, 2, 1, 3), v.transpose(0, 2, 1, 3))
    b, _ = oracle.decode(q, np.ascontiguousarray(k.transpose(0, 2, 1, 3)), np.ascontiguousarray(v.transpose(0, 2, 1, 3)))
    assert np.array_equal(a, b)


# ragged lengths and the empty context
def test_seqlens_and_empty_context():
    q, k, v = rnd((3, 4, 8), 35), rnd((3, 2, 12, 8), 36), rnd((3, 2, 12, 8), 37)
    sl = np.array([0, 5, 12], np.int32)
    out, lse = oracle.decode(q, k, v, seqlens=sl)
    assert np.all(out[0] == 0) and np.all(np.isneginf(lse[0]))
    ro, _ = brute.diffqkv_decode_by_expansion(q[1:2], k[1:2, :, :5], v[1:2, :, :5], oracle.default_scale(8))
    rel_close(out[1:2], ro)
    # poison beyond T_b must not matter
    k2, v2 = k.copy(), v.copy()
    k2[1, :, 5:] = np.nan
    v2[1, :, 5:] = np.nan
    out2, _ = oracle.decode(q, k2, v2, seqlens=sl)
    assert np.array_equal(out2[1], out[1])


# the paper's printed cost-model numbers pin the algorithmic-bytes formula used by the bench
def test_cost_model_golden():
    import os

    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "kv_cost_model.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            p = line.split()
            rows[p[0]] = [float(x) for x in p[1:]]
    per_tok = {}
    for name in ("sigma_1p5b", "gqa_std"):
        n_k, d_k, n_v, d_v, elems = (int(x) for x in rows[name])
        cfg = dict(dtype="bf16", n_k=n_k, n_v=n_v, d_qk=d_k, d_v=d_v)
        assert inputs.kv_bytes_per_token(cfg) == 2 * elems
        per_tok[name] = inputs.kv_bytes_per_token(cfg)
    assert (per_tok["gqa_std"] - per_tok["sigma_1p5b"]) / per_tok["gqa_std"] == rows["limit_reduction"][0]


# KV-cache store: appending token t and attending over t+1 rows is attention over the concatenation
# (the paper concatenates k_t, v_t to the cache before attending); everything else stays untouched.
def test_append_then_decode_is_decode_on_concatenation():
    B, n_q, n_k, n_v, d, T_cap = 3, 8, 2, 4, 8, 12
    q, k, v = rnd((B, n_q, d), 40), rnd((B, n_k, T_cap, d), 41), rnd((B, n_v, T_cap, d), 42)
    k_new, v_new = rnd((B, n_k, d), 43), rnd((B, n_v, d), 44)
    pos = np.array([0, 5, 11], np.int32)
    k2, v2 = oracle.append(k_new, v_new, k, v, pos)
    for b in range(B):
        t = int(pos[b])
        kc = np.concatenate([k[b : b + 1, :, :t], k_new[b : b + 1, :, None]], axis=2)
        vc = np.concatenate([v[b : b + 1, :, :t], v_new[b : b + 1, :, None]], axis=2)
        ref, _ = brute.diffqkv_decode_by_expansion(q[b : b + 1], kc, vc, oracle.default_scale(d))
        got, _ = oracle.decode(q[b : b + 1], k2[b : b + 1], v2[b : b + 1], T=t + 1)
        rel_close(got, ref)
        mask = np.ones(T_cap, bool)
        mask[t] = False
        assert np.array_equal(k2[b][:, mask], k[b][:, mask]) and np.array_equal(v2[b][:, mask], v[b][:, mask])
    # out-of-range positions write nothing
    k3, v3 = oracle.append(k_new, v_new, k, v, np.array([-1, T_cap, 99], np.int32))
    assert np.array_equal(k3, k) and np.array_equal(v3, v)


def test_append_paged_matches_contiguous_view():
    cfg = inputs.config("paged_ragged", B=3, n_q=8, n_k=2, n_v=4, d_qk=16, d_v=16, page_size=4, seqlens=[3, 8, 10],
                        max_pages=4)
    d = inputs.make_paged(cfg)
    kp, vp = inputs.as_numpy(d["k_pool"]), inputs.as_numpy(d["v_pool"])
    bt = d["block_table"].numpy().copy()
    # sequence 1 is exactly at a page boundary: give it (and every sequence) a spare page
    used = set(bt[bt >= 0].tolist())
    spare = [p for p in range(kp.shape[0] + 3) if p not in used]
    kp = np.concatenate([kp, np.zeros((3,) + kp.shape[1:], kp.dtype)])
    vp = np.concatenate([vp, np.zeros((3,) + vp.shape[1:], vp.dtype)])
    for b in range(3):
        row = bt[b]
        row[np.argmax(row < 0)] = spare[b]
    pos = d["seqlens"].numpy()
    k_new, v_new = to_bf16_bits(rnd((3, 2, 16), 45)), to_bf16_bits(rnd((3, 4, 16), 46))
    kp2, vp2 = oracle.append_paged(k_new, v_new, kp, vp, bt, pos)
    kc, vc = brute.gather_paged(kp2, bt, pos + 1, 16), brute.gather_paged(vp2, bt, pos + 1, 16)
    for b in range(3):
        assert np.array_equal(kc[b, :, pos[b]], k_new[b]) and np.array_equal(vc[b, :, pos[b]], v_new[b])
    kc0, vc0 = brute.gather_paged(kp, bt, pos, 16), brute.gather_paged(vp, bt, pos, 16)
    for b in range(3):
        assert np.array_equal(kc[b, :, : pos[b]], kc0[b, :, : pos[b]])


# ---- selective V-cache fetching (top-k) ---------------------------------------------------------------
def topk_by_argsort(q, k, v, scale, top_k, renormalize):
    """Independent numpy statement: full softmax, stable descending argsort of the previous positions."""
    q, k, v = (brute.bf16_bits_to_f64(x) for x in (q, k, v))
    B, n_q, _ = q.shape
    n_k, n_v, T = k.shape[1], v.shape[1], k.shape[2]
    out = np.zeros((B, n_q, v.shape[3]))
    picks = []
    for b in range(B):
        for h in range(n_q):
            kh, vh = h // (n_q // n_k), h // (n_q // n_v)
            s = scale * (k[b, kh] @ q[b, h])
            a = np.exp(s - s.max())
            a /= a.sum()
            order = np.argsort(-a[: T - 1], kind="stable")[:top_k]  # stable: ties keep the lower position first
            idx = np.sort(np.concatenate([order, [T - 1]])).astype(int)
            o = (a[idx, None] * v[b, vh, idx]).sum(axis=0)
            out[b, h] = o / a[idx].sum() if renormalize else o
            picks.append(idx)
    return out, picks


@pytest.mark.parametrize("renorm", [False, True])
def test_topk_matches_argsort_statement(renorm):
    q, k, v = rnd((2, 8, 16), 50), rnd((2, 2, 40, 16), 51), rnd((2, 4, 40, 8), 52)
    for top_k in (0, 1, 5, 38, 39, 100):
        out, _, sel = oracle.decode_topk(q, k, v, top_k, scale=0.7, renormalize=renorm)
        ref, picks = topk_by_argsort(q, k, v, 0.7, top_k, renorm)
        rel_close(out, ref)
        for i, idx in enumerate(picks):
            got = sel.reshape(-1, top_k + 1)[i]
            assert list(got[got >= 0]) == list(idx)


def test_topk_covering_everything_is_plain_attention():
    q, k, v = rnd((2, 4, 8), 53), rnd((2, 1, 17, 8), 54), rnd((2, 2, 17, 8), 55)
    full, lfull = oracle.decode(q, k, v)
    for top_k in (16, 17, 1000):
        for renorm in (False, True):
            out, lse, _ = oracle.decode_topk(q, k, v, top_k, renormalize=renorm)
            rel_close(out, full)
            rel_close(lse, lfull)


def test_topk_ties_go_to_the_lower_position_and_current_token_always_counts():
    # all keys equal => all weights equal: the first top_k positions win; the last token is always in
    q = rnd((1, 2, 8), 56)
    k = np.ones((1, 1, 10, 8), np.float32)
    v = rnd((1, 1, 10, 4), 57)
    out, _, sel = oracle.decode_topk(q, k, v, 3, renormalize=False)
    assert list(sel[0, 0]) == [0, 1, 2, 9]
    rel_close(out[0, 0], v[0, 0, [0, 1, 2, 9]].astype(np.float64).sum(axis=0) / 10.0)
    out, _, sel = oracle.decode_topk(q, k, v, 3, renormalize=True)  # four equal weights: their mean
    assert list(sel[0, 0]) == [0, 1, 2, 9]
    rel_close(out[0, 0], v[0, 0, [0, 1, 2, 9]].astype(np.float64).mean(axis=0))
    # renormalised weights sum to one: constant V comes back unchanged; unnormalised: scaled by the kept mass
    vc = np.full((1, 1, 10, 4), 2.5, np.float32)
    rel_close(oracle.decode_topk(q, k, vc, 3, renormalize=True)[0], np.full((1, 2, 4), 2.5))
    rel_close(oracle.decode_topk(q, k, vc, 3, renormalize=False)[0], np.full((1, 2, 4), 2.5 * 0.4))
    # a current token with a negligible weight is still loaded
    k2 = k.copy()
    k2[0, 0, 9] = -50.0 * np.sign(q[0, 0])
    _, _, sel2 = oracle.decode_topk(q, k2, v, 2)
    assert 9 in list(sel2[0, 0]) and 9 in list(sel2[0, 1])


# ---- augmented Q (observations 3-4 of section 2; the appendix's attention listing) -------------------

def _augq_case(M, hidden, inter, seed):
    return (rnd((M, hidden), seed), rnd((inter, hidden), seed + 1) / np.float32(np.sqrt(hidden)),
            rnd((inter, hidden), seed + 2) / np.float32(np.sqrt(hidden)),
            rnd((hidden, inter), seed + 3) / np.float32(np.sqrt(inter)))


def test_augq_matches_library_linear_and_silu():
    x, wg, wu, wd = _augq_case(5, 24, 40, 80)
    t = lambda a: torch.from_numpy(a.astype(np.float64))
    F = torch.nn.functional
    want = F.linear(F.silu(F.linear(t(x), t(wg))) * F.linear(t(x), t(wu)), t(wd)).numpy()
    rel_close(oracle.augment_q(x, wg, wu, wd), want)


def test_augq_brute_force_loops():
    x, wg, wu, wd = _augq_case(2, 3, 4, 84)
    want = np.zeros((2, 3))
    for m in range(2):
        mid = []
        for i in range(4):
            g = sum(float(wg[i, c]) * float(x[m, c]) for c in range(3))
            u = sum(float(wu[i, c]) * float(x[m, c]) for c in range(3))
            mid.append(g / (1.0 + math.exp(-g)) * u)
        for j in range(3):
            want[m, j] = sum(float(wd[j, i]) * mid[i] for i in range(4))
    rel_close(oracle.augment_q(x, wg, wu, wd), want)


def test_augq_closed_forms():
    x, wg, wu, wd = _augq_case(3, 8, 8, 88)
    # a zero gate closes everything: silu(0) = 0
    assert np.all(oracle.augment_q(x, np.zeros_like(wg), wu, wd) == 0.0)
    # identity up and down projections leave silu(W_gate x) * x
    eye = np.eye(8, dtype=np.float32)
    g = wg.astype(np.float64) @ x.astype(np.float64).T
    rel_close(oracle.augment_q(x, wg, eye, eye), (g / (1.0 + np.exp(-g))).T * x.astype(np.float64))
    # linear in W_up and in W_down, not in W_gate; gate and up are not interchangeable
    base = oracle.augment_q(x, wg, wu, wd)
    rel_close(oracle.augment_q(x, wg, 2 * wu, wd), 2 * base)
    rel_close(oracle.augment_q(x, wg, wu, -4 * wd), -4 * base)  # (powers of two: exact in fp32)
    assert np.max(np.abs(oracle.augment_q(x, wu, wg, wd) - base)) > 1e-3
    # a large gate passes the up branch through: silu(z) -> z
    big = oracle.augment_q(x, 1000 * eye, eye, eye)
    xp = x.astype(np.float64)
    rel_close(big[xp > 0.05], (1000 * xp * xp)[xp > 0.05], tol=1e-9)
    # bf16 inputs are widened exactly
    xb = (x.view(np.uint32) >> 16).astype(np.uint16)
    wb = [(w.view(np.uint32) >> 16).astype(np.uint16) for w in (wg, wu, wd)]
    widen = lambda b: (b.astype(np.uint32) << 16).view(np.float32)
    rel_close(oracle.augment_q(xb, *wb), oracle.augment_q(widen(xb), *[widen(w) for w in wb]))
