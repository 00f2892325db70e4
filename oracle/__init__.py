"""Float64 CPU oracle for DiffQKV attention -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``diffqkv_oracle.c`` (plain C, double precision, two-pass softmax).
Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import
this package.  It knows nothing about the GPU library and imports nothing from it.

Arrays are numpy: fp32 inputs as ``float32``, bf16 inputs as ``uint16`` bit patterns.  Outputs are
``float64``.  Definitions follow section 2 ("Formulation of DiffQKV Attention") of the paper and the
head-index rule ("idx" equation, section 3.2).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "diffqkv_oracle.c"
_SO = _HERE / "libdiffqkv_oracle.so"

F32 = 0
BF16 = 1


def build(force: bool = False) -> Path:
    """Compile the C oracle with gcc (-O2 -fopenmp).  Rebuilds when the source is newer."""
    if force or not _SO.exists() or _SO.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _SO.with_suffix(".so.tmp%d" % os.getpid())
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", str(tmp), str(_SRC), "-lm"]
        )
        os.replace(tmp, _SO)
    return _SO


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_SO))
        i32, i64, f64, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.oracle_decode.restype = i32
        lib.oracle_decode.argtypes = [i32] * 7 + [f64] + [vp] * 3 + [i64] * 6 + [vp, i32, vp, vp]
        lib.oracle_decode_paged.restype = i32
        lib.oracle_decode_paged.argtypes = (
            [i32] * 7 + [f64] + [vp] * 3 + [i64] * 6 + [vp, i32, i32, vp, vp, vp]
        )
        lib.oracle_prefill.restype = i32
        lib.oracle_prefill.argtypes = [i32] * 7 + [f64] + [vp] * 3 + [i32, i32, i32, vp, i32, vp, vp]
        lib.oracle_lse_merge.restype = i32
        lib.oracle_lse_merge.argtypes = [i32, i32, vp, vp, vp, vp]
        lib.oracle_decode_topk.restype = i32
        lib.oracle_decode_topk.argtypes = [i32] * 7 + [f64] + [vp] * 3 + [i64] * 6 + [vp, i32, i32, i32, vp, vp, vp]
        lib.oracle_augment_q.restype = i32
        lib.oracle_augment_q.argtypes = [i32] * 4 + [vp] * 5
        lib.oracle_num_threads.restype = i32
        lib.oracle_num_threads.argtypes = []
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError("oracle inputs must be float32 or uint16 (bf16 bit patterns), got %s" % a.dtype)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _elem_strides(a: np.ndarray):
    assert all(s % a.itemsize == 0 for s in a.strides)
    return [s // a.itemsize for s in a.strides]


def default_scale(d_qk: int) -> float:
    """1/sqrt(d_qk), rounded to float32 the way the GPU boundary receives it."""
    return float(np.float32(1.0 / np.sqrt(np.float64(d_qk))))


def decode(q, k_cache, v_cache, seqlens=None, scale=None, T=None):
    """q [B,n_q,d_qk]; k_cache [B,n_k,T_cap,d_qk]; v_cache [B,n_v,T_cap,d_v] (any row/head/batch
    strides, innermost contiguous).  ``seqlens`` int32 [B] or None (every T_b = T, default T_cap).
    Returns (out float64 [B,n_q,d_v], lse float64 [B,n_q])."""
    code = _dtype_code(q)
    assert _dtype_code(k_cache) == code and _dtype_code(v_cache) == code
    q = np.ascontiguousarray(q)
    B, n_q, d_qk = q.shape
    Bk, n_k, T_cap, dk2 = k_cache.shape
    Bv, n_v, T_cap_v, d_v = v_cache.shape
    assert Bk == B and Bv == B and dk2 == d_qk and T_cap_v == T_cap
    ks, vs = _elem_strides(k_cache), _elem_strides(v_cache)
    assert ks[3] == 1 and vs[3] == 1
    if T is None:
        T = T_cap
    assert 0 <= T <= T_cap
    if seqlens is not None:
        seqlens = np.ascontiguousarray(seqlens, dtype=np.int32)
        assert seqlens.shape == (B,)
    if scale is None:
        scale = default_scale(d_qk)
    out = np.empty((B, n_q, d_v), dtype=np.float64)
    lse = np.empty((B, n_q), dtype=np.float64)
    rc = _load().oracle_decode(
        code, B, n_q, n_k, n_v, d_qk, d_v, float(scale), _ptr(q), _ptr(k_cache), _ptr(v_cache),
        ks[0], ks[1], ks[2], vs[0], vs[1], vs[2], _ptr(seqlens), int(T), _ptr(out), _ptr(lse),
    )
    if rc != 0:
        raise ValueError("oracle_decode rejected its arguments")
    return out, lse


def decode_topk(q, k_cache, v_cache, top_k, seqlens=None, scale=None, T=None, renormalize=True):
    """Selective V-cache fetching: weights from the softmax over all T positions, output from the
    `top_k` previous positions of largest weight plus the current token (position T_b - 1).
    Returns (out [B,n_q,d_v], lse [B,n_q], selected int32 [B,n_q,top_k+1] padded with -1)."""
    code = _dtype_code(q)
    assert _dtype_code(k_cache) == code and _dtype_code(v_cache) == code
    q = np.ascontiguousarray(q)
    B, n_q, d_qk = q.shape
    _, n_k, T_cap, _ = k_cache.shape
    _, n_v, _, d_v = v_cache.shape
    ks, vs = _elem_strides(k_cache), _elem_strides(v_cache)
    assert ks[3] == 1 and vs[3] == 1
    if T is None:
        T = T_cap
    if seqlens is not None:
        seqlens = np.ascontiguousarray(seqlens, dtype=np.int32)
    if scale is None:
        scale = default_scale(d_qk)
    out = np.empty((B, n_q, d_v), dtype=np.float64)
    lse = np.empty((B, n_q), dtype=np.float64)
    sel = np.empty((B, n_q, top_k + 1), dtype=np.int32)
    rc = _load().oracle_decode_topk(
        code, B, n_q, n_k, n_v, d_qk, d_v, float(scale), _ptr(q), _ptr(k_cache), _ptr(v_cache),
        ks[0], ks[1], ks[2], vs[0], vs[1], vs[2], _ptr(seqlens), int(T), int(top_k), 1 if renormalize else 0,
        _ptr(out), _ptr(lse), _ptr(sel),
    )
    if rc != 0:
        raise ValueError("oracle_decode_topk rejected its arguments")
    return out, lse, sel


def decode_paged(q, k_pool, v_pool, block_table, seqlens, scale=None):
    """q [B,n_q,d_qk]; k_pool [n_pages,n_k,P,d_qk]; v_pool [n_pages,n_v,P,d_v]; block_table int32
    [B,max_pages]; seqlens int32 [B].  Returns (out [B,n_q,d_v], lse [B,n_q]) in float64."""
    code = _dtype_code(q)
    assert _dtype_code(k_pool) == code and _dtype_code(v_pool) == code
    q = np.ascontiguousarray(q)
    B, n_q, d_qk = q.shape
    n_pages, n_k, P, dk2 = k_pool.shape
    n_pages_v, n_v, Pv, d_v = v_pool.shape
    assert dk2 == d_qk and Pv == P and n_pages_v == n_pages
    ks, vs = _elem_strides(k_pool), _elem_strides(v_pool)
    assert ks[3] == 1 and vs[3] == 1
    block_table = np.ascontiguousarray(block_table, dtype=np.int32)
    seqlens = np.ascontiguousarray(seqlens, dtype=np.int32)
    assert block_table.shape[0] == B and seqlens.shape == (B,)
    max_pages = block_table.shape[1]
    for b in range(B):  # every page a sequence uses must exist
        used = (int(seqlens[b]) + P - 1) // P
        row = block_table[b, :used]
        assert used <= max_pages and (row >= 0).all() and (row < n_pages).all()
    if scale is None:
        scale = default_scale(d_qk)
    out = np.empty((B, n_q, d_v), dtype=np.float64)
    lse = np.empty((B, n_q), dtype=np.float64)
    rc = _load().oracle_decode_paged(
        code, B, n_q, n_k, n_v, d_qk, d_v, float(scale), _ptr(q), _ptr(k_pool), _ptr(v_pool),
        ks[0], ks[1], ks[2], vs[0], vs[1], vs[2], _ptr(block_table), max_pages, P,
        _ptr(seqlens), _ptr(out), _ptr(lse),
    )
    if rc != 0:
        raise ValueError("oracle_decode_paged rejected its arguments")
    return out, lse


def prefill(q, k, v, causal=True, rows=None, scale=None):
    """q [B,n_q,S_q,d_qk]; k [B,n_k,S_k,d_qk]; v [B,n_v,S_k,d_v], dense.  ``rows``: optional int32
    list of query positions to evaluate (all when None).  Causal masks are bottom-right aligned:
    query i sees keys j <= i + S_k - S_q.  Returns (out [B,n_q,R,d_v], lse [B,n_q,R]) float64."""
    code = _dtype_code(q)
    assert _dtype_code(k) == code and _dtype_code(v) == code
    q, k, v = np.ascontiguousarray(q), np.ascontiguousarray(k), np.ascontiguousarray(v)
    B, n_q, S_q, d_qk = q.shape
    _, n_k, S_k, dk2 = k.shape
    _, n_v, S_kv, d_v = v.shape
    assert dk2 == d_qk and S_kv == S_k and k.shape[0] == B and v.shape[0] == B
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        R = int(rows.shape[0])
    else:
        R = S_q
    if scale is None:
        scale = default_scale(d_qk)
    out = np.empty((B, n_q, R, d_v), dtype=np.float64)
    lse = np.empty((B, n_q, R), dtype=np.float64)
    rc = _load().oracle_prefill(
        code, B, n_q, n_k, n_v, d_qk, d_v, float(scale), _ptr(q), _ptr(k), _ptr(v), S_q, S_k,
        1 if causal else 0, _ptr(rows), R, _ptr(out), _ptr(lse),
    )
    if rc != 0:
        raise ValueError("oracle_prefill rejected its arguments")
    return out, lse


def lse_merge(o_parts, lse_parts):
    """Merge S partial results of one output row: o_parts float64 [S,d_v] (each normalised),
    lse_parts float64 [S].  Returns (out [d_v], lse)."""
    o_parts = np.ascontiguousarray(o_parts, dtype=np.float64)
    lse_parts = np.ascontiguousarray(lse_parts, dtype=np.float64)
    S, d_v = o_parts.shape
    assert lse_parts.shape == (S,)
    out = np.empty((d_v,), dtype=np.float64)
    lse = np.empty((1,), dtype=np.float64)
    _load().oracle_lse_merge(S, d_v, _ptr(o_parts), _ptr(lse_parts), _ptr(out), _ptr(lse))
    return out, float(lse[0])


def append(k_new, v_new, k_cache, v_cache, positions):
    """KV-cache store (section 3.1, "KV Cache"): returns copies of the caches with k_new[b], v_new[b]
    written at token row positions[b]; rows outside [0, T_cap) are skipped.  Plain element copies:
    k_cache [B,n_k,T_cap,d_qk], v_cache [B,n_v,T_cap,d_v], k_new [B,n_k,d_qk], v_new [B,n_v,d_v]."""
    k_out, v_out = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    B, n_k, T_cap, d_qk = k_out.shape
    n_v, d_v = v_out.shape[1], v_out.shape[3]
    for b in range(B):
        t = int(positions[b])
        if t < 0 or t >= T_cap:
            continue
        for h in range(n_k):
            for c in range(d_qk):
                k_out[b, h, t, c] = k_new[b, h, c]
        for h in range(n_v):
            for c in range(d_v):
                v_out[b, h, t, c] = v_new[b, h, c]
    return k_out, v_out


def append_paged(k_new, v_new, k_pool, v_pool, block_table, positions):
    """Paged KV-cache store: token row positions[b] of sequence b is slot positions[b] % P of page
    block_table[b, positions[b] // P].  Returns copies of the pools."""
    k_out, v_out = np.array(k_pool, copy=True), np.array(v_pool, copy=True)
    n_pages, n_k, P, d_qk = k_out.shape
    n_v, d_v = v_out.shape[1], v_out.shape[3]
    B, max_pages = block_table.shape
    for b in range(B):
        t = int(positions[b])
        if t < 0 or t >= max_pages * P:
            continue
        page, slot = int(block_table[b, t // P]), t % P
        for h in range(n_k):
            for c in range(d_qk):
                k_out[page, h, slot, c] = k_new[b, h, c]
        for h in range(n_v):
            for c in range(d_v):
                v_out[page, h, slot, c] = v_new[b, h, c]
    return k_out, v_out


def augment_q(x, w_gate, w_up, w_down):
    """Augmented Q (observations 3-4, section 2): x [M, hidden] -> W_down(silu(W_gate x) * (W_up x)).
    w_gate, w_up [inter, hidden]; w_down [hidden, inter].  Returns float64 [M, hidden]."""
    code = _dtype_code(x)
    assert _dtype_code(w_gate) == code and _dtype_code(w_up) == code and _dtype_code(w_down) == code
    x, w_gate, w_up, w_down = (np.ascontiguousarray(a) for a in (x, w_gate, w_up, w_down))
    M, hidden = x.shape
    inter = w_gate.shape[0]
    assert w_gate.shape == (inter, hidden) and w_up.shape == (inter, hidden) and w_down.shape == (hidden, inter)
    out = np.empty((M, hidden), dtype=np.float64)
    rc = _load().oracle_augment_q(code, M, hidden, inter, _ptr(x), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(out))
    if rc != 0:
        raise ValueError("oracle_augment_q rejected its arguments")
    return out
