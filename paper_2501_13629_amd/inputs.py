"""Seeded synthetic inputs with the shapes of the paper's attention workloads.

This module holds data generation only -- none of the method's arithmetic.  It is the one module
that both the GPU tests/bench and the CPU oracle's callers use, so that both sides see exactly the
same (dtype-rounded) values.  Everything is produced on the host as torch CPU tensors; callers copy
them to the device.

Random numbers come from numpy's counter-based Philox generator, one independent counter block per
4 Mi-element chunk, so that the values do not depend on how many threads fill the buffer.
Shapes follow Sigma's attention (32 query heads; 2-4 K heads; 8-16 V heads; head width 64 or 128;
contexts from 1k to 64k tokens -- model table in the appendix and section 3.3 of the paper).
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

BASE_SEED = 20250113

# The five workloads.  `index` selects the seed (BASE_SEED + index).
CONFIGS = {
    "tiny_fp32": dict(index=0, kind="decode", dtype="f32", B=1, n_q=4, n_k=1, n_v=2, d_qk=64, d_v=64, T=128),
    "decode_4k": dict(index=1, kind="decode", dtype="bf16", B=16, n_q=32, n_k=4, n_v=16, d_qk=64, d_v=64, T=4096),
    "decode_32k": dict(index=2, kind="decode", dtype="bf16", B=8, n_q=32, n_k=2, n_v=8, d_qk=128, d_v=128,
                       T=32768, k_channel_scale=(0.5, 2.0)),
    "paged_ragged": dict(index=3, kind="paged", dtype="bf16", B=64, n_q=32, n_k=4, n_v=16, d_qk=128, d_v=128,
                         T_lo=1024, T_hi=65536, page_size=16),
    "prefill_8k": dict(index=4, kind="prefill", dtype="bf16", B=2, n_q=32, n_k=4, n_v=16, d_qk=128, d_v=128,
                       S=8192),
}
# The same long-context decode and prefill shapes with the K heads at half width (the paper's second
# compression axis, section 2, observation 2: d_qk = d_v / 2); bench workloads beside the five above.
CONFIGS["decode_32k_halfk"] = dict(CONFIGS["decode_32k"], index=5, d_qk=64)
CONFIGS["prefill_8k_halfk"] = dict(CONFIGS["prefill_8k"], index=6, d_qk=64)

_CHUNK = 1 << 22


def config(name: str, **overrides) -> dict:
    """A copy of one of the named workloads, optionally shrunk/changed (tests use small T, B)."""
    cfg = dict(CONFIGS[name])
    cfg["name"] = name
    cfg.update(overrides)
    return cfg


def torch_dtype(cfg) -> torch.dtype:
    return torch.float32 if cfg["dtype"] == "f32" else torch.bfloat16


def _workers() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def normal_tensor(shape, seed: int, stream: int, dtype: torch.dtype, row_scale: torch.Tensor | None = None):
    """N(0,1) values of `shape`, rounded to `dtype` (round-to-nearest-even for bf16).

    `stream` separates the tensors drawn under one seed (0 = Q, 1 = K, 2 = V).  `row_scale`, if
    given, has the shape of the trailing dimensions it scales (broadcast against `shape` from the
    right) and multiplies the fp32 values before rounding."""
    n = int(np.prod(shape))
    out = torch.empty(n, dtype=dtype)
    flat_scale = None
    if row_scale is not None:
        flat_scale = row_scale.to(torch.float32).expand(shape).reshape(-1) if n else None

    def fill(i):
        lo, hi = i * _CHUNK, min(n, (i + 1) * _CHUNK)
        rng = np.random.Generator(np.random.Philox(key=seed, counter=[0, 0, stream, i]))
        x = torch.from_numpy(rng.standard_normal(hi - lo, dtype=np.float32))
        if flat_scale is not None:
            x = x * flat_scale[lo:hi]
        out[lo:hi] = x.to(dtype)

    n_chunks = (n + _CHUNK - 1) // _CHUNK
    if n_chunks <= 1:
        for i in range(n_chunks):
            fill(i)
    else:
        with ThreadPoolExecutor(_workers()) as ex:
            list(ex.map(fill, range(n_chunks)))
    return out.reshape(shape)


def _aux_rng(seed: int) -> np.random.Generator:
    """Generator for the small auxiliary draws (channel scales, lengths, page permutation)."""
    return np.random.Generator(np.random.Philox(key=seed, counter=[0, 0, 99, 0]))


def make_decode(cfg) -> dict:
    """Contiguous-cache decode inputs: q [B,n_q,d_qk], k [B,n_k,T,d_qk], v [B,n_v,T,d_v]."""
    seed = BASE_SEED + cfg["index"]
    dt = torch_dtype(cfg)
    B, n_q, n_k, n_v, d_qk, d_v, T = (cfg[x] for x in ("B", "n_q", "n_k", "n_v", "d_qk", "d_v", "T"))
    aux = _aux_rng(seed)
    k_scale = None
    if cfg.get("k_channel_scale"):
        lo, hi = cfg["k_channel_scale"]
        # one factor per (K head, channel), shared by every sequence and token: outlier channels
        k_scale = torch.from_numpy(aux.uniform(lo, hi, size=(n_k, 1, d_qk)).astype(np.float32))
    q = normal_tensor((B, n_q, d_qk), seed, 0, dt)
    k = normal_tensor((B, n_k, T, d_qk), seed, 1, dt, row_scale=k_scale)
    v = normal_tensor((B, n_v, T, d_v), seed, 2, dt)
    seqlens = None
    if cfg.get("ragged"):
        seqlens = torch.from_numpy(aux.integers(1, T + 1, size=(B,)).astype(np.int32))
    return dict(q=q, k=k, v=v, seqlens=seqlens, T=T)


def log_uniform_lengths(rng: np.random.Generator, B: int, lo: int, hi: int) -> np.ndarray:
    """T_b = min(hi, floor(2 ** U[log2 lo, log2 hi)))."""
    u = rng.uniform(math.log2(lo), math.log2(hi), size=(B,))
    return np.minimum(hi, np.floor(np.exp2(u))).astype(np.int32)


def make_paged(cfg) -> dict:
    """Ragged paged decode inputs.

    Pool layout (head-major inside a page): k_pool [n_pages, n_k, P, d_qk], v_pool
    [n_pages, n_v, P, d_v].  The pool holds exactly sum_b ceil(T_b / P) pages; physical page ids are
    a seeded random permutation dealt to the sequences in order; unused block-table entries are -1.
    The slots of a sequence's last page beyond T_b hold ordinary random values (they must never
    influence the result)."""
    seed = BASE_SEED + cfg["index"]
    dt = torch_dtype(cfg)
    B, n_q, n_k, n_v, d_qk, d_v, P = (cfg[x] for x in ("B", "n_q", "n_k", "n_v", "d_qk", "d_v", "page_size"))
    aux = _aux_rng(seed)
    if "seqlens" in cfg:
        lens = np.asarray(cfg["seqlens"], dtype=np.int32)
    else:
        lens = log_uniform_lengths(aux, B, cfg["T_lo"], cfg["T_hi"])
    pages_per_seq = (lens.astype(np.int64) + P - 1) // P
    n_pages = int(pages_per_seq.sum())
    max_pages = int(cfg.get("max_pages", max(1, int(pages_per_seq.max()))))
    perm = aux.permutation(n_pages).astype(np.int32)
    table = np.full((B, max_pages), -1, dtype=np.int32)
    at = 0
    for b in range(B):
        table[b, : pages_per_seq[b]] = perm[at : at + pages_per_seq[b]]
        at += int(pages_per_seq[b])
    q = normal_tensor((B, n_q, d_qk), seed, 0, dt)
    k_pool = normal_tensor((n_pages, n_k, P, d_qk), seed, 1, dt)
    v_pool = normal_tensor((n_pages, n_v, P, d_v), seed, 2, dt)
    return dict(q=q, k_pool=k_pool, v_pool=v_pool, block_table=torch.from_numpy(table),
                seqlens=torch.from_numpy(lens), page_size=P, max_pages=max_pages, n_pages=n_pages)


def make_prefill(cfg) -> dict:
    """Causal prefill inputs: q [B,n_q,S,d_qk], k [B,n_k,S_k,d_qk], v [B,n_v,S_k,d_v]."""
    seed = BASE_SEED + cfg["index"]
    dt = torch_dtype(cfg)
    B, n_q, n_k, n_v, d_qk, d_v, S = (cfg[x] for x in ("B", "n_q", "n_k", "n_v", "d_qk", "d_v", "S"))
    S_k = cfg.get("S_k", S)
    q = normal_tensor((B, n_q, S, d_qk), seed, 0, dt)
    k = normal_tensor((B, n_k, S_k, d_qk), seed, 1, dt)
    v = normal_tensor((B, n_v, S_k, d_v), seed, 2, dt)
    return dict(q=q, k=k, v=v, S_q=S, S_k=S_k)


def make_augq(M: int, hidden: int, inter: int, dtype: str = "bf16", index: int = 40) -> dict:
    """Augmented-Q inputs: q_in [M, hidden] ~ N(0,1); weights of linear layers [out, in] ~ N(0, 1/in)
    (so that every product keeps unit scale), w_gate and w_up [inter, hidden], w_down [hidden, inter].
    Sigma's widths are hidden 2048 / inter 3072 and 4096 / 6144 (section 3.1 and its model table)."""
    dt = torch.float32 if dtype == "f32" else torch.bfloat16
    seed = BASE_SEED + index
    return dict(
        q_in=normal_tensor((M, hidden), seed, 0, dt),
        w_gate=normal_tensor((inter, hidden), seed, 1, dt, row_scale=torch.full((hidden,), hidden ** -0.5)),
        w_up=normal_tensor((inter, hidden), seed, 2, dt, row_scale=torch.full((hidden,), hidden ** -0.5)),
        w_down=normal_tensor((hidden, inter), seed, 3, dt, row_scale=torch.full((inter,), inter ** -0.5)),
    )


def as_numpy(t: torch.Tensor) -> np.ndarray:
    """Host view for the CPU oracle: fp32 stays float32, bf16 becomes its uint16 bit patterns
    (no value changes; strides preserved)."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.numpy()
    if t.dtype == torch.int32:
        return t.numpy()
    raise TypeError(t.dtype)


def kv_bytes_per_token(cfg) -> int:
    """Cache bytes read per (sequence, token): (n_k d_qk + n_v d_v) * element size -- the
    per-element KV-cache cost model of section 3.1 (equation "cache_0")."""
    s = 4 if cfg["dtype"] == "f32" else 2
    return (cfg["n_k"] * cfg["d_qk"] + cfg["n_v"] * cfg["d_v"]) * s
