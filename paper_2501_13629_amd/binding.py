"""Thin ctypes binding of libdiffqkv.so -- argument marshalling only.

Every step of the attention path runs inside the library's HIP kernels.  PyTorch appears here only
as the owner of device memory and of the HIP stream.  There is no CPU fallback: if the library has
not been built, or the tensors are not on a GPU, the calls raise.

Functions carry the names of the C entry points in ``include/diffqkv.h``.
"""
from __future__ import annotations

import ctypes
import os
from pathlib import Path

import torch

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "libdiffqkv.so"

F32, BF16 = 0, 1

# include/diffqkv.h
EXPORTS = (
    "diffqkv_decode_workspace_bytes", "diffqkv_decode", "diffqkv_decode_static", "diffqkv_decode_paged",
    "diffqkv_prefill_workspace_bytes", "diffqkv_prefill", "diffqkv_strerror",
    "diffqkv_version", "diffqkv_append", "diffqkv_append_paged",
    "diffqkv_decode_topk_workspace_bytes", "diffqkv_decode_topk", "diffqkv_decode_topk_paged",
    "diffqkv_augment_q_workspace_bytes", "diffqkv_augment_q",
)
# include/diffqkv_experimental.h (knobs and measurement aids; per calling thread)
EXPERIMENTAL_EXPORTS = ("diffqkv_set_tuning", "diffqkv_kernel_timer", "diffqkv_kernel_timer_read",
                        "diffqkv_probe_stream_read")


class Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "n_q", "n_k", "n_v", "d_qk", "d_v", "dtype")] + [
        ("softmax_scale", ctypes.c_float)
    ]


class AugqShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("M", "hidden", "inter", "dtype")]


class Tuning(ctypes.Structure):
    _fields_ = [("decode_chunk_tokens", ctypes.c_int32), ("force_generic", ctypes.c_int32),
                ("prefill_waves", ctypes.c_int32), ("decode_ragged_mode", ctypes.c_int32),
                ("decode_workers", ctypes.c_int32), ("reserved", ctypes.c_int32 * 3)]


class DiffQKVError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("diffqkv status %d: %s" % (status, text))
        self.status = status


_lib = None


def load_library() -> ctypes.CDLL:
    """Load the built library.  Raises if it is missing: build it first with
    ``python -m paper_2501_13629_amd.build`` (or ``__graft_entry__.build()``)."""
    global _lib
    if _lib is not None:
        return _lib
    path = Path(os.environ.get("DIFFQKV_LIBRARY", str(LIB_PATH)))  # override: another build of the same library
    if not path.exists():
        raise RuntimeError(
            "%s not found: the HIP library has not been built "
            "(run `python -m paper_2501_13629_amd.build`); there is no fallback path" % path
        )
    lib = ctypes.CDLL(str(path))
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    sp = ctypes.POINTER(Shape)
    lib.diffqkv_set_tuning.restype = None
    lib.diffqkv_set_tuning.argtypes = [ctypes.POINTER(Tuning)]
    lib.diffqkv_decode_workspace_bytes.restype = sz
    lib.diffqkv_decode_workspace_bytes.argtypes = [sp, i32]
    lib.diffqkv_decode.restype = ctypes.c_int
    lib.diffqkv_decode.argtypes = [sp, vp, vp, vp] + [i64] * 6 + [vp, i32, vp, vp, vp, sz, vp]
    lib.diffqkv_decode_static.restype = ctypes.c_int
    lib.diffqkv_decode_static.argtypes = [sp, vp, vp, vp] + [i64] * 6 + [vp, i32, vp, vp, vp]
    lib.diffqkv_decode_paged.restype = ctypes.c_int
    lib.diffqkv_decode_paged.argtypes = [sp, vp, vp, vp] + [i64] * 6 + [vp, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.diffqkv_prefill_workspace_bytes.restype = sz
    lib.diffqkv_prefill_workspace_bytes.argtypes = [sp, i32, i32]
    lib.diffqkv_prefill.restype = ctypes.c_int
    lib.diffqkv_prefill.argtypes = [sp, vp, vp, vp, i32, i32, i32, vp, vp, vp, sz, vp]
    lib.diffqkv_decode_topk_workspace_bytes.restype = sz
    lib.diffqkv_decode_topk_workspace_bytes.argtypes = [sp, i32]
    lib.diffqkv_decode_topk.restype = ctypes.c_int
    lib.diffqkv_decode_topk.argtypes = [sp, vp, vp, vp] + [i64] * 6 + [vp, i32, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.diffqkv_decode_topk_paged.restype = ctypes.c_int
    lib.diffqkv_decode_topk_paged.argtypes = ([sp, vp, vp, vp] + [i64] * 6 +
                                              [vp, i32, i32, vp, i32, i32, vp, vp, vp, vp, sz, vp])
    lib.diffqkv_append.restype = ctypes.c_int
    lib.diffqkv_append.argtypes = [sp, vp, vp, vp, vp] + [i64] * 6 + [vp, i32, vp, vp]
    lib.diffqkv_append_paged.restype = ctypes.c_int
    lib.diffqkv_append_paged.argtypes = [sp, vp, vp, vp, vp] + [i64] * 6 + [vp, i32, i32, vp, vp, vp]
    lib.diffqkv_augment_q_workspace_bytes.restype = sz
    lib.diffqkv_augment_q_workspace_bytes.argtypes = [ctypes.POINTER(AugqShape)]
    lib.diffqkv_augment_q.restype = ctypes.c_int
    lib.diffqkv_augment_q.argtypes = [ctypes.POINTER(AugqShape), vp, vp, vp, vp, vp, vp, sz, vp]
    lib.diffqkv_probe_stream_read.restype = ctypes.c_int
    lib.diffqkv_probe_stream_read.argtypes = [vp, sz, vp, vp]
    lib.diffqkv_strerror.restype = ctypes.c_char_p
    lib.diffqkv_strerror.argtypes = [ctypes.c_int]
    lib.diffqkv_kernel_timer.restype = ctypes.c_int
    lib.diffqkv_kernel_timer.argtypes = [ctypes.c_int]
    lib.diffqkv_kernel_timer_read.restype = ctypes.c_int
    lib.diffqkv_kernel_timer_read.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float),
                                              ctypes.POINTER(ctypes.c_int32)]
    lib.diffqkv_version.restype = ctypes.c_int
    lib.diffqkv_version.argtypes = []
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        raise DiffQKVError(status, load_library().diffqkv_strerror(status).decode())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("diffqkv supports float32 and bfloat16 tensors, got %s" % t.dtype)


def _dev(*tensors):
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise RuntimeError("diffqkv runs on the GPU only: every tensor must be a device tensor")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(t: torch.Tensor):
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def _shape(B, n_q, n_k, n_v, d_qk, d_v, dtype, scale) -> Shape:
    return Shape(B, n_q, n_k, n_v, d_qk, d_v, dtype, 0.0 if scale is None else float(scale))


def diffqkv_set_tuning(decode_chunk_tokens: int = 0, force_generic: bool = False, prefill_waves: int = 0,
                       decode_ragged_mode: int = 0, decode_workers: int = 0):
    t = Tuning(int(decode_chunk_tokens), 1 if force_generic else 0, int(prefill_waves), int(decode_ragged_mode),
               int(decode_workers))
    load_library().diffqkv_set_tuning(ctypes.byref(t))


def diffqkv_kernel_timer(on: bool) -> None:
    """Switch the calling thread's kernel timer on or off (see include/diffqkv_experimental.h)."""
    _check(load_library().diffqkv_kernel_timer(1 if on else 0))


def diffqkv_kernel_timer_read():
    """Wait for the timed launches since the last read; returns (average main-kernel us, average
    second-kernel us, number of main-kernel launches)."""
    a, b, n = ctypes.c_float(0.0), ctypes.c_float(0.0), ctypes.c_int32(0)
    _check(load_library().diffqkv_kernel_timer_read(ctypes.byref(a), ctypes.byref(b), ctypes.byref(n)))
    return float(a.value), float(b.value), int(n.value)


def diffqkv_version() -> int:
    return int(load_library().diffqkv_version())


def diffqkv_decode_workspace_bytes(B, n_q, n_k, n_v, d_qk, d_v, dtype, max_T) -> int:
    s = _shape(B, n_q, n_k, n_v, d_qk, d_v, dtype, None)
    return int(load_library().diffqkv_decode_workspace_bytes(ctypes.byref(s), int(max_T)))


def diffqkv_decode_topk_workspace_bytes(B, n_q, n_k, n_v, d_qk, d_v, dtype, max_T) -> int:
    s = _shape(B, n_q, n_k, n_v, d_qk, d_v, dtype, None)
    return int(load_library().diffqkv_decode_topk_workspace_bytes(ctypes.byref(s), int(max_T)))


def _workspace(nbytes: int, like: torch.Tensor, workspace):
    if workspace is not None:
        return workspace
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=like.device)


def diffqkv_decode(q, k_cache, v_cache, seqlens=None, T=None, scale=None, out=None, lse_out=None,
                   workspace=None, want_lse=False):
    """q [B,n_q,d_qk]; k_cache [B,n_k,T_cap,d_qk]; v_cache [B,n_v,T_cap,d_v] (any batch/head/token
    strides, channels contiguous); seqlens int32 device [B] or None.  Returns out, or (out, lse)."""
    _dev(q, k_cache, v_cache, seqlens, out, lse_out, workspace)
    dt = _dtype_code(q)
    if _dtype_code(k_cache) != dt or _dtype_code(v_cache) != dt:
        raise TypeError("q, k_cache and v_cache must share a dtype")
    if not q.is_contiguous():
        raise ValueError("q must be contiguous")
    B, n_q, d_qk = q.shape
    _, n_k, T_cap, _ = k_cache.shape
    _, n_v, _, d_v = v_cache.shape
    if k_cache.stride(3) != 1 or v_cache.stride(3) != 1:
        raise ValueError("the channel dimension of the caches must be contiguous")
    if T is None:
        T = T_cap
    if T > T_cap:
        raise ValueError("T exceeds the cache capacity")
    if seqlens is not None and (seqlens.dtype != torch.int32 or not seqlens.is_contiguous()):
        raise TypeError("seqlens must be a contiguous int32 tensor")
    if out is None:
        out = torch.empty((B, n_q, d_v), dtype=q.dtype, device=q.device)
    if lse_out is None and want_lse:
        lse_out = torch.empty((B, n_q), dtype=torch.float32, device=q.device)
    s = _shape(B, n_q, n_k, n_v, d_qk, d_v, dt, scale)
    lib = load_library()
    need = int(lib.diffqkv_decode_workspace_bytes(ctypes.byref(s), int(T)))
    workspace = _workspace(need, q, workspace)
    ks, vs = k_cache.stride(), v_cache.stride()
    _check(lib.diffqkv_decode(
        ctypes.byref(s), _ptr(q), _ptr(k_cache), _ptr(v_cache), ks[0], ks[1], ks[2], vs[0], vs[1], vs[2],
        _ptr(seqlens), int(T), _ptr(out), _ptr(lse_out), _ptr(workspace), workspace.numel(), _stream(q)))
    return (out, lse_out) if (want_lse or lse_out is not None) else out


STATIC_SCRATCH_BYTES = 32 << 20  # DIFFQKV_STATIC_SCRATCH_BYTES


def diffqkv_decode_static(q, k_cache, v_cache, out, seqlens=None, T=None, scale=None, lse_out=None):
    """diffqkv_decode without a workspace: the split partials go to the library's static device
    buffer and the call allocates nothing -- so `out` (and `lse_out`, if wanted) come from the caller."""
    _dev(q, k_cache, v_cache, seqlens, out, lse_out)
    dt = _dtype_code(q)
    if _dtype_code(k_cache) != dt or _dtype_code(v_cache) != dt or _dtype_code(out) != dt:
        raise TypeError("q, k_cache, v_cache and out must share a dtype")
    if not q.is_contiguous() or not out.is_contiguous():
        raise ValueError("q and out must be contiguous")
    B, n_q, d_qk = q.shape
    _, n_k, T_cap, _ = k_cache.shape
    _, n_v, _, d_v = v_cache.shape
    if tuple(out.shape) != (B, n_q, d_v):
        raise ValueError("out must be [B, n_q, d_v]")
    if k_cache.stride(3) != 1 or v_cache.stride(3) != 1:
        raise ValueError("the channel dimension of the caches must be contiguous")
    if T is None:
        T = T_cap
    if T > T_cap:
        raise ValueError("T exceeds the cache capacity")
    if seqlens is not None and (seqlens.dtype != torch.int32 or not seqlens.is_contiguous()):
        raise TypeError("seqlens must be a contiguous int32 tensor")
    s = _shape(B, n_q, n_k, n_v, d_qk, d_v, dt, scale)
    ks, vs = k_cache.stride(), v_cache.stride()
    _check(load_library().diffqkv_decode_static(
        ctypes.byref(s), _ptr(q), _ptr(k_cache), _ptr(v_cache), ks[0], ks[1], ks[2], vs[0], vs[1], vs[2],
        _ptr(seqlens), int(T), _ptr(out), _ptr(lse_out), _stream(q)))
    return out


def diffqkv_decode_paged(q, k_pool, v_pool, block_table, seqlens, scale=None, out=None, lse_out=None,
                         workspace=None, want_lse=False):
    """q [B,n_q,d_qk]; k_pool [n_pages,n_k,P,d_qk]; v_pool [n_pages,n_v,P,d_v]; block_table int32
    device [B,max_pages]; seqlens int32 device [B]."""
    _dev(q, k_pool, v_pool, block_table, seqlens, out, lse_out, workspace)
    dt = _dtype_code(q)
    if _dtype_code(k_pool) != dt or _dtype_code(v_pool) != dt:
        raise TypeError("q, k_pool and v_pool must share a dtype")
    if not q.is_contiguous() or not block_table.is_contiguous() or not seqlens.is_contiguous():
        raise ValueError("q, block_table and seqlens must be contiguous")
    if block_table.dtype != torch.int32 or seqlens.dtype != torch.int32:
        raise TypeError("block_table and seqlens must be int32")
    B, n_q, d_qk = q.shape
    _, n_k, P, _ = k_pool.shape
    _, n_v, _, d_v = v_pool.shape
    if k_pool.stride(3) != 1 or v_pool.stride(3) != 1:
        raise ValueError("the channel dimension of the pools must be contiguous")
    max_pages = block_table.shape[1]
    if out is None:
        out = torch.empty((B, n_q, d_v), dtype=q.dtype, device=q.device)
    if lse_out is None and want_lse:
        lse_out = torch.empty((B, n_q), dtype=torch.float32, device=q.device)
    s = _shape(B, n_q, n_k, n_v, d_qk, d_v, dt, scale)
    lib = load_library()
    need = int(lib.diffqkv_decode_workspace_bytes(ctypes.byref(s), int(max_pages * P)))
    workspace = _workspace(need, q, workspace)
    ks, vs = k_pool.stride(), v_pool.stride()
    _check(lib.diffqkv_decode_paged(
        ctypes.byref(s), _ptr(q), _ptr(k_pool), _ptr(v_pool), ks[0], ks[1], ks[2], vs[0], vs[1], vs[2],
        _ptr(block_table), int(max_pages), int(P), _ptr(seqlens), _ptr(out), _ptr(lse_out),
        _ptr(workspace), workspace.numel(), _stream(q)))
    return (out, lse_out) if (want_lse or lse_out is not None) else out


def diffqkv_prefill(q, k, v, causal=True, scale=None, out=None, lse_out=None, want_lse=False):
    """q [B,n_q,S_q,d_qk]; k [B,n_k,S_k,d_qk]; v [B,n_v,S_k,d_v], contiguous."""
    _dev(q, k, v, out, lse_out)
    dt = _dtype_code(q)
    if _dtype_code(k) != dt or _dtype_code(v) != dt:
        raise TypeError("q, k and v must share a dtype")
    if not (q.is_contiguous() and k.is_contiguous() and v.is_contiguous()):
        raise ValueError("q, k and v must be contiguous")
    B, n_q, S_q, d_qk = q.shape
    _, n_k, S_k, _ = k.shape
    _, n_v, _, d_v = v.shape
    if out is None:
        out = torch.empty((B, n_q, S_q, d_v), dtype=q.dtype, device=q.device)
    if lse_out is None and want_lse:
        lse_out = torch.empty((B, n_q, S_q), dtype=torch.float32, device=q.device)
    s = _shape(B, n_q, n_k, n_v, d_qk, d_v, dt, scale)
    _check(load_library().diffqkv_prefill(
        ctypes.byref(s), _ptr(q), _ptr(k), _ptr(v), int(S_q), int(S_k), 1 if causal else 0, _ptr(out),
        _ptr(lse_out), None, 0, _stream(q)))
    return (out, lse_out) if (want_lse or lse_out is not None) else out


def diffqkv_decode_topk(q, k_cache, v_cache, top_k, seqlens=None, T=None, scale=None, renormalize=True, out=None,
                        workspace=None, want_lse=False, want_selection=False):
    """Decode with selective V fetching: softmax over all positions, output from the top_k previous
    positions of largest weight plus the current token.  Returns out[, lse][, selection]."""
    _dev(q, k_cache, v_cache, seqlens, out, workspace)
    dt = _dtype_code(q)
    if _dtype_code(k_cache) != dt or _dtype_code(v_cache) != dt:
        raise TypeError("q, k_cache and v_cache must share a dtype")
    if not q.is_contiguous():
        raise ValueError("q must be contiguous")
    B, n_q, d_qk = q.shape
    _, n_k, T_cap, _ = k_cache.shape
    _, n_v, _, d_v = v_cache.shape
    if T is None:
        T = T_cap
    if T > T_cap:
        raise ValueError("T exceeds the cache capacity")
    if seqlens is not None and (seqlens.dtype != torch.int32 or not seqlens.is_contiguous()):
        raise TypeError("seqlens must be a contiguous int32 tensor")
    if out is None:
        out = torch.empty((B, n_q, d_v), dtype=q.dtype, device=q.device)
    lse = torch.empty((B, n_q), dtype=torch.float32, device=q.device) if want_lse else None
    sel = torch.empty((B, n_q, top_k + 1), dtype=torch.int32, device=q.device) if want_selection else None
    s = _shape(B, n_q, n_k, n_v, d_qk, d_v, dt, scale)
    lib = load_library()
    need = int(lib.diffqkv_decode_topk_workspace_bytes(ctypes.byref(s), int(T)))
    workspace = _workspace(need, q, workspace)
    ks, vs = k_cache.stride(), v_cache.stride()
    _check(lib.diffqkv_decode_topk(
        ctypes.byref(s), _ptr(q), _ptr(k_cache), _ptr(v_cache), ks[0], ks[1], ks[2], vs[0], vs[1], vs[2],
        _ptr(seqlens), int(T), int(top_k), 1 if renormalize else 0, _ptr(out), _ptr(lse), _ptr(sel),
        _ptr(workspace), workspace.numel(), _stream(q)))
    res = [out] + ([lse] if want_lse else []) + ([sel] if want_selection else [])
    return res[0] if len(res) == 1 else tuple(res)


def diffqkv_decode_topk_paged(q, k_pool, v_pool, block_table, seqlens, top_k, scale=None, renormalize=True,
                              out=None, workspace=None, want_lse=False, want_selection=False):
    """Paged variant of diffqkv_decode_topk."""
    _dev(q, k_pool, v_pool, block_table, seqlens, out, workspace)
    dt = _dtype_code(q)
    if _dtype_code(k_pool) != dt or _dtype_code(v_pool) != dt:
        raise TypeError("q, k_pool and v_pool must share a dtype")
    if not q.is_contiguous() or not block_table.is_contiguous() or not seqlens.is_contiguous():
        raise ValueError("q, block_table and seqlens must be contiguous")
    if block_table.dtype != torch.int32 or seqlens.dtype != torch.int32:
        raise TypeError("block_table and seqlens must be int32")
    B, n_q, d_qk = q.shape
    _, n_k, P, _ = k_pool.shape
    _, n_v, _, d_v = v_pool.shape
    max_pages = block_table.shape[1]
    if out is None:
        out = torch.empty((B, n_q, d_v), dtype=q.dtype, device=q.device)
    lse = torch.empty((B, n_q), dtype=torch.float32, device=q.device) if want_lse else None
    sel = torch.empty((B, n_q, top_k + 1), dtype=torch.int32, device=q.device) if want_selection else None
    s = _shape(B, n_q, n_k, n_v, d_qk, d_v, dt, scale)
    lib = load_library()
    need = int(lib.diffqkv_decode_topk_workspace_bytes(ctypes.byref(s), int(max_pages * P)))
    workspace = _workspace(need, q, workspace)
    ks, vs = k_pool.stride(), v_pool.stride()
    _check(lib.diffqkv_decode_topk_paged(
        ctypes.byref(s), _ptr(q), _ptr(k_pool), _ptr(v_pool), ks[0], ks[1], ks[2], vs[0], vs[1], vs[2],
        _ptr(block_table), int(max_pages), int(P), _ptr(seqlens), int(top_k), 1 if renormalize else 0, _ptr(out),
        _ptr(lse), _ptr(sel), _ptr(workspace), workspace.numel(), _stream(q)))
    res = [out] + ([lse] if want_lse else []) + ([sel] if want_selection else [])
    return res[0] if len(res) == 1 else tuple(res)


def diffqkv_append(k_new, v_new, k_cache, v_cache, positions, seqlens_out=None):
    """k_new [B,n_k,d_qk], v_new [B,n_v,d_v] written into row positions[b] of k_cache [B,n_k,T_cap,d_qk]
    and v_cache [B,n_v,T_cap,d_v] (in place).  positions: int32 device [B]."""
    _dev(k_new, v_new, k_cache, v_cache, positions, seqlens_out)
    dt = _dtype_code(k_cache)
    if _dtype_code(k_new) != dt or _dtype_code(v_new) != dt or _dtype_code(v_cache) != dt:
        raise TypeError("k_new, v_new and the caches must share a dtype")
    if not (k_new.is_contiguous() and v_new.is_contiguous() and positions.is_contiguous()):
        raise ValueError("k_new, v_new and positions must be contiguous")
    if positions.dtype != torch.int32 or (seqlens_out is not None and seqlens_out.dtype != torch.int32):
        raise TypeError("positions and seqlens_out must be int32")
    B, n_k, T_cap, d_qk = k_cache.shape
    _, n_v, _, d_v = v_cache.shape
    if tuple(k_new.shape) != (B, n_k, d_qk) or tuple(v_new.shape) != (B, n_v, d_v):
        raise ValueError("k_new / v_new do not match the caches")
    if k_cache.stride(3) != 1 or v_cache.stride(3) != 1:
        raise ValueError("the channel dimension of the caches must be contiguous")
    n_q = n_k * n_v  # any common multiple: the append does not involve query heads
    s = _shape(B, n_q, n_k, n_v, d_qk, d_v, dt, None)
    ks, vs = k_cache.stride(), v_cache.stride()
    _check(load_library().diffqkv_append(
        ctypes.byref(s), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache), ks[0], ks[1], ks[2], vs[0], vs[1],
        vs[2], _ptr(positions), int(T_cap), _ptr(seqlens_out), _stream(k_cache)))


def diffqkv_append_paged(k_new, v_new, k_pool, v_pool, block_table, positions, seqlens_out=None):
    """Paged variant: k_pool [n_pages,n_k,P,d_qk], v_pool [n_pages,n_v,P,d_v], block_table int32 [B,max_pages]."""
    _dev(k_new, v_new, k_pool, v_pool, block_table, positions, seqlens_out)
    dt = _dtype_code(k_pool)
    if _dtype_code(k_new) != dt or _dtype_code(v_new) != dt or _dtype_code(v_pool) != dt:
        raise TypeError("k_new, v_new and the pools must share a dtype")
    if not (k_new.is_contiguous() and v_new.is_contiguous() and positions.is_contiguous()
            and block_table.is_contiguous()):
        raise ValueError("k_new, v_new, positions and block_table must be contiguous")
    if positions.dtype != torch.int32 or block_table.dtype != torch.int32:
        raise TypeError("positions and block_table must be int32")
    _, n_k, P, d_qk = k_pool.shape
    _, n_v, _, d_v = v_pool.shape
    B, max_pages = block_table.shape
    if tuple(k_new.shape) != (B, n_k, d_qk) or tuple(v_new.shape) != (B, n_v, d_v):
        raise ValueError("k_new / v_new do not match the pools")
    s = _shape(B, n_k * n_v, n_k, n_v, d_qk, d_v, dt, None)
    ks, vs = k_pool.stride(), v_pool.stride()
    _check(load_library().diffqkv_append_paged(
        ctypes.byref(s), _ptr(k_new), _ptr(v_new), _ptr(k_pool), _ptr(v_pool), ks[0], ks[1], ks[2], vs[0], vs[1],
        vs[2], _ptr(block_table), int(max_pages), int(P), _ptr(positions), _ptr(seqlens_out), _stream(k_pool)))


def diffqkv_probe_stream_read(buf: torch.Tensor, sink: torch.Tensor):
    """Launch the stream-read probe over `buf` (any dtype, byte size a multiple of 16)."""
    _dev(buf, sink)
    nbytes = buf.numel() * buf.element_size()
    assert sink.dtype == torch.float32 and sink.numel() >= 4096
    _check(load_library().diffqkv_probe_stream_read(_ptr(buf), nbytes, _ptr(sink), _stream(buf)))


def diffqkv_augment_q(q_in, w_gate, w_up, w_down, out=None, workspace=None):
    """Augmented Q: q_in [M, hidden] -> W_down(silu(W_gate q_in) * (W_up q_in)) [M, hidden].
    w_gate, w_up [inter, hidden]; w_down [hidden, inter]; all contiguous, one dtype."""
    _dev(q_in, w_gate, w_up, w_down, out, workspace)
    dt = _dtype_code(q_in)
    if any(_dtype_code(w) != dt for w in (w_gate, w_up, w_down)):
        raise TypeError("q_in and the weights must share a dtype")
    if not all(t.is_contiguous() for t in (q_in, w_gate, w_up, w_down)):
        raise ValueError("q_in and the weights must be contiguous")
    M, hidden = q_in.shape
    inter = w_gate.shape[0]
    if tuple(w_gate.shape) != (inter, hidden) or tuple(w_up.shape) != (inter, hidden) or \
            tuple(w_down.shape) != (hidden, inter):
        raise ValueError("weight shapes do not match q_in")
    if out is None:
        out = torch.empty_like(q_in)
    elif tuple(out.shape) != (M, hidden) or out.dtype != q_in.dtype or not out.is_contiguous():
        raise ValueError("out must be a contiguous [M, hidden] tensor of the input dtype")
    lib = load_library()
    s = AugqShape(int(M), int(hidden), int(inter), dt)
    need = int(lib.diffqkv_augment_q_workspace_bytes(ctypes.byref(s)))
    ws = _workspace(need, q_in, workspace)
    _check(lib.diffqkv_augment_q(ctypes.byref(s), _ptr(q_in), _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(out),
                                 _ptr(ws), ws.numel() * ws.element_size(), _stream(q_in)))
    return out
