"""Host-side checks of the C ABI: the library loads, exports every symbol the header declares, and
its argument validation returns the documented status codes without touching a GPU."""
import ctypes
import os
import re

import pytest

from paper_2501_13629_amd import binding
from paper_2501_13629_amd.binding import Shape

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

OK, E_NULL, E_SHAPE, E_HEADS, E_ALIGN, E_WS, E_UNSUPPORTED = 0, -1, -2, -3, -4, -5, -6


@pytest.fixture(scope="module")
def lib():
    if not binding.LIB_PATH.exists():
        from paper_2501_13629_amd import build

        build.build()
    return binding.load_library()


def declared_functions(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(diffqkv_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    product, experimental = declared_functions("diffqkv.h"), declared_functions("diffqkv_experimental.h")
    assert len(product) >= 12 and len(experimental) == 4
    for name in product + experimental:
        assert hasattr(lib, name), name
    assert set(product) == set(binding.EXPORTS)
    assert set(experimental) == set(binding.EXPERIMENTAL_EXPORTS)
    # the product header declares no knob and no measurement aid
    assert not any(n in product for n in ("diffqkv_set_tuning", "diffqkv_kernel_timer", "diffqkv_probe_stream_read"))


def test_version_and_strerror(lib):
    assert lib.diffqkv_version() >= 100
    assert lib.diffqkv_strerror(0) == b"ok"
    for code in range(-8, 0):
        assert len(lib.diffqkv_strerror(code)) > 3


def shape(B=2, n_q=8, n_k=2, n_v=4, d_qk=64, d_v=64, dtype=1, scale=0.0):
    return Shape(B, n_q, n_k, n_v, d_qk, d_v, dtype, scale)


def decode(lib, s, q=0x1000, k=0x2000, v=0x3000, ks=(8192, 4096, 64), vs=(8192, 4096, 64), T=64, out=0x4000,
           ws=0x5000, ws_bytes=1 << 30):
    vp = ctypes.c_void_p
    return lib.diffqkv_decode(ctypes.byref(s), vp(q), vp(k), vp(v), *ks, *vs, None, T, vp(out), None, vp(ws),
                              ws_bytes, None)


def test_decode_validation_codes(lib):
    vp = ctypes.c_void_p
    assert lib.diffqkv_decode(None, vp(16), vp(16), vp(16), 64, 64, 64, 64, 64, 64, None, 1, vp(16), None, None, 0,
                              None) == E_NULL
    assert decode(lib, shape(n_q=0)) == E_SHAPE
    assert decode(lib, shape(d_qk=60)) == E_SHAPE
    assert decode(lib, shape(d_v=512)) == E_SHAPE
    assert decode(lib, shape(dtype=7)) == E_SHAPE
    assert decode(lib, shape(scale=-1.0)) == E_SHAPE
    assert decode(lib, shape(), T=-1) == E_SHAPE
    assert decode(lib, shape(n_q=8, n_k=3)) == E_HEADS
    assert decode(lib, shape(n_q=12, n_k=4, n_v=6)) == E_HEADS  # neither divides the other
    assert decode(lib, shape(), q=0) == E_NULL
    assert decode(lib, shape(), out=0) == E_NULL
    assert decode(lib, shape(), k=0x2004) == E_ALIGN
    assert decode(lib, shape(), ks=(8192, 4096, 60)) == E_ALIGN
    assert decode(lib, shape(), ks=(8192, 4096, 32)) == E_SHAPE  # rows would overlap
    # a context long enough to need splits needs a workspace
    s = shape(B=1)
    need = lib.diffqkv_decode_workspace_bytes(ctypes.byref(s), 1 << 16)
    assert need > 0
    assert decode(lib, s, T=1 << 16, ws=0) == E_WS
    assert decode(lib, s, T=1 << 16, ws_bytes=4096) == E_WS  # far below any plan for this shape
    # an empty batch is a valid no-op and launches nothing
    assert decode(lib, shape(B=0), q=0, k=0, v=0, out=0, ws=0, ws_bytes=0) == OK


def test_paged_and_prefill_validation_codes(lib):
    vp = ctypes.c_void_p
    s = shape()

    def paged(max_pages=4, page=16, seqlens=0x6000, bt=0x7000, kst=(4096, 1024, 64)):
        return lib.diffqkv_decode_paged(ctypes.byref(s), vp(0x1000), vp(0x2000), vp(0x3000), *kst, 4096, 1024, 64,
                                        vp(bt), max_pages, page, vp(seqlens), vp(0x4000), None, vp(0x5000),
                                        1 << 30, None)

    assert paged(page=0) == E_SHAPE
    assert paged(max_pages=-1) == E_SHAPE
    assert paged(max_pages=1 << 30, page=16) == E_SHAPE
    assert paged(seqlens=0) == E_NULL
    assert paged(bt=0) == E_NULL
    assert paged(kst=(4096, 1024, 68)) == E_ALIGN

    def prefill(S_q=16, S_k=16, causal=1, q=0x1000):
        return lib.diffqkv_prefill(ctypes.byref(s), vp(q), vp(0x2000), vp(0x3000), S_q, S_k, causal, vp(0x4000),
                                   None, None, 0, None)

    assert prefill(S_q=0) == E_SHAPE
    assert prefill(S_q=32, S_k=16) == E_SHAPE
    assert prefill(q=0) == E_NULL
    assert prefill(q=0x1008) == E_ALIGN


def test_topk_and_augmented_q_validation_codes(lib):
    vp = ctypes.c_void_p
    s = shape()

    def topk(top_k=100, T=64, q=0x1000, ws=0x5000, ws_bytes=1 << 30, kst=(8192, 4096, 64)):
        return lib.diffqkv_decode_topk(ctypes.byref(s), vp(q), vp(0x2000), vp(0x3000), *kst, 8192, 4096, 64, None, T,
                                       top_k, 0, vp(0x4000), None, None, vp(ws), ws_bytes, None)

    assert topk(top_k=-1) == E_SHAPE
    assert topk(top_k=513) == E_UNSUPPORTED  # valid, but more than the select kernel keeps in LDS
    assert topk(T=-1) == E_SHAPE
    assert topk(q=0) == E_NULL
    assert topk(q=0x1004) == E_ALIGN
    assert topk(kst=(8192, 4096, 32)) == E_SHAPE
    assert topk(ws=0) == E_WS
    assert topk(ws_bytes=64) == E_WS
    need = lib.diffqkv_decode_topk_workspace_bytes(ctypes.byref(s), 1000)
    assert need == 2 * 8 * 1024 * 4  # one fp32 score row per (sequence, query head), padded to 128 tokens

    A = binding.AugqShape

    def augq(a, q=0x1000, wd=0x4000, ws=0x6000, ws_bytes=1 << 30):
        return lib.diffqkv_augment_q(ctypes.byref(a), vp(q), vp(0x2000), vp(0x3000), vp(wd), vp(0x5000), vp(ws),
                                     ws_bytes, None)

    assert lib.diffqkv_augment_q(None, vp(16), vp(16), vp(16), vp(16), vp(16), vp(16), 0, None) == E_NULL
    assert augq(A(-1, 64, 96, 1)) == E_SHAPE
    assert augq(A(4, 0, 96, 1)) == E_SHAPE
    assert augq(A(4, 60, 96, 1)) == E_SHAPE  # rows must be whole 16-byte pieces
    assert augq(A(4, 64, 96, 5)) == E_SHAPE
    assert augq(A(4, 1 << 21, 1 << 21, 1)) == E_UNSUPPORTED  # a product of 2^42 weights
    assert augq(A(4, 64, 96, 1), q=0) == E_NULL
    assert augq(A(4, 64, 96, 1), wd=0x4008) == E_ALIGN
    assert augq(A(4, 64, 96, 1), ws=0) == E_WS
    assert augq(A(4, 64, 96, 1), ws_bytes=100) == E_WS
    assert augq(A(0, 64, 96, 1), q=0, ws=0, ws_bytes=0) == OK  # no tokens: a valid no-op
    a = A(16, 2048, 3072, 1)
    assert lib.diffqkv_augment_q_workspace_bytes(ctypes.byref(a)) == 16 * 3072 * 2
    a = A(3, 64, 96, 0)
    assert lib.diffqkv_augment_q_workspace_bytes(ctypes.byref(a)) == 16 * 96 * 4  # whole blocks of 16 tokens


def test_split_plan_is_a_function_of_shapes(lib):
    s = shape(B=8, n_q=32, n_k=2, n_v=8, d_qk=128, d_v=128)
    a = lib.diffqkv_decode_workspace_bytes(ctypes.byref(s), 32768)
    b = lib.diffqkv_decode_workspace_bytes(ctypes.byref(s), 32768)
    assert a == b and a % 256 == 0 and a > 0
    # short contexts run in a single pass and need no workspace
    assert lib.diffqkv_decode_workspace_bytes(ctypes.byref(s), 128) == 0
    # the figure covers the equal-slice plan for ragged calls: 1024 units of 32 tokens, smallest slice
    # 8 units (8 x 2 x 1024 units over 2048 wavefronts) => 129 partial slots per row, plus the prefix table
    assert a == 256 + 8 * 32 * 129 * 129 * 4
    # fixed-size chunks only: the knob changes the plan; resetting restores it
    binding.diffqkv_set_tuning(decode_ragged_mode=2)
    f = lib.diffqkv_decode_workspace_bytes(ctypes.byref(s), 32768)
    binding.diffqkv_set_tuning(decode_chunk_tokens=512, decode_ragged_mode=2)
    c = lib.diffqkv_decode_workspace_bytes(ctypes.byref(s), 32768)
    binding.diffqkv_set_tuning()
    assert f == 8 * 32 * 16 * 129 * 4 and c == 8 * 32 * 64 * 129 * 4
    assert lib.diffqkv_decode_workspace_bytes(ctypes.byref(s), 32768) == a


def test_knobs_are_per_thread_and_validation_runs_concurrently(lib):
    """Two threads validate decode calls at the same time, each under its own experimental knobs: the
    knobs of one thread never show in the other's split plan, and every call returns its own status."""
    import threading

    s = shape(B=8, n_q=32, n_k=2, n_v=8, d_qk=128, d_v=128)
    default = lib.diffqkv_decode_workspace_bytes(ctypes.byref(s), 32768)
    results, barrier = {}, threading.Barrier(2)

    def worker(name, chunk, want_bytes):
        binding.diffqkv_set_tuning(decode_chunk_tokens=chunk, decode_ragged_mode=2 if chunk else 0)
        barrier.wait()
        ok = True
        for i in range(2000):
            ok &= lib.diffqkv_decode_workspace_bytes(ctypes.byref(s), 32768) == want_bytes
            ok &= decode(lib, shape(n_q=8, n_k=3)) == E_HEADS
            ok &= decode(lib, shape(), T=-1) == E_SHAPE
            ok &= decode(lib, shape(), k=0x2004) == E_ALIGN
            ok &= decode(lib, shape(B=1), T=1 << 16, ws=0) == E_WS
            ok &= decode(lib, shape(B=0), q=0, k=0, v=0, out=0, ws=0, ws_bytes=0) == OK
        results[name] = ok
        binding.diffqkv_set_tuning()

    threads = [threading.Thread(target=worker, args=("chunk512", 512, 8 * 32 * 64 * 129 * 4)),
               threading.Thread(target=worker, args=("default", 0, default))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert results == {"chunk512": True, "default": True}
    assert lib.diffqkv_decode_workspace_bytes(ctypes.byref(s), 32768) == default  # this thread never set a knob


def test_static_decode_refuses_sizes_beyond_its_buffer(lib):
    """The entry point that allocates nothing checks the size before it touches a device."""
    s = shape(B=64, n_q=32, n_k=2, n_v=8, d_qk=128, d_v=128)
    assert lib.diffqkv_decode_workspace_bytes(ctypes.byref(s), 32768) > binding.STATIC_SCRATCH_BYTES
    vp = ctypes.c_void_p
    rc = lib.diffqkv_decode_static(ctypes.byref(s), vp(0x1000), vp(0x2000), vp(0x3000), 1 << 23, 1 << 22, 128,
                                   1 << 25, 1 << 22, 128, None, 32768, vp(0x4000), None, None)
    assert rc == -8 and b"static" in lib.diffqkv_strerror(rc)
    # an empty batch is a valid no-op here too
    e = shape(B=0)
    assert lib.diffqkv_decode_static(ctypes.byref(e), None, None, None, 64, 64, 64, 64, 64, 64, None, 16, None, None,
                                     None) == OK


def test_binding_refuses_cpu_tensors():
    import torch

    q = torch.zeros(1, 4, 64)
    k = torch.zeros(1, 1, 8, 64)
    v = torch.zeros(1, 2, 8, 64)
    with pytest.raises(RuntimeError, match="GPU only"):
        binding.diffqkv_decode(q, k, v)


def test_append_validation_codes(lib):
    vp = ctypes.c_void_p
    s = shape()

    def app(k_new=0x1000, pos=0x6000, kst=(8192, 4096, 64), cap=64, sh=s):
        return lib.diffqkv_append(ctypes.byref(sh), vp(k_new), vp(0x2000), vp(0x3000), vp(0x4000), *kst, 8192, 4096,
                                  64, vp(pos), cap, None, None)

    assert app(k_new=0) == E_NULL
    assert app(pos=0) == E_NULL
    assert app(cap=-1) == E_SHAPE
    assert app(kst=(8192, 4096, 60)) == E_ALIGN
    assert app(sh=shape(B=0)) == OK
    assert lib.diffqkv_append_paged(ctypes.byref(s), vp(0x1000), vp(0x2000), vp(0x3000), vp(0x4000), 4096, 1024, 64,
                                    4096, 1024, 64, vp(0x7000), 4, 0, vp(0x6000), None, None) == E_SHAPE
