"""GPU: diffqkv_decode_static -- the decode entry point that allocates nothing -- against diffqkv_decode.

The partial results of the context splits go to the library's static device buffer instead of a
caller's workspace.  Same kernels, same split plan: the outputs must be bit-identical to
diffqkv_decode's (and so inside the oracle tolerance, which is checked too), on two calls in a row that
share the buffer, the second one smaller.  Sizes beyond the buffer are refused."""
import ctypes

import pytest
import torch

import util
from paper_2501_13629_amd import binding, inputs

pytestmark = pytest.mark.gpu


def both(cfg, seqlens=None):
    d = inputs.make_decode(cfg)
    if seqlens is not None:
        d["seqlens"] = torch.tensor(seqlens, dtype=torch.int32)
    q, k, v, sl = util.dev(d["q"]), util.dev(d["k"]), util.dev(d["v"]), util.dev(d["seqlens"])
    ref, ref_lse = binding.diffqkv_decode(q, k, v, seqlens=sl, want_lse=True)
    out = torch.full_like(ref, float("nan"))
    lse = torch.full_like(ref_lse, float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    binding.diffqkv_decode_static(q, k, v, out, seqlens=sl, lse_out=lse)
    after = torch.cuda.memory_stats()["allocation.all.allocated"]
    torch.cuda.synchronize()
    assert after == before, "the binding of the static call must not allocate through torch either"
    assert torch.equal(out.view(torch.int16), ref.view(torch.int16)), str(cfg)
    assert torch.equal(lse.view(torch.int32), ref_lse.view(torch.int32)), str(cfg)
    oracle_out, oracle_lse = util.oracle_decode(d)
    util.check(out, oracle_out, cfg["dtype"], str(cfg))
    util.check_lse(lse, oracle_lse, str(cfg))


def test_two_calls_in_a_row_the_second_smaller():
    """Several splits per row in both calls; the second call's partials cover only a part of what the
    first one left in the shared buffer."""
    both(inputs.config("decode_32k", B=4, T=9000, index=201))
    both(inputs.config("decode_32k", B=2, T=3000 + 77, index=202))
    # ragged lengths (the equal-slice plan, with its prefix table at the front of the buffer), then a
    # context short enough for a single pass that touches no scratch at all
    both(inputs.config("decode_32k", B=5, T=9000, index=203), seqlens=[9000, 33, 4097, 0, 8191])
    both(inputs.config("decode_4k", B=3, T=100, index=204))
    both(inputs.config("tiny_fp32"))


def test_headline_shape_fits_and_matches():
    both(inputs.config("decode_32k"))


def test_sizes_beyond_the_static_buffer_are_refused():
    """B = 64 sequences of 32 query heads with 129 partial slots each need 136 MB: refused, nothing runs."""
    lib = binding.load_library()
    s = binding.Shape(64, 32, 2, 8, 128, 128, binding.BF16, 0.0)
    need = lib.diffqkv_decode_workspace_bytes(ctypes.byref(s), 32768)
    assert need > binding.STATIC_SCRATCH_BYTES
    vp = ctypes.c_void_p
    rc = lib.diffqkv_decode_static(ctypes.byref(s), vp(0x1000), vp(0x2000), vp(0x3000), 1 << 23, 1 << 22, 128,
                                   1 << 25, 1 << 22, 128, None, 32768, vp(0x4000), None, None)
    assert rc == -8
    assert b"static" in lib.diffqkv_strerror(rc)
