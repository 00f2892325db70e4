"""GPU parity: diffqkv_decode (through the C ABI) against the float64 oracle, element by element."""
import numpy as np
import pytest
import torch

import oracle
import util
from paper_2501_13629_amd import binding, inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _reset_tuning():
    binding.diffqkv_set_tuning()
    yield
    binding.diffqkv_set_tuning()


def run_case(cfg, force_generic=False, chunk=0, want_lse=True):
    d = inputs.make_decode(cfg)
    binding.diffqkv_set_tuning(decode_chunk_tokens=chunk, force_generic=force_generic)
    out, lse = binding.diffqkv_decode(util.dev(d["q"]), util.dev(d["k"]), util.dev(d["v"]),
                                      seqlens=util.dev(d["seqlens"]), want_lse=True)
    torch.cuda.synchronize()
    ref, ref_lse = util.oracle_decode(d)
    err = util.check(out, ref, cfg["dtype"], str(cfg))
    util.check_lse(lse, ref_lse, str(cfg))
    return err


def test_config1_tiny_fp32():
    run_case(inputs.config("tiny_fp32"))


# (n_q, n_k, n_v, d_qk, d_v): Sigma's shapes, plain GQA / MHA / MQA, n_k > n_v, wide groups, d_qk != d_v
SHAPES = [
    (32, 4, 16, 64, 64), (32, 2, 8, 128, 128), (32, 4, 16, 128, 128), (8, 2, 4, 128, 128), (8, 2, 2, 64, 64),
    (4, 4, 4, 64, 64), (16, 1, 1, 128, 128), (8, 4, 2, 64, 64), (32, 1, 2, 64, 64), (16, 2, 4, 64, 128),
    (16, 2, 8, 128, 64), (6, 3, 3, 128, 128), (24, 2, 4, 64, 64),
]
# context lengths spanning one sub-tile, ragged tails, several 128-token tiles and several splits
LENGTHS = [1, 17, 128, 129, 300, 1000, 2500]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_small_shapes(shape, dtype):
    n_q, n_k, n_v, d_qk, d_v = shape
    for T in LENGTHS:
        cfg = inputs.config("decode_4k", B=3, n_q=n_q, n_k=n_k, n_v=n_v, d_qk=d_qk, d_v=d_v, T=T, dtype=dtype,
                            index=100 + T % 97)
        run_case(cfg)


@pytest.mark.parametrize("shape", [(32, 4, 16, 64, 64), (32, 2, 8, 128, 128)])
def test_generic_kernel_matches_too(shape):
    n_q, n_k, n_v, d_qk, d_v = shape
    for T in (1, 129, 1000):
        cfg = inputs.config("decode_4k", B=2, n_q=n_q, n_k=n_k, n_v=n_v, d_qk=d_qk, d_v=d_v, T=T, index=7)
        run_case(cfg, force_generic=True)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_ragged_lengths_including_empty(dtype):
    cfg = inputs.config("decode_4k", B=6, T=700, dtype=dtype, index=11)
    d = inputs.make_decode(cfg)
    d["seqlens"] = torch.tensor([0, 1, 700, 255, 256, 257], dtype=torch.int32)
    for chunk in (0, 128):
        binding.diffqkv_set_tuning(decode_chunk_tokens=chunk)
        out, lse = binding.diffqkv_decode(util.dev(d["q"]), util.dev(d["k"]), util.dev(d["v"]),
                                          seqlens=util.dev(d["seqlens"]), want_lse=True)
        ref, ref_lse = util.oracle_decode(d)
        util.check(out, ref, dtype)
        util.check_lse(lse, ref_lse)
        assert torch.all(out[0] == 0) and torch.all(torch.isneginf(lse[0]))
    # single pass (one split) with an empty sequence
    d["seqlens"] = torch.tensor([0, 1, 100, 255, 13, 64], dtype=torch.int32)
    binding.diffqkv_set_tuning()
    out, lse = binding.diffqkv_decode(util.dev(d["q"]), util.dev(d["k"]), util.dev(d["v"]),
                                      seqlens=util.dev(d["seqlens"]), T=255, want_lse=True)
    ref, ref_lse = util.oracle_decode(d, T=255)
    util.check(out, ref, dtype)
    util.check_lse(lse, ref_lse)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_poisoned_tail_is_ignored(dtype):
    """Cache rows beyond T_b may hold NaN: the result must be bit-identical to a clean cache."""
    cfg = inputs.config("decode_4k", B=3, n_q=32, n_k=2, n_v=8, d_qk=128, d_v=128, T=600, dtype=dtype, index=12)
    d = inputs.make_decode(cfg)
    sl = torch.tensor([600, 333, 17], dtype=torch.int32)
    q, k, v = util.dev(d["q"]), util.dev(d["k"]), util.dev(d["v"])
    clean = binding.diffqkv_decode(q, k, v, seqlens=sl.cuda())
    kp, vp = k.clone(), v.clone()
    for b in range(3):
        kp[b, :, int(sl[b]):] = float("nan")
        vp[b, :, int(sl[b]):] = float("nan")
    dirty = binding.diffqkv_decode(q, kp, vp, seqlens=sl.cuda())
    assert torch.equal(clean.view(torch.int16 if dtype == "bf16" else torch.int32),
                       dirty.view(torch.int16 if dtype == "bf16" else torch.int32))
    d["seqlens"] = sl
    util.check(dirty, util.oracle_decode(d)[0], dtype)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_token_major_cache_through_strides(dtype):
    """The paper's cost model stores the cache as (b, s, n, d); the strides make that callable."""
    cfg = inputs.config("decode_4k", B=2, n_q=32, n_k=4, n_v=16, d_qk=64, d_v=64, T=515, dtype=dtype, index=13)
    d = inputs.make_decode(cfg)
    k_tm = util.dev(d["k"]).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)  # [B,n,T,d] view of [B,T,n,d]
    v_tm = util.dev(d["v"]).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert not k_tm.is_contiguous()
    out = binding.diffqkv_decode(util.dev(d["q"]), k_tm, v_tm)
    util.check(out, util.oracle_decode(d)[0], dtype)


def test_custom_scale_and_capacity_larger_than_T():
    cfg = inputs.config("decode_4k", B=2, T=900, index=14)
    d = inputs.make_decode(cfg)
    out = binding.diffqkv_decode(util.dev(d["q"]), util.dev(d["k"]), util.dev(d["v"]), T=777, scale=0.2)
    ref, _ = oracle.decode(inputs.as_numpy(d["q"]), inputs.as_numpy(d["k"]), inputs.as_numpy(d["v"]), T=777,
                           scale=float(np.float32(0.2)))
    util.check(out, ref, "bf16")


def test_bitwise_repeatable():
    cfg = inputs.config("decode_32k", B=2, T=5000, index=15)
    d = inputs.make_decode(cfg)
    q, k, v = util.dev(d["q"]), util.dev(d["k"]), util.dev(d["v"])
    a = binding.diffqkv_decode(q, k, v).view(torch.int16).clone()
    for _ in range(3):
        assert torch.equal(a, binding.diffqkv_decode(q, k, v).view(torch.int16))


def test_config2_decode_4k_full():
    run_case(inputs.config("decode_4k"))


def test_config3_decode_32k_full():
    """The headline workload at full size, default launch configuration (the one bench.py times)."""
    run_case(inputs.config("decode_32k"))


def test_half_k_decode_32k_full():
    """The 32k decode workload with K heads of half width (d_qk 64, d_v 128), default launch configuration."""
    run_case(inputs.config("decode_32k_halfk"))


def test_bytes_model_sanity_k_heads():
    """Fewer K heads must never make the answer depend on anything but the head map: the same
    K/V data seen through n_k = 16 (K duplicated per V head, the 'group sharing' workaround of the
    paper's appendix) gives the same output as n_k = 4."""
    cfg = inputs.config("decode_4k", B=2, T=1500, index=16)
    d = inputs.make_decode(cfg)
    q, k, v = util.dev(d["q"]), util.dev(d["k"]), util.dev(d["v"])
    a = binding.diffqkv_decode(q, k, v)
    k_exp = k.repeat_interleave(4, dim=1).contiguous()
    b = binding.diffqkv_decode(q, k_exp, v)
    ref = util.oracle_decode(d)[0]
    util.check(a, ref, "bf16")
    util.check(b, ref, "bf16")


@pytest.mark.parametrize("mode", [0, 2])
def test_ragged_many_sequences_both_plans(mode):
    """Many sequences of very uneven length (some empty), more than one sequence per thread in the
    prefix scan of the equal-slice plan; mode 2 forces fixed-size chunks on the same inputs."""
    B, T_cap = 301, 777
    cfg = inputs.config("decode_4k", B=B, n_q=16, n_k=2, n_v=4, d_qk=128, d_v=128, T=T_cap, index=17)
    d = inputs.make_decode(cfg)
    rng = np.random.default_rng(17)
    sl = rng.integers(0, T_cap + 1, size=B).astype(np.int32)
    sl[[0, 5, 300]] = [0, T_cap, 1]
    sl[100:140] = 0
    d["seqlens"] = torch.from_numpy(sl)
    binding.diffqkv_set_tuning(decode_ragged_mode=mode)
    out, lse = binding.diffqkv_decode(util.dev(d["q"]), util.dev(d["k"]), util.dev(d["v"]),
                                      seqlens=util.dev(d["seqlens"]), want_lse=True)
    ref, ref_lse = util.oracle_decode(d)
    util.check(out, ref, "bf16")
    util.check_lse(lse, ref_lse)
    assert torch.all(out[100:140] == 0)


def test_ragged_plans_agree_on_long_contexts():
    """A few long sequences: slices of the equal-slice plan cross sequence and head boundaries."""
    cfg = inputs.config("decode_32k", B=5, T=9000, index=18)
    d = inputs.make_decode(cfg)
    d["seqlens"] = torch.tensor([9000, 33, 4097, 0, 8191], dtype=torch.int32)
    ref, ref_lse = util.oracle_decode(d)
    for mode in (0, 2):
        binding.diffqkv_set_tuning(decode_ragged_mode=mode)
        out, lse = binding.diffqkv_decode(util.dev(d["q"]), util.dev(d["k"]), util.dev(d["v"]),
                                          seqlens=util.dev(d["seqlens"]), want_lse=True)
        util.check(out, ref, "bf16", "mode %d" % mode)
        util.check_lse(lse, ref_lse)
