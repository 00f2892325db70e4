"""GPU parity: decode with selective V-cache fetching (top-k) against the float64 oracle."""
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


def weights64(d, b, h, T, scale):
    """float64 softmax weights of one (sequence, head), to judge near-ties at the selection boundary."""
    import brute

    q, k = brute.bf16_bits_to_f64(inputs.as_numpy(d["q"])), None
    n_q, n_k = d["q"].shape[1], d["k"].shape[1]
    kk = brute.bf16_bits_to_f64(inputs.as_numpy(d["k"][b, h // (n_q // n_k), :T]))
    s = scale * (kk @ q[b, h])
    a = np.exp(s - s.max())
    return a / a.sum()


def check_selection(sel_gpu, sel_ref, d, seqlens, scale):
    """Same set, except that positions whose weights are equal to rounding may swap."""
    B, n_q, _ = sel_gpu.shape
    for b in range(B):
        for h in range(n_q):
            g = set(int(x) for x in sel_gpu[b, h] if x >= 0)
            r = set(int(x) for x in sel_ref[b, h] if x >= 0)
            assert len(g) == len(r), (b, h, len(g), len(r))
            if g != r:
                a = weights64(d, b, h, int(seqlens[b]), scale)
                only_g, only_r = sorted(g - r), sorted(r - g)
                for i, j in zip(only_g, only_r):
                    assert abs(a[i] - a[j]) <= 1e-5 * max(a[i], a[j]), (b, h, i, j, a[i], a[j])


def run(cfg, top_k, renorm, seqlens=None, force_generic=False):
    d = inputs.make_decode(cfg)
    if seqlens is not None:
        d["seqlens"] = torch.tensor(seqlens, dtype=torch.int32)
    binding.diffqkv_set_tuning(force_generic=force_generic)
    out, lse, sel = binding.diffqkv_decode_topk(util.dev(d["q"]), util.dev(d["k"]), util.dev(d["v"]), top_k,
                                                seqlens=util.dev(d["seqlens"]), renormalize=renorm, want_lse=True,
                                                want_selection=True)
    torch.cuda.synchronize()
    sl = None if d["seqlens"] is None else d["seqlens"].numpy()
    ref, ref_lse, ref_sel = oracle.decode_topk(inputs.as_numpy(d["q"]), inputs.as_numpy(d["k"]),
                                               inputs.as_numpy(d["v"]), top_k, seqlens=sl, renormalize=renorm)
    util.check(out, ref, cfg["dtype"], "top_k=%d renorm=%s %s" % (top_k, renorm, cfg))
    util.check_lse(lse, ref_lse)
    lens = sl if sl is not None else np.full(cfg["B"], cfg["T"])
    check_selection(sel.cpu().numpy(), ref_sel, d, lens, oracle.default_scale(cfg["d_qk"]))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("heads", [(32, 4, 16, 64, 64), (32, 2, 8, 128, 128), (8, 2, 2, 64, 128), (8, 4, 2, 64, 64),
                                   (32, 1, 2, 64, 64)])
@pytest.mark.parametrize("renorm", [False, True])
def test_small_shapes(dtype, heads, renorm):
    n_q, n_k, n_v, d_qk, d_v = heads
    for T, top_k in ((1, 4), (2, 0), (40, 100), (300, 7), (1500, 100), (2500, 100), (2500, 512)):
        cfg = inputs.config("decode_4k", B=2, n_q=n_q, n_k=n_k, n_v=n_v, d_qk=d_qk, d_v=d_v, T=T, dtype=dtype,
                            index=120 + T % 89)
        run(cfg, top_k, renorm)


def test_ragged_lengths():
    cfg = inputs.config("decode_32k", B=6, T=1300, index=121)
    run(cfg, 100, False, seqlens=[0, 1, 2, 101, 102, 1300])
    run(cfg, 100, True, seqlens=[1300, 555, 0, 100, 3, 129], force_generic=True)


def test_covering_top_k_equals_full_decode():
    cfg = inputs.config("decode_4k", B=2, T=400, index=122)
    d = inputs.make_decode(cfg)
    q, k, v = util.dev(d["q"]), util.dev(d["k"]), util.dev(d["v"])
    full = binding.diffqkv_decode(q, k, v)
    for renorm in (False, True):
        sel = binding.diffqkv_decode_topk(q, k, v, 512, renormalize=renorm)
        assert float((sel.float() - full.float()).abs().max()) <= 2e-2
    util.check(sel, util.oracle_decode(d)[0], "bf16")


def test_ties_go_to_the_lower_position():
    """Identical K rows give bit-identical scores: the winners must be the first top_k positions."""
    cfg = inputs.config("decode_4k", B=2, n_q=8, n_k=2, n_v=4, d_qk=64, d_v=64, T=700, index=123)
    d = inputs.make_decode(cfg)
    d["k"][:] = d["k"][:, :, :1]
    q, k, v = util.dev(d["q"]), util.dev(d["k"]), util.dev(d["v"])
    out, sel = binding.diffqkv_decode_topk(q, k, v, 33, want_selection=True)
    want = sorted(list(range(33)) + [699])
    for row in sel.cpu().numpy().reshape(-1, 34):
        assert sorted(int(x) for x in row) == want
    ref, _, _ = oracle.decode_topk(inputs.as_numpy(d["q"]), inputs.as_numpy(d["k"]), inputs.as_numpy(d["v"]), 33)
    util.check(out, ref, "bf16")


def test_thousands_of_ties_take_the_exact_fallback():
    """More equal scores than the candidate buffer of the select kernel holds: the exact radix select over
    the whole row takes over, and the lower positions still win."""
    cfg = inputs.config("decode_4k", B=1, n_q=8, n_k=2, n_v=4, d_qk=64, d_v=64, T=6000, index=125)
    d = inputs.make_decode(cfg)
    d["k"][:] = d["k"][:, :, :1]
    d["k"][:, :, 4500] = d["k"][:, :, 4500] * 0 + d["q"][:, :2]  # one row that differs: larger or smaller score
    q, k, v = util.dev(d["q"]), util.dev(d["k"]), util.dev(d["v"])
    out, sel = binding.diffqkv_decode_topk(q, k, v, 100, want_selection=True)
    ref, _, ref_sel = oracle.decode_topk(inputs.as_numpy(d["q"]), inputs.as_numpy(d["k"]), inputs.as_numpy(d["v"]), 100)
    for g, r in zip(sel.cpu().numpy().reshape(-1, 101), ref_sel.reshape(-1, 101)):
        assert sorted(int(x) for x in g) == sorted(int(x) for x in r)
    util.check(out, ref, "bf16")


def test_rows_longer_than_the_register_resident_part():
    """Above 32768 previous positions the select kernel reads the score row twice."""
    cfg = inputs.config("decode_4k", B=1, n_q=8, n_k=2, n_v=4, d_qk=64, d_v=64, T=40000, index=126)
    run(cfg, 100, False)
    run(cfg, 512, True, seqlens=[32770])


def test_bitwise_repeatable():
    """Counting in the select kernel uses integer LDS atomics, whose order varies; the selection, the order
    of the weighted sum and so every output bit do not."""
    cfg = inputs.config("decode_32k", B=2, T=5000, index=127)
    d = inputs.make_decode(cfg)
    q, k, v = util.dev(d["q"]), util.dev(d["k"]), util.dev(d["v"])
    out, lse, sel = binding.diffqkv_decode_topk(q, k, v, 100, want_lse=True, want_selection=True)
    a, b, c = out.view(torch.int16).clone(), lse.view(torch.int32).clone(), sel.clone()
    for _ in range(3):
        out, lse, sel = binding.diffqkv_decode_topk(q, k, v, 100, want_lse=True, want_selection=True)
        assert torch.equal(a, out.view(torch.int16)) and torch.equal(b, lse.view(torch.int32)) and torch.equal(c, sel)


@pytest.mark.parametrize("page_size", [16, 4])
def test_paged(page_size):
    cfg = inputs.config("paged_ragged", B=5, seqlens=[1, 17, 700, 1029, 2304], page_size=page_size, index=124)
    d = inputs.make_paged(cfg)
    out, sel = binding.diffqkv_decode_topk_paged(util.dev(d["q"]), util.dev(d["k_pool"]), util.dev(d["v_pool"]),
                                                 util.dev(d["block_table"]), util.dev(d["seqlens"]), 100,
                                                 want_selection=True)
    # the oracle works on the contiguous view of the same tokens
    import brute

    sl = d["seqlens"].numpy()
    kc = brute.gather_paged(inputs.as_numpy(d["k_pool"]), d["block_table"].numpy(), sl, 2304)
    vc = brute.gather_paged(inputs.as_numpy(d["v_pool"]), d["block_table"].numpy(), sl, 2304)
    ref, _, ref_sel = oracle.decode_topk(inputs.as_numpy(d["q"]), kc, vc, 100, seqlens=sl)
    util.check(out, ref, "bf16")
    contiguous = {"q": d["q"], "k": torch.from_numpy(kc.view(np.int16)).view(torch.bfloat16)}
    check_selection(sel.cpu().numpy(), ref_sel, contiguous, sl, oracle.default_scale(cfg["d_qk"]))


def test_config3_shape_top100_full():
    """Full 32k-context workload, top-100: all eight sequences against the oracle, outputs and selections."""
    cfg = inputs.config("decode_32k")
    d = inputs.make_decode(cfg)
    out, lse, sel = binding.diffqkv_decode_topk(util.dev(d["q"]), util.dev(d["k"]), util.dev(d["v"]), 100,
                                                want_lse=True, want_selection=True)
    torch.cuda.synchronize()
    ref, ref_lse, ref_sel = oracle.decode_topk(inputs.as_numpy(d["q"]), inputs.as_numpy(d["k"]),
                                               inputs.as_numpy(d["v"]), 100)
    util.check(out, ref, "bf16", "all %d sequences" % cfg["B"])
    util.check_lse(lse, ref_lse)
    check_selection(sel.cpu().numpy(), ref_sel, d, np.full(cfg["B"], cfg["T"]), oracle.default_scale(cfg["d_qk"]))
