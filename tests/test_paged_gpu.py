"""GPU parity: diffqkv_decode_paged against the float64 oracle."""
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


def oracle_paged(d, rows=None):
    sel = slice(None) if rows is None else rows
    return oracle.decode_paged(inputs.as_numpy(d["q"])[sel], inputs.as_numpy(d["k_pool"]), inputs.as_numpy(d["v_pool"]),
                               d["block_table"].numpy()[sel], d["seqlens"].numpy()[sel])


def gpu_paged(d, **kw):
    return binding.diffqkv_decode_paged(util.dev(d["q"]), util.dev(d["k_pool"]), util.dev(d["v_pool"]),
                                        util.dev(d["block_table"]), util.dev(d["seqlens"]), want_lse=True, **kw)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("page_size", [16, 32, 64, 4])
@pytest.mark.parametrize("heads", [(32, 4, 16, 128), (32, 2, 8, 128), (32, 4, 16, 64), (8, 2, 2, 64)])
def test_small_paged(dtype, page_size, heads):
    n_q, n_k, n_v, d = heads
    cfg = inputs.config("paged_ragged", B=7, n_q=n_q, n_k=n_k, n_v=n_v, d_qk=d, d_v=d, page_size=page_size,
                        dtype=dtype, seqlens=[1, 15, 16, 17, 700, 1029, 2304], index=40 + page_size)
    d_ = inputs.make_paged(cfg)
    out, lse = gpu_paged(d_)
    ref, ref_lse = oracle_paged(d_)
    util.check(out, ref, dtype, str(cfg))
    util.check_lse(lse, ref_lse)


def test_paged_equals_contiguous_on_gpu():
    """Same tokens through a permuted page pool and through a contiguous cache: same numbers
    (identical split plan, identical arithmetic order => bit-identical)."""
    cfg = inputs.config("paged_ragged", B=4, seqlens=[2048, 777, 1, 2047], index=50)
    d = inputs.make_paged(cfg)
    P, T_cap = 16, 2048
    kp, vp, bt = util.dev(d["k_pool"]), util.dev(d["v_pool"]), d["block_table"]
    kc = torch.zeros(4, 4, T_cap, 128, dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros(4, 16, T_cap, 128, dtype=torch.bfloat16, device="cuda")
    for b in range(4):
        n = (int(d["seqlens"][b]) + P - 1) // P
        pages = bt[b, :n].long().cuda()
        kc[b, :, : n * P] = kp[pages].permute(1, 0, 2, 3).reshape(4, n * P, 128)
        vc[b, :, : n * P] = vp[pages].permute(1, 0, 2, 3).reshape(16, n * P, 128)
    a, _ = gpu_paged(d)
    b_ = binding.diffqkv_decode(util.dev(d["q"]), kc, vc, seqlens=util.dev(d["seqlens"]), T=T_cap)
    assert torch.equal(a.view(torch.int16), b_.view(torch.int16))


def test_poisoned_page_tails_and_unused_pages():
    cfg = inputs.config("paged_ragged", B=3, seqlens=[5, 100, 1000], index=51, max_pages=80)
    d = inputs.make_paged(cfg)
    clean, _ = gpu_paged(d)
    kp, vp = util.dev(d["k_pool"]).clone(), util.dev(d["v_pool"]).clone()
    for b in range(3):
        T = int(d["seqlens"][b])
        last_page = int(d["block_table"][b, (T - 1) // 16])
        kp[last_page, :, T % 16 if T % 16 else 16:] = float("nan")
        vp[last_page, :, T % 16 if T % 16 else 16:] = float("nan")
    d2 = dict(d, k_pool=kp, v_pool=vp)
    dirty, _ = gpu_paged(d2)
    assert torch.equal(clean.view(torch.int16), dirty.view(torch.int16))
    util.check(dirty, oracle_paged(d)[0], "bf16")


def test_config4_ragged_paged_full():
    """The full ragged workload in the default launch configuration (the one bench.py times): every one
    of the 64 sequences is compared with the oracle, element by element, against the same pool."""
    cfg = inputs.config("paged_ragged")
    d = inputs.make_paged(cfg)
    out, lse = gpu_paged(d)
    torch.cuda.synchronize()
    ref, ref_lse = oracle_paged(d)
    assert ref.shape[0] == cfg["B"] == 64
    util.check(out, ref, "bf16", "all %d sequences" % cfg["B"])
    util.check_lse(lse, ref_lse)
