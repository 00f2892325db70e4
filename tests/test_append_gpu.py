"""GPU parity: diffqkv_append / diffqkv_append_paged against the oracle's plain copies (bit exact)."""
import numpy as np
import pytest
import torch

import oracle
import util
from paper_2501_13629_amd import binding, inputs

pytestmark = pytest.mark.gpu


def bits(t):
    return inputs.as_numpy(t.cpu())


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("heads", [(4, 16, 64, 64), (2, 8, 128, 128), (4, 2, 64, 128), (1, 1, 8, 256)])
def test_append_contiguous_bit_exact(dtype, heads):
    n_k, n_v, d_qk, d_v = heads
    n_q = max(n_k, n_v) * 2
    cfg = inputs.config("decode_4k", B=5, n_q=n_q, n_k=n_k, n_v=n_v, d_qk=d_qk, d_v=d_v, T=70, dtype=dtype, index=80)
    d = inputs.make_decode(cfg)
    new = inputs.make_decode(inputs.config("decode_4k", B=5, n_q=n_q, n_k=n_k, n_v=n_v, d_qk=d_qk, d_v=d_v, T=1,
                                           dtype=dtype, index=81))
    k_new, v_new = new["k"][:, :, 0].contiguous(), new["v"][:, :, 0].contiguous()
    pos = torch.tensor([0, 69, 33, 70, -1], dtype=torch.int32)  # the last two are out of range
    k, v = d["k"].cuda(), d["v"].cuda()
    sl = torch.full((5,), -7, dtype=torch.int32, device="cuda")
    binding.diffqkv_append(k_new.cuda(), v_new.cuda(), k, v, pos.cuda(), seqlens_out=sl)
    torch.cuda.synchronize()
    rk, rv = oracle.append(bits(k_new), bits(v_new), bits(d["k"]), bits(d["v"]), pos.numpy())
    assert np.array_equal(bits(k), rk) and np.array_equal(bits(v), rv)
    assert sl.cpu().tolist() == [1, 70, 34, -7, -7]
    # token-major cache through strides, positions updated in place
    k_tm = d["k"].cuda().permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    v_tm = d["v"].cuda().permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    p2 = pos.cuda().clone()
    binding.diffqkv_append(k_new.cuda(), v_new.cuda(), k_tm, v_tm, p2, seqlens_out=p2)
    assert np.array_equal(bits(k_tm.contiguous()), rk) and np.array_equal(bits(v_tm.contiguous()), rv)
    assert p2.cpu().tolist() == [1, 70, 34, 70, -1]


@pytest.mark.parametrize("page_size", [16, 4])
def test_append_paged_bit_exact_then_decode(page_size):
    cfg = inputs.config("paged_ragged", B=4, seqlens=[1, 15, 16, 333], page_size=page_size, index=82,
                        max_pages=400 // page_size)
    d = inputs.make_paged(cfg)
    n_pages = d["k_pool"].shape[0]
    # one spare page per sequence at the end of the pool, linked after the pages in use
    kp = torch.cat([d["k_pool"], torch.zeros((4,) + d["k_pool"].shape[1:], dtype=d["k_pool"].dtype)])
    vp = torch.cat([d["v_pool"], torch.zeros((4,) + d["v_pool"].shape[1:], dtype=d["v_pool"].dtype)])
    bt = d["block_table"].clone()
    for b in range(4):
        used = (int(d["seqlens"][b]) + page_size - 1) // page_size
        bt[b, used] = n_pages + b
    new = inputs.make_decode(inputs.config("decode_4k", B=4, n_q=32, n_k=4, n_v=16, d_qk=128, d_v=128, T=1, index=83))
    k_new, v_new = new["k"][:, :, 0].contiguous(), new["v"][:, :, 0].contiguous()
    pos = d["seqlens"].clone()
    kp_d, vp_d, sl = kp.cuda(), vp.cuda(), pos.cuda().clone()
    binding.diffqkv_append_paged(k_new.cuda(), v_new.cuda(), kp_d, vp_d, bt.cuda(), sl, seqlens_out=sl)
    torch.cuda.synchronize()
    rk, rv = oracle.append_paged(bits(k_new), bits(v_new), bits(kp), bits(vp), bt.numpy(), pos.numpy())
    assert np.array_equal(bits(kp_d), rk) and np.array_equal(bits(vp_d), rv)
    assert sl.cpu().tolist() == [int(x) + 1 for x in pos]
    # the appended token takes part in the next decode step
    out = binding.diffqkv_decode_paged(d["q"].cuda(), kp_d, vp_d, bt.cuda(), sl)
    ref, _ = oracle.decode_paged(bits(d["q"]), rk, rv, bt.numpy(), sl.cpu().numpy())
    util.check(out, ref, "bf16")
