"""Kernel-time sweep: DiffQKV (n_k = 4) against a grouped-query baseline (n_k = n_v = 16) on synthetic
tensors of Sigma-1.5B's attention shape.

    python -m paper_2501_13629_amd.ket_sweep [--batch 1] [--prefix 2048,4096,16384,32768,65536]

The paper's kernel-execution-time experiment (section 3.3, "KET Results"; appendix "Detailed
Efficiency Results") times its split and combine kernels on the trained model with n_q = 32,
n_v = 16, head width 64, for n_k = 4 (Sigma) and n_k = 16 (Std), over prefix lengths 2k-32k.  The
weights are not needed to time attention: this re-runs the same shapes on seeded random tensors and
reports, per prefix length, the average split and combine kernel times (HIP events attached to each
dispatch: the library's experimental kernel timer) and
the relative saving, next to the cost model's limit (32 - 20) / 32 = 37.5 % (section 3.1).
"""
import argparse
import json
import sys

import torch

from . import binding, inputs


def time_decode(cfg, steps=60, sets=4):
    host = inputs.make_decode(cfg)
    dev = torch.device("cuda:0")
    q = host["q"].to(dev)
    kv_bytes = cfg["B"] * cfg["T"] * inputs.kv_bytes_per_token(cfg)
    sets = max(2, min(sets, int(3e9 // max(kv_bytes, 1))))
    caches = [(host["k"].to(dev), host["v"].to(dev))]
    for _ in range(sets - 1):
        caches.append((caches[0][0].clone(), caches[0][1].clone()))
    out = torch.empty((cfg["B"], cfg["n_q"], cfg["d_v"]), dtype=q.dtype, device=dev)
    ws = torch.empty(max(256, binding.diffqkv_decode_workspace_bytes(
        cfg["B"], cfg["n_q"], cfg["n_k"], cfg["n_v"], cfg["d_qk"], cfg["d_v"], binding.BF16, cfg["T"])),
        dtype=torch.uint8, device=dev)
    for i in range(5):
        binding.diffqkv_decode(q, *caches[i % sets], out=out, workspace=ws)
    torch.cuda.synchronize()
    binding.diffqkv_kernel_timer(True)
    for i in range(steps):
        binding.diffqkv_decode(q, *caches[i % sets], out=out, workspace=ws)
    torch.cuda.synchronize()
    split, comb, _ = binding.diffqkv_kernel_timer_read()
    binding.diffqkv_kernel_timer(False)
    return split, comb, kv_bytes


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--prefix", default="2048,4096,16384,32768,65536")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("ket_sweep needs a GPU", file=sys.stderr)
        sys.exit(2)
    binding.load_library()
    rows = []
    for T in [int(x) for x in args.prefix.split(",")]:
        res = {}
        for name, n_k in (("std", 16), ("sigma", 4)):
            cfg = inputs.config("decode_4k", B=args.batch, n_q=32, n_k=n_k, n_v=16, d_qk=64, d_v=64, T=T, index=90)
            res[name] = time_decode(cfg)
        s_std, c_std, b_std = res["std"]
        s_sig, c_sig, b_sig = res["sigma"]
        rows.append({
            "prefix": T, "batch": args.batch,
            "split_us_std": round(s_std, 2), "split_us_sigma": round(s_sig, 2),
            "combine_us_std": round(c_std, 2), "combine_us_sigma": round(c_sig, 2),
            "split_gain": round(1 - s_sig / s_std, 4), "total_gain": round(1 - (s_sig + c_sig) / (s_std + c_std), 4),
            "bytes_ratio": round(b_sig / b_std, 4),
            "split_GBps_std": round(b_std / s_std / 1e3, 1), "split_GBps_sigma": round(b_sig / s_sig / 1e3, 1),
        })
        print(json.dumps(rows[-1]), flush=True)
    print(json.dumps({"limit_gain_cost_model": 0.375, "rows": len(rows)}))


if __name__ == "__main__":
    main()
