#!/usr/bin/env python3
"""Per-call microbenchmark of the HBM- and MFMA-bound entry points of libllmc.so.

Runs llmc_fingerprint, llmc_match and llmc_gather_hits (through the C ABI) on synthetic
tensors of a given shape, a few times each, and prints one line per kernel with the
duration measured by the library's HIP events and the algorithmic GB/s or TFLOP/s.
It also performs a plain device-to-device copy of known size: when this script is run
under `rocprofv3 --pmc FETCH_SIZE` (or WRITE_SIZE) that copy is the reference against
which the byte counters of the other kernels are scaled.

    python -m paper_2512_16843_amd.kernel_bench --B 64 --S 384 --d 768 --k 256 --N 16384

With --dense-rows R it runs, instead, the miss path alone: one post-LayerNorm encoder block
(d, d / 64 heads, FFN 4 d, erf-GELU) over R sequences of S tokens, i.e. the four linear
layers, the attention and the two LayerNorms that a cache-gated layer launches for R misses.

    python -m paper_2512_16843_amd.kernel_bench --dense-rows 28

With --bit-keys it runs, instead, llmc_match_bits over N random sign-bit keys of k bits and B queries
(half of them bank keys with a few bits flipped).

    python -m paper_2512_16843_amd.kernel_bench --bit-keys --B 4096 --N 1048576 --iters 3
"""
import argparse
import json
import sys

import torch

from . import llmc

CALIB_COPY_BYTES = 256 << 20


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--B", type=int, default=64)
    ap.add_argument("--S", type=int, default=384)
    ap.add_argument("--d", type=int, default=768)
    ap.add_argument("--k", type=int, default=256)
    ap.add_argument("--N", type=int, default=16384)
    ap.add_argument("--act-slots", type=int, default=2048, help="distinct cached-output rows (keys share them)")
    ap.add_argument("--iters", type=int, default=5)
    ap.add_argument("--dense-rows", type=int, default=0,
                    help="run the dense block of the miss path over this many sequences instead of the gate's kernels")
    ap.add_argument("--bit-keys", action="store_true", help="run the Hamming match of sign-bit keys instead")
    args = ap.parse_args()
    B, S, d, k, N, A = args.B, args.S, args.d, args.k, args.N, min(args.act_slots, args.N)
    dev, dt = "cuda", torch.bfloat16
    torch.manual_seed(0)
    llmc.lib()

    cal_src = torch.full((CALIB_COPY_BYTES,), 7, dtype=torch.uint8, device=dev)
    cal_dst = torch.empty_like(cal_src)
    for _ in range(3):
        cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    if args.dense_rows > 0:
        dense(args)
        return
    if args.bit_keys:
        bit_keys(args)
        return

    # several distinct inputs so that repeated launches do not re-read a cache-resident tensor
    hs = [torch.randn((B, S, d), device=dev, dtype=torch.float32).to(dt) for _ in range(args.iters)]
    P = (torch.randn((d, k), device=dev) / k ** 0.5).to(dt)
    fp = torch.empty((B, k), dtype=dt, device=dev)
    inv = torch.empty((B,), dtype=torch.float32, device=dev)
    ws_fp = torch.empty((llmc.llmc_fingerprint_workspace_bytes(B, S, d),), dtype=torch.uint8, device=dev)

    act_slot = (torch.randperm(N, device=dev) % A).int().contiguous()
    bank = llmc.Bank(N, k, S, d, dt, dev, n_act_slots=A, act_slot=act_slot)
    bank.fp.copy_(torch.nn.functional.normalize(torch.randn((N, k), device=dev), dim=1).to(dt))
    llmc.llmc_inv_norm(bank.fp, bank.inv_norm)
    bank.valid.fill_(1)
    bank.act.copy_(torch.randn((A, S, d), device=dev, dtype=torch.float32).to(dt))
    bank.refresh()
    idx = torch.empty((B,), dtype=torch.int32, device=dev)
    sim = torch.empty((B,), dtype=torch.float32, device=dev)
    hit = torch.empty((B,), dtype=torch.uint8, device=dev)
    ws_m = torch.empty((llmc.llmc_match_workspace_bytes(bank, B),), dtype=torch.uint8, device=dev)
    out = torch.empty((B, S, d), dtype=dt, device=dev)
    rows = torch.arange(B, dtype=torch.int32, device=dev)
    n = torch.tensor([B], dtype=torch.int32, device=dev)

    def step(i):
        llmc.llmc_fingerprint(hs[i % len(hs)], P, None, fp, inv, ws_fp)
        llmc.llmc_match(bank, fp, inv, -2.0, idx, sim, hit, None, ws_m)      # tau = -2: every row "hits"
        llmc.llmc_gather_hits(bank, idx, rows, n, B, out)

    step(0)
    torch.cuda.synchronize()
    llmc.llmc_profile_begin(8 * args.iters)
    for i in range(args.iters):
        step(i)
    rep = llmc.llmc_profile_report()
    llmc.llmc_profile_end()
    e = 2
    work = {
        "pool_kernel": (0.0, float(B) * S * d * e),
        "project_kernel": (2.0 * B * d * k, d * k * e),
        "match_stream_kernel": (2.0 * B * N * k, float(N) * k * e),
        "match_bf16_kernel": (2.0 * B * N * k, float(N) * k * e),
        "match_finalize_kernel": (0.0, 0.0),
        "gather_kernel": (0.0, 2.0 * B * S * d * e),
    }
    res = {"shape": {"B": B, "S": S, "d": d, "k": k, "N": N, "act_slots": A}, "calib_copy_bytes": CALIB_COPY_BYTES,
           "kernels": {}}
    for name, (cnt, ms) in sorted(rep.items()):
        us = ms * 1e3 / cnt
        fl, by = work.get(name, (0.0, 0.0))
        res["kernels"][name] = {"avg_us": round(us, 2), "gbs": round(by / us / 1e3, 1), "tflops": round(fl / us / 1e6, 2),
                                "algorithmic_bytes": by}
        print("%-24s avg %9.2f us  %9.1f GB/s  %8.2f TFLOP/s" % (name, us, by / us / 1e3, fl / us / 1e6), file=sys.stderr)
    bank.close()
    print(json.dumps(res))


def bit_keys(args):
    B, N, k = args.B, args.N, args.k
    W_ = k // 32
    bank = torch.randint(-2 ** 31, 2 ** 31, (N, W_), dtype=torch.int64, device="cuda").to(torch.int32)
    q = torch.randint(-2 ** 31, 2 ** 31, (B, W_), dtype=torch.int64, device="cuda").to(torch.int32)
    src = torch.randint(0, N, (B // 2,), device="cuda")
    flips = torch.zeros((B // 2, W_), dtype=torch.int32, device="cuda")
    flips[:, 0] = 0x00010101                                    # three bits away from a bank key
    q[: B // 2] = bank[src] ^ flips
    valid = torch.ones((N,), dtype=torch.uint8, device="cuda")
    idx = torch.empty((B,), dtype=torch.int32, device="cuda")
    dist = torch.empty((B,), dtype=torch.int32, device="cuda")
    hit = torch.empty((B,), dtype=torch.uint8, device="cuda")
    ws = torch.empty((llmc.llmc_match_bits_workspace_bytes(N, k, B),), dtype=torch.uint8, device="cuda")
    max_h = llmc.llmc_max_hamming(0.95, k)
    llmc.llmc_match_bits(bank, valid, q, max_h, idx, dist, hit, ws)
    torch.cuda.synchronize()
    llmc.llmc_profile_begin(4 * args.iters)
    for _ in range(args.iters):
        llmc.llmc_match_bits(bank, valid, q, max_h, idx, dist, hit, ws)
    rep = llmc.llmc_profile_report()
    llmc.llmc_profile_end()
    res = {"shape": {"B": B, "N": N, "key_bits": k}, "calib_copy_bytes": CALIB_COPY_BYTES,
           "hits": int(hit.sum()), "kernels": {}}
    for name, (cnt, ms) in sorted(rep.items()):
        us = ms * 1e3 / cnt
        scan = name in ("match_bits_mma_kernel", "match_bits_kernel")
        ops = 2.0 * B * N * k if scan else 0.0                    # bit pairs compared, as multiply-adds
        res["kernels"][name] = {"avg_us": round(us, 2), "tera_bit_ops_per_s": round(ops / us / 1e6, 1),
                                "algorithmic_bytes": float(N) * k / 8 if scan else 0.0}
        print("%-28s avg %9.2f us  %9.1f T bit-ops/s" % (name, us, ops / us / 1e6), file=sys.stderr)
    print(json.dumps(res))


def dense(args):
    from . import workloads as W
    from .engine import GatedStack
    R, S, d = args.dense_rows, args.S, args.d
    cfg = W.scaled(W.BERT_BASE, n_layers=1, B=R, S=S, d=d, n_heads=d // 64, d_ff=4 * d)
    ws = W.make_layer_weights(cfg, seed=0)
    Ps = W.make_projection(cfg.d, cfg.k, cfg.torch_dtype, seed=3, n_layers=1)
    st = GatedStack(cfg, ws, Ps, cached_layers=[])
    hs = [(torch.randn((R, S, d), device="cuda") * 0.5).to(cfg.torch_dtype) for _ in range(args.iters)]
    st.forward(hs[0], tau=2.0)
    torch.cuda.synchronize()
    llmc.llmc_profile_begin(16 * args.iters)
    for i in range(args.iters):
        st.forward(hs[i], tau=2.0)
    rep = llmc.llmc_profile_report()
    llmc.llmc_profile_end()
    T, e = float(R * S), 2
    work = {   # (flops, bytes) per launch, averaged over the launches of one block
        "gemm_bf16_kernel": (2.0 * T * d * 12 * d / 4, (T * d * e * (1 + 3 + 1 + 2 + 1 + 4 + 4 + 2) + 12.0 * d * d * e) / 4),
        "attention_kernel": (4.0 * R * S * S * d, T * d * e * 4),
        "layernorm_kernel": (8.0 * T * d, 2.0 * T * d * e),
    }
    res = {"shape": {"rows": R, "S": S, "d": d, "d_ff": 4 * d}, "calib_copy_bytes": CALIB_COPY_BYTES, "kernels": {}}
    for name, (cnt, ms) in sorted(rep.items()):
        us = ms * 1e3 / cnt
        fl, by = work.get(name, (0.0, 0.0))
        res["kernels"][name] = {"launches_per_block": cnt // args.iters, "avg_us": round(us, 2),
                                "gbs": round(by / us / 1e3, 1), "tflops": round(fl / us / 1e6, 2),
                                "algorithmic_bytes": by}
        print("%-24s %2d per block  avg %9.2f us  %9.1f GB/s  %8.2f TFLOP/s"
              % (name, cnt // args.iters, us, by / us / 1e3, fl / us / 1e6), file=sys.stderr)
    st.close()
    print(json.dumps(res))


if __name__ == "__main__":
    main()
