#!/usr/bin/env python3
"""Benchmark of the cache-gated forward on one MI355X.

A step is one pass of the whole hot path -- fingerprint, bank match, threshold +
compaction, gather of cached outputs, dense block for the misses -- through all
layers of the BERT-base-shaped stack (12 layers, d = 768, batch 64 x 384 tokens,
16,384-entry bank per layer) on one synthetic query batch resident in HBM.
Banks are built first by the library's own all-miss + insert path.
--workload selects the GPT-2-small-shaped decoder or the BERT-large-shaped stack
with dynamic banks instead; the default is the configuration the metric is quoted on.

Timed steps are replays of a HIP graph that records exactly one step's library launches
(--no-graph enqueues them from Python instead).

Prints ONE JSON line: whole-job sequences/s at the headline threshold, the sweep over
thresholds with measured hit rates, the roofline of the dominant kernel (per-kernel
durations from HIP events recorded on the launch stream), and the CPU oracle timed on
a bounded sample of the same batch.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "seq/s cache-gated 12L d768 forward vs hit rate; match MFMA% + gather HBM GB/s"
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
FP32_VALU_PEAK_TFLOPS = 157.3
INT_VALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12      # 32-bit integer vector instructions: one per lane per clock, 39.3 T/s
CALIB_COPY_BYTES = 256 << 20
DIAL_TAU = 0.9999
# HBM bytes per launch at the bench shape (64 rows of 384 x 768 bf16), from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs of paper_2512_16843_amd/kernel_bench.py, each scaled by what the counter read for that
# script's 256 MiB device-to-device copy (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0): see profiles/.
# Set an entry to None when its kernel changes.
MEASURED_TRAFFIC_BYTES = {
    "gather_kernel": (18349.1 * 2.0 + 36900.5) * 1024,    # algorithmic: 2 x 37,748,736
    "pool_kernel": (18478.2 * 2.0 + 1152.0) * 1024,       # algorithmic: 37,748,736 read (all 64 rows pooled)
}


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def kernel_work(cfg, name, miss, hit, e=2, carry=False, copied=None):
    """Algorithmic flops and bytes of ALL launches of `name` in one step, given per-layer miss/hit counts.
    carry: rows reused at layer l - 1 bring their token mean along and are not pooled at layer l."""
    d, dff, S, B, N, k = cfg.d, cfg.d_ff, cfg.S, cfg.B, cfg.n_bank, cfg.k
    L = len(miss)
    tok = [m * S for m in miss]
    if name == "gemm_bf16_kernel":
        fl = sum(2.0 * t * (4 * d * d + 2 * d * dff) for t in tok)
        by = sum((4 * d * d + 2 * d * dff) * e + t * (d + 3 * d + d + d + d + dff + dff + d) * e for t in tok)
        return fl, by, "mfma"
    if name == "attention_kernel":
        causal = 0.5 if cfg.arch == 1 else 1.0
        fl = sum(4.0 * m * S * S * d * causal for m in miss)
        by = sum(m * S * 4 * d * e for m in miss)
        return fl, by, "alu"
    if name == "layernorm_kernel":
        return sum(8.0 * t * d * 2 for t in tok), sum(2 * 2 * t * d * e for t in tok), "hbm"
    if name == "gather_kernel":
        # with deferred copies only the layers that copy in their reuse step count: copied = (plain, just-in-time)
        rows = float(sum(hit)) if copied is None else float(copied[0])
        return 0.0, 2.0 * rows * S * d * e, "hbm"
    if name == "materialize_kernel":
        return 0.0, 2.0 * float(copied[1] if copied else 0) * S * d * e, "hbm"
    if name == "pool_kernel":
        rows = float(L * B) if not carry else float(B + sum(B - h for h in hit[:-1]))
        return rows * S * d, rows * S * d * e, "hbm"
    if name == "project_kernel":
        rows = float(L * B) if not carry else float(B + sum(B - h for h in hit[:-1]))      # carried keys are copied
        return 2.0 * rows * d * k, L * (d * k * e + B * k * e), "hbm"
    if name in ("match_bf16_kernel", "match_stream_kernel"):
        return L * 2.0 * B * N * k, L * float(N) * k * e, "hbm" if B < 300 else "mfma"
    if name == "match_finalize_kernel":
        return L * 2.0 * B * 32 * k, L * float(B) * 32 * k * e, "hbm"
    if name == "insert_kernel":
        return 0.0, sum(2.0 * m * S * d * e for m in miss), "hbm"
    return 0.0, 0.0, "hbm"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--tau", type=float, default=0.95, help="headline threshold")
    ap.add_argument("--workload", choices=["bert-base", "gpt2-small", "bert-large-dynamic"], default="bert-base",
                    help="bert-base: the configuration the metric is quoted on (default); gpt2-small: causal decoder, "
                         "prefix-sharing queries; bert-large-dynamic: 24 layers with insertion and LRU eviction over a "
                         "stream of stem-sharing batches")
    ap.add_argument("--no-dial", action="store_true", help="skip the hit-rate dial leg")
    ap.add_argument("--no-graph", action="store_true",
                    help="enqueue every timed step from Python instead of replaying a HIP graph of it")
    ap.add_argument("--no-carry", action="store_true",
                    help="banks keep neither the token mean nor the next-layer key of cached outputs (every layer pools "
                         "and projects every row again)")
    ap.add_argument("--bank", type=int, default=None, help="bank entries per layer (default: the config's 16384)")
    ap.add_argument("--layers", type=int, default=None, help="debug: fewer layers")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stress", action="store_true", help="skip the 1M-key bank-match stress leg")
    ap.add_argument("--cpu-rows", type=int, default=2, help="sequences of the batch the oracle is timed on")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the path runs on ONE GPU (it is single-device); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2512_16843_amd import llmc, workloads as W
    from paper_2512_16843_amd.engine import GatedStack

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    llmc.lib()
    if args.workload == "bert-large-dynamic":
        print(json.dumps(bench_dynamic(args, llmc, W, GatedStack)))
        return
    decoder = args.workload == "gpt2-small"
    cfg = W.GPT2_SMALL if decoder else W.BERT_BASE
    if args.bank or args.layers:
        cfg = W.scaled(cfg, n_bank=args.bank or cfg.n_bank, n_layers=args.layers or cfg.n_layers)
    dev = "cuda"

    t0 = time.time()
    ws = W.make_layer_weights(cfg, seed=0)
    tok, pos = W.make_embeddings(cfg, seed=0)
    tok, pos = tok.to(dev), pos.to(dev)
    Ps = W.make_projection(cfg.d, cfg.k, cfg.torch_dtype, seed=3, n_layers=cfg.n_layers)
    src = W.make_sources(cfg, cfg.n_bank, seed=1)
    st = GatedStack(cfg, ws, Ps, keep_means=not args.no_carry, keep_next_keys=not args.no_carry)
    log("inputs drawn and %d banks allocated in %.1f s" % (cfg.n_layers, time.time() - t0))

    # ---- bank build: all-miss forward with insertion over the source sequences -------------------
    torch.cuda.synchronize()
    t0 = time.time()
    src_t = torch.from_numpy(src).to(dev)
    for s in range(0, cfg.n_bank, cfg.B):
        h = W.embed(src_t[s:s + cfg.B], tok, pos, cfg.torch_dtype)
        st.forward(h, tau=2.0, flags=llmc.INSERT_ON_MISS, tick=1)
    torch.cuda.synchronize()
    build_s = time.time() - t0
    assert all(int(b.valid.sum()) == cfg.n_bank for b in st.banks)
    log("banks built: %d sequences x %d layers in %.1f s (%.1f seq/s all-miss with insertion)"
        % (cfg.n_bank, cfg.n_layers, build_s, cfg.n_bank / build_s))

    # a plain device-to-device copy of known size: the reference against which HBM byte counters
    # (FETCH_SIZE / WRITE_SIZE) of a profiled run are scaled
    cal_src = torch.full((CALIB_COPY_BYTES,), 7, dtype=torch.uint8, device=dev)
    cal_dst = torch.empty_like(cal_src)
    for _ in range(3):
        cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    # ---- query batch ----
    if decoder:
        # every row shares a prefix of random length (25-75 % of the sequence) with a bank source, fresh suffix
        ids, srcmap, _ = W.make_prefix_queries(cfg, src, seed=2)
        recipe = "each query = a bank source's prefix of 25-75 % of the tokens + a fresh suffix"
    else:
        # 60 % perturbed copies of bank sources (3 % of tokens resampled), 40 % fresh
        n_dup = int(round(0.6 * cfg.B))
        n_sub = int(round(0.03 * cfg.S))
        ids, srcmap = W.make_substitution_queries(cfg, src, n_dup=n_dup, n_subst=n_sub, seed=2)
        recipe = "60% perturbed copies (3% tokens resampled) + 40% fresh"
    h0 = W.embed(torch.from_numpy(ids).to(dev), tok, pos, cfg.torch_dtype)

    def run(tau, steps, warmup, h=None):
        """W untimed eager steps (they also settle the engine's launch-shape hints), then K timed steps.  With
        --graph (default) the step -- the same sequence of library launches, nothing else -- is recorded once in a
        HIP graph and the timed steps are replays of it: at high hit rates a step is ~145 short launches and the
        Python / ctypes side of enqueueing them is otherwise as long as their execution."""
        h = h0 if h is None else h
        for _ in range(warmup):
            st.forward(h, tau=tau)
        torch.cuda.synchronize()
        if args.no_graph:
            step = lambda: st.forward(h, tau=tau)
        else:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                st.forward(h, tau=tau)
            torch.cuda.synchronize()
            step = graph.replay
            for _ in range(2):
                step()
            torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t) / steps
        cnt = st.hit_counts().numpy()
        return dt, cnt

    def row_of(tau, dt, cnt):
        hits = cnt[:, llmc.CNT_HIT]
        return {"tau": tau if tau <= 1.0 else "no-cache", "ms_per_step": round(dt * 1e3, 4),
                "seq_per_s": round(cfg.B / dt, 2), "hit_rate": round(float(hits.sum()) / (cfg.B * cfg.n_layers), 4),
                "hit_rate_first_layer": round(float(hits[0]) / cfg.B, 4),
                "hit_rate_last_layer": round(float(hits[-1]) / cfg.B, 4),
                "near_tau_rows": int(cnt[:, llmc.CNT_NEAR_TAU].sum()),
                "near_tie_rows": int(cnt[:, llmc.CNT_NEAR_TIE].sum())}

    def show(row):
        log("tau=%s  %.3f ms/step  %.1f seq/s  hit rate %.3f (layer 1: %.3f, layer %d: %.3f)"
            % (row["tau"], row["ms_per_step"], row["seq_per_s"], row["hit_rate"], row["hit_rate_first_layer"],
               cfg.n_layers, row["hit_rate_last_layer"]))

    # the other thresholds of the sweep first; the headline threshold is timed LAST, so that the
    # final steps * launches_per_step library kernels of a trace are exactly the timed region
    sweep = []
    for tau in sorted(set([0.95] if decoder else [0.90, 0.95, 0.98]) - {args.tau}) + [2.0]:
        dt, cnt = run(tau, args.steps, args.warmup)
        sweep.append(row_of(tau, dt, cnt))
        show(sweep[-1])

    # ---- hit-rate dial: a fraction rho of the rows are exact copies of bank sources (similarity 1), the rest
    # fresh; at a threshold just below 1 only the copies hit, so the measured hit rate follows rho ----
    dial = []
    if not args.no_dial:
        for rho in (0.25, 0.5, 0.75, 0.9):
            ids_d, _ = W.make_dial_queries(cfg, src, rho, seed=7)
            h_d = W.embed(torch.from_numpy(ids_d).to(dev), tok, pos, cfg.torch_dtype)
            dt, cnt = run(DIAL_TAU, max(5, args.steps // 2), max(2, args.warmup // 2), h_d)
            row = row_of(DIAL_TAU, dt, cnt)
            row["rho"] = rho
            dial.append(row)
            log("dial rho=%.2f tau=%s  %.3f ms/step  %.1f seq/s  hit rate %.3f"
                % (rho, DIAL_TAU, row["ms_per_step"], row["seq_per_s"], row["hit_rate"]))
            del h_d

    # ---- per-kernel durations: HIP events on the launch stream around every kernel --------------
    def profile(tau, steps=5):
        st.forward(h0, tau=tau)
        torch.cuda.synchronize()
        llmc.llmc_profile_begin(steps * cfg.n_layers * 24)
        for _ in range(steps):
            st.forward(h0, tau=tau)
        rep = llmc.llmc_profile_report()
        llmc.llmc_profile_end()
        cnt = st.hit_counts().numpy()
        miss = [int(x) for x in cnt[:, llmc.CNT_MISS]]
        hit = [int(x) for x in cnt[:, llmc.CNT_HIT]]
        copied = st.copied_rows()
        out = {}
        for name, (n, ms) in rep.items():
            fl, by, bound = kernel_work(cfg, name, miss, hit, carry=not args.no_carry, copied=copied)
            t_step = ms * 1e-3 / steps
            out[name] = {"launches_per_step": n // steps, "avg_us": round(ms * 1e3 / n, 3),
                         "ms_per_step": round(ms / steps, 4), "bound": bound,
                         "tflops": round(fl / t_step / 1e12, 3) if t_step > 0 else 0.0,
                         "gbs": round(by / t_step / 1e9, 2) if t_step > 0 else 0.0}
        return out

    prof_nocache = profile(2.0)
    prof_head = profile(args.tau)
    for tag, pr in (("tau=%s" % args.tau, prof_head), ("no-cache", prof_nocache)):
        for name, r in sorted(pr.items(), key=lambda kv: -kv[1]["ms_per_step"]):
            log("%-9s %-24s %3d launches/step  avg %9.2f us  %8.4f ms/step  %8.2f TFLOP/s %9.1f GB/s"
                % (tag, name, r["launches_per_step"], r["avg_us"], r["ms_per_step"], r["tflops"], r["gbs"]))
    launches_per_step = sum(r["launches_per_step"] for r in prof_head.values())
    # Event brackets around single ~15 us kernels add a few us each.  The gather launches of the headline
    # step (one per layer: that layer's bank, that layer's hit rows) are also replayed back to back between
    # ONE pair of events on the same stream: that average is the launch duration rocprofv3 reports.
    hit_head = [int(x) for x in st.hit_counts().numpy()[:, llmc.CNT_HIT]]
    gather_replay_us = replay_gathers(llmc, st, cfg, reps=20) if sum(hit_head) else None
    if gather_replay_us:
        log("gather replay at the headline threshold: %.2f us per launch -> %.1f GB/s"
            % (gather_replay_us, sum(2.0 * h * cfg.S * cfg.d * 2 for h in hit_head) / cfg.n_layers / gather_replay_us / 1e3))

    # ---- CPU oracle on a bounded sample of the same batch (before the headline run) -----------------
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, st, ws, Ps, h0, args.tau, args.cpu_rows)
        log("cpu oracle: %.3f seq/s on %d threads (%s)" % (cpu["value"], cpu["cores"], cpu["sample"]))

    # ---- bank-match stress shape (1,048,576 keys x 256, 4,096 queries) and its gather ------------------
    stress = None
    if not args.no_stress and not decoder:
        stress = match_stress(llmc, W)
        log("match stress: %.1f us -> %.1f TFLOP/s (%.1f%% of bf16 MFMA peak); finalize %.1f us; gather of %d hits "
            "%.1f us -> %.1f GB/s (%.1f%% of HBM peak)"
            % (stress["match_us"], stress["match_tflops"], 100 * stress["match_frac_mfma"], stress["finalize_us"],
               stress["hits"], stress["gather_us"], stress["gather_gbs"], 100 * stress["gather_frac_hbm"]))
        sb = stress["sign_bit_keys"]
        log("sign-bit keys on the same bank (%d bits, %d MB instead of 512): Hamming match %.1f us (+%.1f us) -> %.2f T "
            "word-ops/s (%.1f%% of the integer vector peak); %d hits; hit rows in the cosine match's cluster %.4f, same "
            "decision %.4f" % (sb["key_bits"], sb["bank_bytes"] >> 20, sb["match_us"], sb["other_us"],
                               sb["tera_word_ops_per_s"], 100 * sb["frac_int_valu_peak"], sb["hits"],
                               sb["same_cluster_as_cosine_match_on_hits"], sb["same_decision_as_cosine_match"]))
        ls = sb["lsh"]
        log("bucketed lookup (%d bands of 16 bits, index %d MB): build %.1f us, lookup of 4096 queries %.1f us; bucket "
            "members visited per query: median %d, max %d of 1,048,576; same slot as the full Hamming match on hits %.4f, "
            "same decision %.4f" % (ls["bands"], ls["index_bytes"] >> 20, ls["build_us"], ls["match_us"],
                                    ls["visited_per_query_median"], ls["visited_per_query_max"],
                                    ls["same_slot_as_full_match_on_hits"], ls["same_decision_as_full_match"]))

    # ---- headline: the last GPU work of the run ------------------------------------------------------
    dt_head, cnt_head = run(args.tau, args.steps, args.warmup)
    sweep.append(row_of(args.tau, dt_head, cnt_head))
    show(sweep[-1])
    sweep.sort(key=lambda r: (r["tau"] == "no-cache", r["tau"] if r["tau"] != "no-cache" else 9))
    log("library kernel launches per step at the headline threshold: %d" % launches_per_step)

    # The dominant kernel of the headline run decides the roofline object.  Kernels that had no work at this
    # hit rate (miss-path launches with zero misses) only show their launch bracket and are not candidates.
    # Its duration is the slice of a step that moves the most HBM bytes per launch.  With deferred copies the reuse
    # step of all layers but the last hands references on instead of copying, so at high hit rates most launches
    # of a step are short latency-bound kernels (match, finalize, compaction, empty launches) for which a
    # bandwidth or flop roofline says little; the one full-size copy per step is the launch that a roofline bounds.
    def has_work(name, r):
        return r["tflops"] > 0 or r["gbs"] > 0
    latency_class = ("match_finalize_kernel", "project_kernel", "compact_kernel", "select_kernel", "materialize_kernel",
                     "match_stream_kernel" if cfg.B < 300 else "")
    cands = {k: v for k, v in prof_head.items()
             if has_work(k, v) and k not in latency_class and not (k == "gemm_bf16_kernel" and v["tflops"] == 0)}
    name, r = max(cands.items(), key=lambda kv: kv[1]["ms_per_step"])
    avg_us = r["avg_us"]
    if name == "gather_kernel" and gather_replay_us:
        avg_us = gather_replay_us
        by = sum(2.0 * h * cfg.S * cfg.d * 2 for h in hit_head) / cfg.n_layers
        r = dict(r, gbs=round(by / avg_us / 1e3, 2), avg_us=round(avg_us, 3))
    if r["bound"] == "mfma":
        roof = {"kernel": name, "bound": "mfma", "achieved": r["tflops"], "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(r["tflops"] / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None}
    elif r["bound"] == "alu":
        roof = {"kernel": name, "bound": "alu", "achieved": r["tflops"], "peak": FP32_VALU_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(r["tflops"] / FP32_VALU_PEAK_TFLOPS, 4), "traffic": None}
    else:
        roof = {"kernel": name, "bound": "hbm", "achieved": r["gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(r["gbs"] / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC_BYTES.get(name)}
    roof["avg_launch_us"] = r["avg_us"]

    result = {
        "metric": METRIC, "value": round(cfg.B / dt_head, 2), "unit": "seq/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(dt_head * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s %s: %d layers, d=%d, batch %d x %d tokens, bank %d x k=%d per layer, %s, static banks"
                               % (cfg.name, "causal decoder" if decoder else "encoder", cfg.n_layers, cfg.d, cfg.B,
                                  cfg.S, cfg.n_bank, cfg.k, recipe),
                   "tau": args.tau,
                   "hit_rate": round(float(cnt_head[:, llmc.CNT_HIT].sum()) / (cfg.B * cfg.n_layers), 4),
                   "bank_build_s": round(build_s, 2), "launches_per_step": launches_per_step,
                   "timed_steps": "eager launches from Python" if args.no_graph else "replays of a HIP graph of one step",
                   "carried_keys_and_deferred_copies": not args.no_carry},
        "sweep": sweep,
        "dial": dial,
        "roofline": roof,
        "kernels": {"headline": prof_head, "no_cache": prof_nocache},
        "match_stress": stress,
        "cpu_baseline": cpu,
    }
    st.close()
    print(json.dumps(result))


def replay_gathers(llmc, st, cfg, reps):
    """Average duration of the per-layer gather launches of the last forward, replayed back to back."""
    import torch
    rows, ns = [], []
    for g in st.gate:
        r = torch.nonzero(g.hit).flatten().int().contiguous()
        rows.append(r if r.numel() else torch.zeros((1,), dtype=torch.int32, device=r.device))
        ns.append(torch.tensor([r.numel()], dtype=torch.int32, device=r.device))
    out = st.buf[0]
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    def once():
        for l in range(cfg.n_layers):
            llmc.llmc_gather_hits(st.banks[l], st.gate[l].idx, rows[l], ns[l], cfg.B, out)
    once()
    torch.cuda.synchronize()
    a.record()
    for _ in range(reps):
        once()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e3 / (reps * cfg.n_layers)


def match_stress(llmc, W, iters=10):
    """Top-1 cosine + threshold over a 1,048,576-key clustered bank for 4,096 queries, then the gather
    of the matched 384 x 768 outputs for the hits; per-kernel times from the library's HIP events."""
    import torch
    N, k, S, d, A, B, tau = 1048576, 256, 384, 768, 4096, 4096, 0.95
    data = W.make_clustered_bank(4096, 256, k, 0.05, B, seed=5)
    bank = llmc.Bank(N, k, S, d, torch.bfloat16, "cuda", n_act_slots=A, act_slot=data["cluster"].cuda())
    bank.fp.copy_(data["bank"])
    llmc.llmc_inv_norm(bank.fp, bank.inv_norm)
    bank.valid.fill_(1)
    bank.act.copy_(torch.randn((A, S, d), device="cuda", dtype=torch.bfloat16))
    bank.refresh()
    q = data["queries"].cuda()
    qinv = torch.empty((B,), dtype=torch.float32, device="cuda")
    llmc.llmc_inv_norm(q, qinv)
    idx = torch.empty((B,), dtype=torch.int32, device="cuda")
    sim = torch.empty((B,), dtype=torch.float32, device="cuda")
    hit = torch.empty((B,), dtype=torch.uint8, device="cuda")
    ws = torch.empty((llmc.llmc_match_workspace_bytes(bank, B),), dtype=torch.uint8, device="cuda")
    out = torch.empty((B, S, d), dtype=torch.bfloat16, device="cuda")
    llmc.llmc_match(bank, q, qinv, tau, idx, sim, hit, None, ws)
    rows = torch.nonzero(hit).flatten().int().contiguous()
    n = torch.tensor([rows.numel()], dtype=torch.int32, device="cuda")
    llmc.llmc_gather_hits(bank, idx, rows, n, B, out)
    torch.cuda.synchronize()
    llmc.llmc_profile_begin(4 * iters)
    for _ in range(iters):
        llmc.llmc_match(bank, q, qinv, tau, idx, sim, hit, None, ws)
        llmc.llmc_gather_hits(bank, idx, rows, n, B, out)
    rep = llmc.llmc_profile_report()
    llmc.llmc_profile_end()
    us = {name: ms * 1e3 / cnt for name, (cnt, ms) in rep.items()}
    H = int(rows.numel())
    m_us, g_us = us["match_stream_kernel"], us["gather_kernel"]
    tfl = 2.0 * B * N * k / m_us / 1e6
    gbs = 2.0 * H * S * d * 2 / g_us / 1e3

    # ---- the same bank and queries as sign-bit keys: each 256-vector is projected by a seeded Gaussian P
    # [256, 256] and only the signs are kept (32 bytes per key instead of 512); match by Hamming distance ----
    kb = 256
    gen = torch.Generator(device="cuda").manual_seed(21)
    P = (torch.randn((k, kb), generator=gen, device="cuda") / kb ** 0.5).to(torch.bfloat16)
    bank_bits = torch.empty((N, kb // 32), dtype=torch.int32, device="cuda")
    q_bits = torch.empty((B, kb // 32), dtype=torch.int32, device="cuda")
    chunk = 32768
    ws_f = torch.empty((llmc.llmc_fingerprint_workspace_bytes(chunk, 1, k),), dtype=torch.uint8, device="cuda")
    for s0 in range(0, N, chunk):
        llmc.llmc_fingerprint_bits(bank.fp[s0:s0 + chunk].view(-1, 1, k), P, None, bank_bits[s0:s0 + chunk], ws_f)
    llmc.llmc_fingerprint_bits(q.view(B, 1, k), P, None, q_bits, ws_f)
    max_h = llmc.llmc_max_hamming(tau, kb)
    idx_b = torch.empty((B,), dtype=torch.int32, device="cuda")
    dist_b = torch.empty((B,), dtype=torch.int32, device="cuda")
    hit_b = torch.empty((B,), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty((llmc.llmc_match_bits_workspace_bytes(N, kb, B),), dtype=torch.uint8, device="cuda")
    llmc.llmc_match_bits(bank_bits, bank.valid, q_bits, max_h, idx_b, dist_b, hit_b, ws_b)
    torch.cuda.synchronize()
    llmc.llmc_profile_begin(4 * iters)
    for _ in range(iters):
        llmc.llmc_match_bits(bank_bits, bank.valid, q_bits, max_h, idx_b, dist_b, hit_b, ws_b)
    rep_b = llmc.llmc_profile_report()
    llmc.llmc_profile_end()
    us_b = {name: ms * 1e3 / cnt for name, (cnt, ms) in rep_b.items()}
    # bucketed lookup over the same bit keys: 16 bands of 16 bits, compare only with bucket members
    index = torch.empty((llmc.llmc_lsh_index_bytes(N, kb),), dtype=torch.uint8, device="cuda")
    idx_l = torch.empty((B,), dtype=torch.int32, device="cuda")
    dist_l = torch.empty((B,), dtype=torch.int32, device="cuda")
    hit_l = torch.empty((B,), dtype=torch.uint8, device="cuda")
    visited = torch.empty((B,), dtype=torch.int32, device="cuda")
    llmc.llmc_lsh_build(bank_bits, bank.valid, index)
    llmc.llmc_match_bits_lsh(bank_bits, index, q_bits, max_h, idx_l, dist_l, hit_l, visited)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    ev[0].record()
    for _ in range(iters):
        llmc.llmc_lsh_build(bank_bits, bank.valid, index)
    ev[1].record()
    for _ in range(iters):
        llmc.llmc_match_bits_lsh(bank_bits, index, q_bits, max_h, idx_l, dist_l, hit_l, visited)
    ev[2].record()
    torch.cuda.synchronize()
    hb_ = hit_b.bool()
    lsh = {"bands": kb // 16, "index_bytes": int(index.numel()),
           "build_us": round(ev[0].elapsed_time(ev[1]) * 1e3 / iters, 1),
           "match_us": round(ev[1].elapsed_time(ev[2]) * 1e3 / iters, 1),
           "visited_per_query_median": int(visited.float().median()), "visited_per_query_max": int(visited.max()),
           "same_slot_as_full_match_on_hits": round(float((idx_l == idx_b)[hb_].float().mean()), 4) if bool(hb_.any()) else 1.0,
           "same_decision_as_full_match": round(float((hit_l == hit_b).float().mean()), 4)}
    del index
    cluster = data["cluster"].cuda()
    hb = hit.bool()
    same_cluster = float((cluster[idx_b.long()] == cluster[idx.long()])[hb].float().mean()) if bool(hb.any()) else 1.0
    same_decision = float((hit_b == hit).float().mean())
    word_ops = 2.0 * B * N * (kb // 32)                  # one XOR and one popcount-accumulate per 32 bit pairs
    bits = {"key_bits": kb, "bank_bytes": N * kb // 8, "max_hamming": int(max_h),
            "match_us": round(us_b["match_bits_kernel"], 2),
            "other_us": round(sum(v for n_, v in us_b.items() if n_ != "match_bits_kernel"), 2),
            "tera_word_ops_per_s": round(word_ops / us_b["match_bits_kernel"] / 1e6, 2),
            "frac_int_valu_peak": round(word_ops / us_b["match_bits_kernel"] / 1e6 / INT_VALU_PEAK_TOPS, 4),
            "hits": int(hit_b.sum()), "same_cluster_as_cosine_match_on_hits": round(same_cluster, 4),
            "same_decision_as_cosine_match": round(same_decision, 4), "lsh": lsh}
    del bank_bits, q_bits, ws_f, ws_b
    bank.close()
    res = {"workload": "bank-match stress: 1,048,576 bf16 keys x 256 in 4,096 clusters, 4,096 queries, tau 0.95, "
                       "gather of 384 x 768 bf16 outputs for the hits",
           "hits": H, "match_us": round(m_us, 2), "match_tflops": round(tfl, 1),
           "match_frac_mfma": round(tfl / MFMA_BF16_PEAK_TFLOPS, 4), "finalize_us": round(us["match_finalize_kernel"], 2),
           "gather_us": round(g_us, 2), "gather_gbs": round(gbs, 1), "gather_frac_hbm": round(gbs / HBM_PEAK_GBS, 4),
           "sign_bit_keys": bits}
    del bank, out
    torch.cuda.empty_cache()
    return res


def cpu_baseline(cfg, st, ws, Ps, h0, tau, n_rows):
    """Time the oracle's gated forward (all layers) on the first rows of the batch.

    The oracle reads the banks the GPU built: keys come to the host whole, cached
    outputs are fetched row by row when a hit needs them.
    """
    import numpy as np
    import torch
    from oracle import llmc_oracle as O

    npf = lambda t: t.detach().float().cpu().numpy()

    class LazyAct:
        def __init__(self, t):
            self.t = t

        def __getitem__(self, j):
            return npf(self.t[int(j)])

    banks = []
    for b in st.banks:
        ob = O.Bank(1, cfg.k, 1, 1, cfg.dtype)
        ob.N, ob.S, ob.d, ob.A = b.n_slots, b.S, b.d, b.n_act_slots
        ob.fp, ob.inv_norm, ob.valid = npf(b.fp), npf(b.inv_norm), b.valid.cpu().numpy()
        ob.act_slot = np.arange(b.n_slots, dtype=np.int32)
        ob.act = LazyAct(b.act)
        banks.append(ob)
    wnp = [{k: npf(v) for k, v in w.items()} for w in ws]
    Pnp = [npf(p) for p in Ps]
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    tau32 = float(np.float32(tau))
    n = max(1, min(n_rows, cfg.B))
    while True:
        x = npf(h0[:n])
        t = time.perf_counter()
        _, res = O.infer(x, banks, Pnp, [None] * cfg.n_layers, wnp, cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu,
                         tau=tau32, out_dtype=cfg.dtype)
        dt = time.perf_counter() - t
        if dt >= 8.0 or n >= cfg.B:
            break
        n = min(cfg.B, max(n + 1, int(n * min(8.0, 12.0 / max(dt, 1e-3)))))
    # a whole batch that takes less than ~10 s (high hit rates leave the oracle little to do) is repeated
    passes, total = 1, dt
    while total < 10.0 and passes < 40:
        t = time.perf_counter()
        O.infer(x, banks, Pnp, [None] * cfg.n_layers, wnp, cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu, tau=tau32,
                out_dtype=cfg.dtype)
        total += time.perf_counter() - t
        passes += 1
    hits = sum(int(r.hit.sum()) for r in res)
    return {"value": round(n * passes / total, 4), "unit": "seq/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d pass(es) over the first %d of %d sequences of the batch through all %d layers at tau=%s "
                      "against the GPU-built banks (%d of %d row-layers hit), %.1f s"
                      % (passes, n, cfg.B, cfg.n_layers, tau, hits, n * cfg.n_layers, total)}


def bench_dynamic(args, llmc, W, GatedStack):
    """BERT-large-shaped stack with bank insertion and LRU eviction active: banks pre-filled to capacity by a
    warm-up stream, then segments of 50 successive batches of stem-sharing candidates (64 groups of 4 sequences
    sharing an 80-token stem).  A step is one batch through all 24 layers, inserts and evictions included."""
    import numpy as np
    import torch
    cfg = W.BERT_LARGE
    if args.bank or args.layers:
        cfg = W.scaled(cfg, n_bank=args.bank or cfg.n_bank, n_layers=args.layers or cfg.n_layers)
    dev = "cuda"
    ws = W.make_layer_weights(cfg, seed=0)
    tok, pos = W.make_embeddings(cfg, seed=0)
    tok, pos = tok.to(dev), pos.to(dev)
    Ps = W.make_projection(cfg.d, cfg.k, cfg.torch_dtype, seed=3, n_layers=cfg.n_layers)
    st = GatedStack(cfg, ws, Ps, keep_means=not args.no_carry, keep_next_keys=not args.no_carry)
    stream = W.StemStream(cfg, group=4, stem_len=80, n_stems=512, seed=4)
    flags = llmc.INSERT_ON_MISS | llmc.UPDATE_LRU
    tick = 0
    t0 = time.time()
    for _ in range(cfg.n_bank // cfg.B):
        tick += 1
        ids, _ = stream.next_batch()
        st.forward(W.embed(torch.from_numpy(ids).to(dev), tok, pos, cfg.torch_dtype), tau=2.0, flags=flags, tick=tick)
    torch.cuda.synchronize()
    fill_s = time.time() - t0
    log("banks pre-filled: %d batches x %d layers in %.1f s (%.1f seq/s all-miss with insertion)"
        % (cfg.n_bank // cfg.B, cfg.n_layers, fill_s, cfg.n_bank / fill_s))
    n_batches, segments = 50, []
    for seg in range(3):
        hs = []
        for _ in range(n_batches):
            ids, _ = stream.next_batch()
            hs.append(W.embed(torch.from_numpy(ids).to(dev), tok, pos, cfg.torch_dtype))
        counters = []
        torch.cuda.synchronize()
        t = time.perf_counter()
        for h in hs:
            tick += 1
            st.forward(h, tau=args.tau, flags=flags, tick=tick)
            counters.append(torch.stack([g.counters for g in st.gate]))      # device-side copy, no host sync
        torch.cuda.synchronize()
        dt = time.perf_counter() - t
        cnt = torch.stack(counters).cpu().numpy()                            # [batch, layer, word]
        hit_rate = cnt[:, :, llmc.CNT_HIT].sum(axis=1) / float(cfg.B * cfg.n_layers)
        segments.append({"batches": n_batches, "seconds": round(dt, 4), "seq_per_s": round(n_batches * cfg.B / dt, 2),
                         "hit_rate": round(float(hit_rate.mean()), 4),
                         "hit_rate_first_last_batch": [round(float(hit_rate[0]), 4), round(float(hit_rate[-1]), 4)],
                         "inserted": int(cnt[:, :, llmc.CNT_INSERTED].sum()),
                         "evicted": int(cnt[:, :, llmc.CNT_EVICTED].sum())})
        log("segment %d: %d batches in %.3f s -> %.1f seq/s, hit rate %.3f, %d inserts, %d evictions"
            % (seg, n_batches, dt, segments[-1]["seq_per_s"], segments[-1]["hit_rate"], segments[-1]["inserted"],
               segments[-1]["evicted"]))
        del hs
    # the same shapes without the cache
    h = W.embed(torch.from_numpy(stream.next_batch()[0]).to(dev), tok, pos, cfg.torch_dtype)
    for _ in range(2):
        st.forward(h, tau=2.0)
    torch.cuda.synchronize()
    t = time.perf_counter()
    for _ in range(5):
        st.forward(h, tau=2.0)
    torch.cuda.synchronize()
    nocache = 5 * cfg.B / (time.perf_counter() - t)
    log("no-cache: %.1f seq/s" % nocache)
    best = max(segments, key=lambda r: r["seq_per_s"])
    last = segments[-1]
    st.close()
    return {"metric": METRIC, "value": last["seq_per_s"], "unit": "seq/s", "n_gpus": 1, "steps": n_batches, "warmup": 0,
            "ms_per_step": round(last["seconds"] / n_batches * 1e3, 4), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "%s encoder, dynamic banks: %d layers, d=%d, batch %d x %d tokens (64 groups of 4 "
                                   "candidates sharing an 80-token stem, 512 recurring stems), bank %d x k=%d per layer "
                                   "pre-filled to capacity, INSERT_ON_MISS | UPDATE_LRU, every miss evicts"
                                   % (cfg.name, cfg.n_layers, cfg.d, cfg.B, cfg.S, cfg.n_bank, cfg.k),
                       "tau": args.tau, "hit_rate": last["hit_rate"], "prefill_s": round(fill_s, 1)},
            "segments": segments, "no_cache_seq_per_s": round(nocache, 2), "best_segment_seq_per_s": best["seq_per_s"],
            "roofline": None, "cpu_baseline": None}


if __name__ == "__main__":
    main()
