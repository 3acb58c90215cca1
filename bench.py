#!/usr/bin/env python3
"""Benchmark of the cache-gated forward on one MI355X.

A step is one pass of the whole hot path -- fingerprint, bank match, threshold + compaction, gather of cached
outputs, dense block for the misses -- through all layers of the BERT-base-shaped stack (12 layers, d = 768,
batch 64 x 384 tokens, 16,384-entry bank per layer) on one synthetic query batch resident in HBM.  Banks are
built first by the library's own all-miss + insert path.

The default run reports, in ONE JSON line:
  * the threshold sweep {0.90, 0.95, 0.98} for both fingerprint variants -- the plain linear map (c = 0) and
    the centred one (c = -P^T mu, mu = mean pooled vector of the bank sources) -- with measured hit rates, the
    no-cache run, and a hit-rate dial; `value` is the centred variant at the headline threshold, the point
    where the perturbed copies are reused and the fresh rows are computed;
  * `roofline`: the kernel with the largest share of the headline step, from per-kernel HIP events; `rooflines`:
    the other kernels of the path at the shapes that bound them (1M-key match, gather of 2,048 rows, pooling of
    4,096 sequences, the 64-query match of the step);
  * compact legs for the GPT-2-small-shaped decoder and the BERT-large-shaped stack with dynamic banks;
  * `cpu_baseline`: the CPU oracle timed on a bounded sample of the same batch, on all host threads and on one,
    plus the oracle's match on a sample of the 1M-key stress queries.
Timed steps are replays of a HIP graph that records exactly one step's library launches (--no-graph enqueues
them from Python instead).  --workload runs one of the other model configurations alone.
"""
import argparse
import hashlib
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
MFMA_INT8_PEAK_TOPS = 5000.0
FP32_VALU_PEAK_TFLOPS = 157.3
INT_VALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12      # 32-bit integer vector instructions: one per lane per clock, 39.3 T/s
CALIB_COPY_BYTES = 256 << 20
DIAL_TAU = 0.9999
CSRC = os.path.join(ROOT, "paper_2512_16843_amd", "csrc")

# HBM bytes per launch from `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` runs (KiB per dispatch), each
# scaled by what the same counter read for a plain 256 MiB device-to-device copy; see profiles/.  An entry is
# tied to the sources of its kernel: `sources` are hashed, and when the hash no longer matches (the kernel has
# changed since the counters were taken) the benchmark reports null instead of a stale figure.
# name -> (bytes per launch, source files, sha256 of their concatenation when the counters were taken)
MEASURED_TRAFFIC = {
    # profiles/kernel_bench_dense_block_trace_and_counters.txt: one block over 28 sequences (the headline's mean miss
    # count is 27.7), average over the block's launches of the kernel
    "gemm_bf16_kernel": (132532043, ['gemm.h', 'mma.h', 'layer.hip'], "b36c4e5feea01b4b"),
    "attention_kernel": (132213306, ['attention.hip', 'mma.h'], "115938f4b5152aea"),
    # profiles/kernel_bench_bert_base_shape_trace_and_hbm_counters.txt: 64 sequences, bank of 16384 keys
    "pool_kernel": (39019714, ['fingerprint.hip'], "83917709d3f168a6"),
    "match_stream_kernel": (9152651, ['match.hip', 'mma.h'], "620ba3edc6b4ef7f"),
}


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def source_hash(files):
    h = hashlib.sha256()
    for f in files:
        with open(os.path.join(CSRC, f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(name):
    ent = MEASURED_TRAFFIC.get(name)
    if not ent:
        return None
    nbytes, files, digest = ent
    return nbytes if source_hash(files) == digest else None


def kernel_work(cfg, name, miss, hit, e=2, carry=False, copied=None):
    """Algorithmic flops and bytes of ALL launches of `name` in one step, given per-layer miss/hit counts.
    carry: rows reused at layer l - 1 bring their token mean along and are not pooled at layer l."""
    d, dff, S, B, N, k = cfg.d, cfg.d_ff, cfg.S, cfg.B, cfg.n_bank, cfg.k
    L = len(miss)
    tok = [m * S for m in miss]
    if name == "gemm_bf16_kernel":
        fl = sum(2.0 * t * (4 * d * d + 2 * d * dff) for t in tok)
        by = sum(((4 * d * d + 2 * d * dff) * e if t else 0) + t * (d + 3 * d + 3 * d + d + dff + dff + 2 * d) * e for t in tok)    # operands, residuals, outputs
        return fl, by, "mfma"
    if name == "attention_kernel":
        causal = 0.5 if cfg.arch == 1 else 1.0
        fl = sum(4.0 * m * S * S * d * causal for m in miss)
        by = sum(m * S * 4 * d * e for m in miss)
        return fl, by, "mfma"
    if name == "layernorm_kernel":
        return sum(8.0 * t * d * 2 for t in tok), sum(2 * 2 * t * d * e for t in tok), "hbm"
    if name == "gather_kernel":
        # with deferred copies only the layers that copy in their reuse step count: copied = (plain, just-in-time)
        rows = float(sum(hit)) if copied is None else float(copied[0])
        return 0.0, 2.0 * rows * S * d * e, "hbm"
    if name == "materialize_kernel":
        return 0.0, 2.0 * float(copied[1] if copied else 0) * S * d * e, "hbm"
    if name == "pool_kernel":
        # stored means carry the reused rows; a post-LayerNorm block pools the rows it computes on the way out
        rows = float(L * B) if not carry else (float(B) if cfg.arch == 0 else float(B + sum(B - h for h in hit[:-1])))
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


def roof_entry(name, bound, flops, nbytes, us, note=None, traffic=None):
    """One roofline record: algorithmic work of the launches measured / their summed duration."""
    if bound == "mfma":
        ach, peak, unit = flops / us / 1e6, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s"
    elif bound == "alu":
        ach, peak, unit = flops / us / 1e6, FP32_VALU_PEAK_TFLOPS, "TFLOP/s"
    else:
        ach, peak, unit = nbytes / us / 1e3, HBM_PEAK_GBS, "GB/s"
    r = {"kernel": name, "bound": bound, "achieved": round(ach, 2), "peak": peak, "unit": unit,
         "frac": round(ach / peak, 4), "traffic": traffic, "us": round(us, 3)}
    if note:
        r["shape"] = note
    return r


class Leg:
    """One model configuration on the device: weights, tables, sources, and (per fingerprint variant) the banks."""

    def __init__(self, cfg, args, llmc, W, GatedStack):
        import torch
        self.cfg, self.args, self.llmc, self.W, self.GatedStack, self.torch = cfg, args, llmc, W, GatedStack, torch
        self.dev = "cuda"
        self.ws = W.make_layer_weights(cfg, seed=0)
        tok, pos = W.make_embeddings(cfg, seed=0)
        self.tok, self.pos = tok.to(self.dev), pos.to(self.dev)
        self.Ps = W.make_projection(cfg.d, cfg.k, cfg.torch_dtype, seed=3, n_layers=cfg.n_layers)
        self.src = W.make_sources(cfg, cfg.n_bank, seed=1)
        self.src_t = torch.from_numpy(self.src).to(self.dev)
        self.offsets = None
        self.st = None
        self.variant = None

    def embed(self, ids):
        torch = self.torch
        t = ids if isinstance(ids, torch.Tensor) else torch.from_numpy(ids).to(self.dev)
        return self.W.embed(t, self.tok, self.pos, self.cfg.torch_dtype)

    def source_batches(self):
        for s in range(0, self.cfg.n_bank, self.cfg.B):
            yield self.embed(self.src_t[s:s + self.cfg.B])

    def centring(self):
        """c_l = -P_l^T mu_l from an uncached forward of the bank sources (inputs of the path, like P_l)."""
        if self.offsets is None:
            from paper_2512_16843_amd.centring import centring_offsets
            t0 = time.time()
            self.offsets = centring_offsets(self.cfg, self.ws, self.Ps, self.source_batches())
            log("%s: centring offsets from %d sources in %.1f s" % (self.cfg.name, self.cfg.n_bank, time.time() - t0))
        return self.offsets

    def build_prefix_maps(self, weight=3.0):
        """Keys from the token average AND the prefix attention statistics (first quarter of the tokens, the shortest
        prefix a query of this workload shares with its source): the map of the second feature is a second seeded
        Gaussian, scaled per layer so that the centred attention feature carries `weight` times the length of the
        centred token average; both features are centred on the bank sources."""
        from paper_2512_16843_amd.centring import prefix_feature_stats
        torch, cfg, W = self.torch, self.cfg, self.W
        self.prefix_tokens = cfg.S // 4
        Pa = W.make_projection(cfg.d, cfg.k, cfg.torch_dtype, seed=13, n_layers=cfg.n_layers)
        t0 = time.time()
        stats = prefix_feature_stats(cfg, self.ws, [torch.cat([self.Ps[l], Pa[l]]) for l in range(cfg.n_layers)],
                                     self.source_batches(), self.prefix_tokens)
        self.P2, cs = [], []
        for l, (mu, var_p, var_a) in enumerate(stats):
            w = weight * (var_p / max(var_a, 1e-30)) ** 0.5
            P2 = torch.cat([self.Ps[l].float(), Pa[l].float() * w]).to(cfg.torch_dtype)
            self.P2.append(P2)
            cs.append((-(mu @ P2.to(torch.float64))).to(torch.float32).contiguous())
        log("%s: centring of both fingerprint features over %d sources in %.1f s" % (cfg.name, cfg.n_bank, time.time() - t0))
        return cs

    def build(self, variant):
        """Banks of one fingerprint variant, built by the all-miss forward with insertion over the sources."""
        torch, cfg, llmc = self.torch, self.cfg, self.llmc
        self.close()
        cs = self.centring() if variant == "centred" else None
        carry = not self.args.no_carry
        if variant == "centred+prefix":
            cs = self.build_prefix_maps()
            self.st = self.GatedStack(cfg, self.ws, self.Ps, biases=cs, prefix_tokens=self.prefix_tokens, proj2=self.P2)
        else:
            self.st = self.GatedStack(cfg, self.ws, self.Ps, biases=cs, keep_means=carry, keep_next_keys=carry)
        self.variant, self.cs = variant, cs
        torch.cuda.synchronize()
        t0 = time.time()
        for h in self.source_batches():
            self.st.forward(h, tau=2.0, flags=llmc.INSERT_ON_MISS, tick=1)
        torch.cuda.synchronize()
        self.build_s = time.time() - t0
        assert all(int(b.valid.sum()) == cfg.n_bank for b in self.st.banks)
        log("%s %s: banks built, %d sequences x %d layers in %.1f s (%.1f seq/s all-miss with insertion)"
            % (cfg.name, variant, cfg.n_bank, cfg.n_layers, self.build_s, cfg.n_bank / self.build_s))
        return self.st

    def close(self):
        if self.st is not None:
            self.st.close()
            self.st = None
            self.torch.cuda.empty_cache()

    def run(self, h, tau, steps, warmup):
        """W untimed eager steps (they also settle the engine's launch-shape hints), then K timed steps: replays of
        a HIP graph that records the step's library launches and nothing else (or eager launches with --no-graph)."""
        torch, st = self.torch, self.st
        for _ in range(warmup):
            st.forward(h, tau=tau)
        torch.cuda.synchronize()
        if self.args.no_graph:
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
        return dt, st.hit_counts().numpy()

    def row(self, tau, dt, cnt, **extra):
        cfg, llmc = self.cfg, self.llmc
        hits = cnt[:, llmc.CNT_HIT]
        r = {"variant": self.variant, "tau": tau if tau <= 1.0 else "no-cache", "ms_per_step": round(dt * 1e3, 4),
             "seq_per_s": round(cfg.B / dt, 2), "hit_rate": round(float(hits.sum()) / (cfg.B * cfg.n_layers), 4),
             "hit_rate_first_layer": round(float(hits[0]) / cfg.B, 4),
             "hit_rate_last_layer": round(float(hits[-1]) / cfg.B, 4),
             "near_tau_rows": int(cnt[:, llmc.CNT_NEAR_TAU].sum()), "near_tie_rows": int(cnt[:, llmc.CNT_NEAR_TIE].sum())}
        r.update(extra)
        log("%s %s tau=%s%s  %.3f ms/step  %.1f seq/s  hit rate %.3f (layer 1: %.3f, layer %d: %.3f)"
            % (cfg.name, self.variant, r["tau"], "".join(" %s=%s" % kv for kv in extra.items()), r["ms_per_step"],
               r["seq_per_s"], r["hit_rate"], r["hit_rate_first_layer"], cfg.n_layers, r["hit_rate_last_layer"]))
        return r

    def dial(self, rhos, steps, warmup):
        """Hit-rate dial: a fraction rho of the rows are exact copies of bank sources (similarity 1), the rest
        fresh; at a threshold just below 1 only the copies hit, so the measured hit rate follows rho."""
        out = []
        for rho in rhos:
            ids, _ = self.W.make_dial_queries(self.cfg, self.src, rho, seed=7)
            h = self.embed(ids)
            dt, cnt = self.run(h, DIAL_TAU, steps, warmup)
            out.append(self.row(DIAL_TAU, dt, cnt, rho=rho))
            del h
        return out

    def profile(self, h, tau, steps=5):
        """Per-kernel durations of `steps` eager steps: the library launches every kernel with its own start / stop
        events while recording is on."""
        torch, st, cfg, llmc = self.torch, self.st, self.cfg, self.llmc
        for _ in range(2):
            st.forward(h, tau=tau)
            torch.cuda.synchronize()
        llmc.llmc_profile_begin(steps * cfg.n_layers * 24)
        for _ in range(steps):
            st.forward(h, tau=tau)
        rep = llmc.llmc_profile_report()
        llmc.llmc_profile_end()
        cnt = st.hit_counts().numpy()
        miss = [int(x) for x in cnt[:, llmc.CNT_MISS]]
        hit = [int(x) for x in cnt[:, llmc.CNT_HIT]]
        copied = st.copied_rows()
        out = {}
        total_ms = sum(ms for _, ms in rep.values()) / steps
        for name, (n, ms) in rep.items():
            fl, by, bound = kernel_work(cfg, name, miss, hit, carry=not self.args.no_carry, copied=copied)
            t_step = ms * 1e-3 / steps
            out[name] = {"launches_per_step": n // steps, "avg_us": round(ms * 1e3 / n, 3),
                         "ms_per_step": round(ms / steps, 4), "share": round(ms / steps / total_ms, 4), "bound": bound,
                         "flops_per_step": fl, "bytes_per_step": by,
                         "tflops": round(fl / t_step / 1e12, 3) if t_step > 0 else 0.0,
                         "gbs": round(by / t_step / 1e9, 2) if t_step > 0 else 0.0}
        return out, total_ms


def show_profile(tag, pr):
    for name, r in sorted(pr.items(), key=lambda kv: -kv[1]["ms_per_step"]):
        log("%-16s %-24s %3d launches/step  avg %9.2f us  %8.4f ms/step (%4.1f%%)  %8.2f TFLOP/s %9.1f GB/s"
            % (tag, name, r["launches_per_step"], r["avg_us"], r["ms_per_step"], 100 * r["share"], r["tflops"], r["gbs"]))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--tau", type=float, default=0.95, help="headline threshold")
    ap.add_argument("--workload", choices=["bert-base", "gpt2-small", "bert-large-dynamic"], default="bert-base",
                    help="bert-base: the configuration the metric is quoted on, with compact legs of the other two "
                         "(default); gpt2-small / bert-large-dynamic: that configuration alone")
    ap.add_argument("--no-dial", action="store_true", help="skip the hit-rate dial leg")
    ap.add_argument("--no-graph", action="store_true",
                    help="enqueue every timed step from Python instead of replaying a HIP graph of it")
    ap.add_argument("--no-carry", action="store_true",
                    help="banks keep neither the token mean nor the next-layer key of cached outputs (every layer pools "
                         "and projects every row again)")
    ap.add_argument("--bank", type=int, default=None, help="bank entries per layer (default: the config's)")
    ap.add_argument("--layers", type=int, default=None, help="debug: fewer layers")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stress", action="store_true", help="skip the 1M-key bank-match stress leg")
    ap.add_argument("--no-other-legs", action="store_true", help="skip the GPT-2-small and BERT-large legs of the default run")
    ap.add_argument("--counters-only", action="store_true",
                    help="for hardware-counter runs (rocprofv3 --pmc): the calibration copy, then warm-up and timed steps "
                         "of the headline configuration launched eagerly, and nothing else (no per-kernel event timing)")
    ap.add_argument("--cpu-rows", type=int, default=2, help="sequences of the batch the oracle is first timed on")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the path runs on ONE GPU (it is single-device); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2512_16843_amd import llmc, workloads as W
    from paper_2512_16843_amd.engine import GatedStack

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    llmc.lib()

    def scaled(cfg):
        if args.bank or args.layers:
            return W.scaled(cfg, n_bank=args.bank or cfg.n_bank, n_layers=args.layers or cfg.n_layers)
        return cfg

    if args.workload == "bert-large-dynamic":
        print(json.dumps(bench_dynamic(args, llmc, W, GatedStack, scaled(W.BERT_LARGE), full_line=True)))
        return
    if args.workload == "gpt2-small":
        print(json.dumps(bench_decoder(args, llmc, W, GatedStack, scaled(W.GPT2_SMALL), full_line=True)))
        return

    # a plain device-to-device copy of known size: the reference against which HBM byte counters
    # (FETCH_SIZE / WRITE_SIZE) of a profiled run are scaled
    cal_src = torch.full((CALIB_COPY_BYTES,), 7, dtype=torch.uint8, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    for _ in range(3):
        cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    if args.counters_only:
        args.no_graph = True
        cfg = scaled(W.BERT_BASE)
        leg = Leg(cfg, args, llmc, W, GatedStack)
        ids, _ = W.make_substitution_queries(cfg, leg.src, n_dup=int(round(0.6 * cfg.B)), n_subst=int(round(0.03 * cfg.S)), seed=2)
        h0 = leg.embed(ids)
        leg.build("centred")
        dt, cnt = leg.run(h0, args.tau, args.steps, args.warmup)
        print(json.dumps({"counters_only": True, "ms_per_step": round(dt * 1e3, 4), "steps": args.steps,
                          "warmup": args.warmup, "calib_copy_bytes": CALIB_COPY_BYTES,
                          "hit_rate": round(float(cnt[:, llmc.CNT_HIT].sum()) / (cfg.B * cfg.n_layers), 4)}))
        leg.close()
        return

    # ---- the other two model configurations first (their banks do not fit beside the BERT-base ones) ----------
    gpt2 = large = None
    if not args.no_other_legs:
        gpt2 = bench_decoder(args, llmc, W, GatedStack, scaled(W.GPT2_SMALL), full_line=False)
        large = bench_dynamic(args, llmc, W, GatedStack, scaled(W.BERT_LARGE), full_line=False)

    # ---- bank-match stress shape (1,048,576 keys x 256, 4,096 queries), its gather, pooling at 4,096 sequences ---
    stress = None
    if not args.no_stress:
        stress = match_stress(llmc, W)
        log("match stress: %.1f us -> %.1f TFLOP/s (%.1f%% of bf16 MFMA peak); finalize %.1f us; gather of %d hits "
            "%.1f us -> %.1f GB/s (%.1f%% of HBM peak); pooling of 4096 sequences %.1f us -> %.1f GB/s (%.1f%%)"
            % (stress["match_us"], stress["match_tflops"], 100 * stress["match_frac_mfma"], stress["finalize_us"],
               stress["hits"], stress["gather_us"], stress["gather_gbs"], 100 * stress["gather_frac_hbm"],
               stress["pool_us"], stress["pool_gbs"], 100 * stress["pool_frac_hbm"]))

    # ---- the configuration the metric is quoted on ----------------------------------------------------------------
    cfg = scaled(W.BERT_BASE)
    leg = Leg(cfg, args, llmc, W, GatedStack)
    # 60 % perturbed copies of bank sources (3 % of tokens resampled), 40 % fresh
    n_dup = int(round(0.6 * cfg.B))
    n_sub = int(round(0.03 * cfg.S))
    ids, srcmap = W.make_substitution_queries(cfg, leg.src, n_dup=n_dup, n_subst=n_sub, seed=2)
    recipe = "60% perturbed copies (3% tokens resampled) + 40% fresh"
    h0 = leg.embed(ids)
    taus = [0.90, 0.95, 0.98]
    sweep = []
    leg.build("uncentred")
    for tau in taus:
        dt, cnt = leg.run(h0, tau, args.steps, args.warmup)
        sweep.append(leg.row(tau, dt, cnt))
    st = leg.build("centred")
    for tau in [t for t in taus if t != args.tau] + [2.0]:
        dt, cnt = leg.run(h0, tau, args.steps, args.warmup)
        sweep.append(leg.row(tau, dt, cnt))
    dial = [] if args.no_dial else leg.dial((0.25, 0.5, 0.75, 0.9, 1.0), max(5, args.steps // 2), max(2, args.warmup // 2))

    prof_nocache, _ = leg.profile(h0, 2.0)
    prof_head, prof_total_ms = leg.profile(h0, args.tau)
    show_profile("tau=%s" % args.tau, prof_head)
    show_profile("no-cache", prof_nocache)
    launches_per_step = sum(r["launches_per_step"] for r in prof_head.values())

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, st, leg.ws, leg.Ps, leg.cs, h0, args.tau, args.cpu_rows)
        log("cpu oracle: %.3f seq/s on %d threads, %.3f seq/s on 1 thread (%s)"
            % (cpu["value"], cpu["cores"], cpu["single_core"]["value"], cpu["sample"]))
        if stress is not None:
            cpu["stress_match"] = stress.pop("cpu_oracle")

    # ---- headline: the last GPU work of the run ------------------------------------------------------
    dt_head, cnt_head = leg.run(h0, args.tau, args.steps, args.warmup)
    sweep.append(leg.row(args.tau, dt_head, cnt_head))
    sweep.sort(key=lambda r: (r["variant"], r["tau"] == "no-cache", r["tau"] if r["tau"] != "no-cache" else 9))
    log("library kernel launches per step at the headline threshold: %d; sum of kernel durations %.3f ms, step %.3f ms"
        % (launches_per_step, prof_total_ms, dt_head * 1e3))

    # roofline: the kernel with the largest share of the headline step's kernel time, whatever it is
    name, r = max(prof_head.items(), key=lambda kv: kv[1]["ms_per_step"])
    us_step = r["ms_per_step"] * 1e3
    roof = roof_entry(name, r["bound"], r["flops_per_step"], r["bytes_per_step"], us_step, traffic=measured_traffic(name))
    roof.update({"share_of_step": r["share"], "launches_per_step": r["launches_per_step"], "avg_launch_us": r["avg_us"],
                 "note": "all launches of the kernel in one headline step: their algorithmic work / their summed duration"})
    del roof["us"]
    rooflines = []
    for kname in ("gemm_bf16_kernel", "attention_kernel", "layernorm_kernel", "pool_kernel", "gather_kernel",
                  "match_stream_kernel", "match_finalize_kernel"):
        for tag, pr in (("headline", prof_head), ("no_cache", prof_nocache)):
            if kname in pr and (pr[kname]["flops_per_step"] or pr[kname]["bytes_per_step"]) and kname != name:
                k_ = pr[kname]
                if tag == "no_cache" and any(x["kernel"] == kname for x in rooflines):
                    continue
                rooflines.append(roof_entry(kname, k_["bound"], k_["flops_per_step"], k_["bytes_per_step"],
                                            k_["ms_per_step"] * 1e3, note="%s step of the %s config" % (tag, cfg.name),
                                            traffic=measured_traffic(kname)))
    if stress is not None:
        rooflines += stress.pop("rooflines")

    result = {
        "metric": METRIC, "value": round(cfg.B / dt_head, 2), "unit": "seq/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(dt_head * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s encoder: %d layers, d=%d, batch %d x %d tokens, bank %d x k=%d per layer, %s, static banks"
                               % (cfg.name, cfg.n_layers, cfg.d, cfg.B, cfg.S, cfg.n_bank, cfg.k, recipe),
                   "tau": args.tau, "variant": "centred fingerprint (c = -P^T mu of the bank sources)",
                   "hit_rate": round(float(cnt_head[:, llmc.CNT_HIT].sum()) / (cfg.B * cfg.n_layers), 4),
                   "bank_build_s": round(leg.build_s, 2), "launches_per_step": launches_per_step,
                   "timed_steps": "eager launches from Python" if args.no_graph else "replays of a HIP graph of one step",
                   "carried_keys_and_deferred_copies": not args.no_carry},
        "sweep": sweep,
        "dial": dial,
        "roofline": roof,
        "rooflines": rooflines,
        "kernels": {"headline": prof_head, "no_cache": prof_nocache},
        "match_stress": stress,
        "gpt2_small": gpt2,
        "bert_large_dynamic": large,
        "cpu_baseline": cpu,
    }
    leg.close()
    print(json.dumps(result))


def match_stress(llmc, W, iters=10):
    """Top-1 cosine + threshold over a 1,048,576-key clustered bank for 4,096 queries, the gather of the matched
    384 x 768 outputs for the hits, and the pooling of 4,096 sequences; per-kernel times from the library's events."""
    import numpy as np
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
    P = (torch.randn((d, k), device="cuda") / k ** 0.5).to(torch.bfloat16)
    fp = torch.empty((B, k), dtype=torch.bfloat16, device="cuda")
    finv = torch.empty((B,), dtype=torch.float32, device="cuda")
    ws_fp = torch.empty((llmc.llmc_fingerprint_workspace_bytes(B, S, d),), dtype=torch.uint8, device="cuda")
    llmc.llmc_match(bank, q, qinv, tau, idx, sim, hit, None, ws)
    rows = torch.nonzero(hit).flatten().int().contiguous()
    n = torch.tensor([rows.numel()], dtype=torch.int32, device="cuda")
    llmc.llmc_gather_hits(bank, idx, rows, n, B, out)
    llmc.llmc_fingerprint(bank.act, P, None, fp, finv, ws_fp)
    torch.cuda.synchronize()
    llmc.llmc_profile_begin(8 * iters)
    for _ in range(iters):
        llmc.llmc_match(bank, q, qinv, tau, idx, sim, hit, None, ws)
        llmc.llmc_gather_hits(bank, idx, rows, n, B, out)
        llmc.llmc_fingerprint(bank.act, P, None, fp, finv, ws_fp)        # 4,096 sequences of 384 x 768, 2.4 GB
    rep = llmc.llmc_profile_report()
    llmc.llmc_profile_end()
    us = {name: ms * 1e3 / cnt for name, (cnt, ms) in rep.items()}
    H = int(rows.numel())
    m_us, g_us, p_us = us["match_stream_kernel"], us["gather_kernel"], us["pool_kernel"]
    fin_us = us.get("match_finalize_kernel", 0.0)
    tfl = 2.0 * B * N * k / m_us / 1e6
    gbs = 2.0 * H * S * d * 2 / g_us / 1e3
    pgbs = float(A) * S * d * 2 / p_us / 1e3
    shape = "1,048,576 bf16 keys x 256, 4,096 queries"
    rooflines = [roof_entry("match_stream_kernel", "mfma", 2.0 * B * N * k, float(N) * k * 2, m_us, note=shape,
                            traffic=measured_traffic("match_skew_kernel")),
                 roof_entry("gather_kernel", "hbm", 0.0, 2.0 * H * S * d * 2, g_us,
                            note="%d rows of 384 x 768 bf16" % H, traffic=measured_traffic("gather_kernel@stress")),
                 roof_entry("pool_kernel", "hbm", 0.0, float(A) * S * d * 2, p_us, note="4,096 sequences of 384 x 768 bf16",
                            traffic=measured_traffic("pool_kernel@stress"))]

    # ---- the CPU oracle's match on a sample of the same queries (all threads, then one) ----
    cpu_oracle = stress_cpu_oracle(q, qinv, bank, idx)

    # ---- the same bank and queries as sign-bit keys: each 256-vector is projected by a seeded Gaussian P
    # [256, 256] and only the signs are kept (32 bytes per key instead of 512); match by Hamming distance ----
    kb = 256
    gen = torch.Generator(device="cuda").manual_seed(21)
    Pb = (torch.randn((k, kb), generator=gen, device="cuda") / kb ** 0.5).to(torch.bfloat16)
    bank_bits = torch.empty((N, kb // 32), dtype=torch.int32, device="cuda")
    q_bits = torch.empty((B, kb // 32), dtype=torch.int32, device="cuda")
    chunk = 32768
    ws_f = torch.empty((llmc.llmc_fingerprint_workspace_bytes(chunk, 1, k),), dtype=torch.uint8, device="cuda")
    for s0 in range(0, N, chunk):
        llmc.llmc_fingerprint_bits(bank.fp[s0:s0 + chunk].view(-1, 1, k), Pb, None, bank_bits[s0:s0 + chunk], ws_f)
    llmc.llmc_fingerprint_bits(q.view(B, 1, k), Pb, None, q_bits, ws_f)
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
    # 4,096 queries of 256-bit keys run as an int8 matrix product; 256 queries at a time stay on the vector ALU
    # (XOR + popcount): time that scan on the first 256 queries for comparison
    Bv = 256
    ws_v = torch.empty((llmc.llmc_match_bits_workspace_bytes(N, kb, Bv),), dtype=torch.uint8, device="cuda")
    qv_bits = q_bits[:Bv].contiguous()
    llmc.llmc_match_bits(bank_bits, bank.valid, qv_bits, max_h, idx_b[:Bv], dist_b[:Bv], hit_b[:Bv], ws_v)
    torch.cuda.synchronize()
    llmc.llmc_profile_begin(4 * iters)
    for _ in range(iters):
        llmc.llmc_match_bits(bank_bits, bank.valid, qv_bits, max_h, idx_b[:Bv], dist_b[:Bv], hit_b[:Bv], ws_v)
    rep_v = llmc.llmc_profile_report()
    llmc.llmc_profile_end()
    us_v = {name: ms * 1e3 / cnt for name, (cnt, ms) in rep_v.items()}
    del ws_v
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
    word_ops = 2.0 * Bv * N * (kb // 32)                 # one XOR and one popcount-accumulate per 32 bit pairs
    int8_ops = 2.0 * B * N * kb                          # the same scan as a product of 0/1 bytes
    mma_us = us_b["match_bits_mma_kernel"]
    bits = {"key_bits": kb, "bank_bytes": N * kb // 8, "max_hamming": int(max_h),
            "match_us": round(mma_us, 2),
            "other_us": round(sum(v for n_, v in us_b.items() if n_ != "match_bits_mma_kernel"), 2),
            "int8_peta_ops_per_s": round(int8_ops / mma_us / 1e9, 3),
            "frac_int8_mfma_peak": round(int8_ops / mma_us / 1e6 / MFMA_INT8_PEAK_TOPS, 4),
            "vector_scan_256_queries": {
                "match_us": round(us_v["match_bits_kernel"], 2),
                "tera_word_ops_per_s": round(word_ops / us_v["match_bits_kernel"] / 1e6, 2),
                "frac_int_valu_peak": round(word_ops / us_v["match_bits_kernel"] / 1e6 / INT_VALU_PEAK_TOPS, 4)},
            "hits": int(hit_b.sum()), "same_cluster_as_cosine_match_on_hits": round(same_cluster, 4),
            "same_decision_as_cosine_match": round(same_decision, 4), "lsh": lsh}
    log("sign-bit keys on the same bank (%d bits, %d MB instead of 512): Hamming match on the matrix cores %.1f us -> "
        "%.2f P int8-ops/s (%.1f%% of the int8 peak); vector scan of 256 queries %.1f us (%.1f%% of the integer "
        "vector peak); bucketed lookup %.1f us (index build %.1f us), same decision %.4f"
        % (kb, bits["bank_bytes"] >> 20, bits["match_us"], bits["int8_peta_ops_per_s"], 100 * bits["frac_int8_mfma_peak"],
           us_v["match_bits_kernel"], 100 * bits["vector_scan_256_queries"]["frac_int_valu_peak"],
           lsh["match_us"], lsh["build_us"], lsh["same_decision_as_full_match"]))
    del bank_bits, q_bits, ws_f, ws_b
    bank.close()
    res = {"workload": "bank-match stress: 1,048,576 bf16 keys x 256 in 4,096 clusters, 4,096 queries, tau 0.95, "
                       "gather of 384 x 768 bf16 outputs for the hits",
           "hits": H, "match_us": round(m_us, 2), "match_tflops": round(tfl, 1),
           "match_frac_mfma": round(tfl / MFMA_BF16_PEAK_TFLOPS, 4), "finalize_us": round(fin_us, 2),
           "gather_us": round(g_us, 2), "gather_gbs": round(gbs, 1), "gather_frac_hbm": round(gbs / HBM_PEAK_GBS, 4),
           "pool_us": round(p_us, 2), "pool_gbs": round(pgbs, 1), "pool_frac_hbm": round(pgbs / HBM_PEAK_GBS, 4),
           "sign_bit_keys": bits, "rooflines": rooflines, "cpu_oracle": cpu_oracle}
    del bank, out
    torch.cuda.empty_cache()
    return res


def host_threads():
    try:
        from threadpoolctl import threadpool_info
        return max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        return os.cpu_count() or 1


def stress_cpu_oracle(q, qinv, bank, idx_gpu, n_queries=128):
    """The oracle's match (fp64, all 1,048,576 keys) on the first queries of the stress batch: all threads, one thread."""
    import numpy as np
    from threadpoolctl import threadpool_limits
    from oracle import llmc_oracle as O
    npf = lambda t: t.detach().float().cpu().numpy()
    fp, inv = npf(bank.fp), npf(bank.inv_norm)
    valid = np.ones(fp.shape[0], np.uint8)
    qs, qis = npf(q[:n_queries]), npf(qinv[:n_queries])
    out = {"unit": "queries/s", "kind": "oracle",
           "sample": "first %d of 4,096 queries against all 1,048,576 keys (fp64)" % n_queries}
    for tag, limit in (("all", None), ("one", 1)):
        t = time.perf_counter()
        if limit:
            with threadpool_limits(limits=limit):
                oi, _ = O.match(qs, qis, fp, inv, valid)
        else:
            oi, _ = O.match(qs, qis, fp, inv, valid)
        dt = time.perf_counter() - t
        if tag == "all":
            out["value"], out["cores"], out["seconds"] = round(n_queries / dt, 2), int(host_threads()), round(dt, 2)
            out["agree_with_gpu"] = int((oi == idx_gpu[:n_queries].cpu().numpy()).sum())
        else:
            out["single_core"] = {"value": round(n_queries / dt, 2), "cores": 1, "seconds": round(dt, 2)}
    log("cpu oracle on the stress match: %.1f queries/s on %d threads, %.1f on one (%d of %d slots equal to the GPU's)"
        % (out["value"], out["cores"], out["single_core"]["value"], out["agree_with_gpu"], n_queries))
    return out


def cpu_baseline(cfg, st, ws, Ps, cs, h0, tau, n_rows):
    """Time the oracle's gated forward (all layers) on the first rows of the batch, on all host threads and on one.

    The oracle reads the banks the GPU built: keys come to the host whole, cached
    outputs are fetched row by row when a hit needs them.
    """
    import numpy as np
    import torch
    from threadpoolctl import threadpool_limits
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
    cnp = [None if cs is None else npf(c) for c in (cs or [None] * cfg.n_layers)]
    tau32 = float(np.float32(tau))

    def timed(n, limit):
        x = npf(h0[:n])
        t = time.perf_counter()
        if limit:
            with threadpool_limits(limits=limit):
                _, res = O.infer(x, banks, Pnp, cnp, wnp, cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu, tau=tau32,
                                 out_dtype=cfg.dtype)
        else:
            _, res = O.infer(x, banks, Pnp, cnp, wnp, cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu, tau=tau32,
                             out_dtype=cfg.dtype)
        return time.perf_counter() - t, sum(int(r.hit.sum()) for r in res)

    def sample(limit, budget):
        """Grow the sample (a prefix of the batch) until one pass takes about `budget` seconds."""
        n = max(1, min(n_rows, cfg.B))
        while True:
            dt, hits = timed(n, limit)
            if dt >= 0.6 * budget or n >= cfg.B:
                return n, dt, hits
            n = min(cfg.B, max(n + 1, int(n * min(8.0, budget / max(dt, 1e-3)))))

    n, dt, hits = sample(None, 12.0)
    n1, dt1, hits1 = sample(1, 10.0)
    cores = int(host_threads())
    return {"value": round(n / dt, 4), "unit": "seq/s", "cores": cores, "kind": "oracle",
            "sample": "one pass over the first %d of %d sequences of the batch through all %d layers at tau=%s against the "
                      "GPU-built banks (%d of %d row-layers hit), %.1f s"
                      % (n, cfg.B, cfg.n_layers, tau, hits, n * cfg.n_layers, dt),
            "single_core": {"value": round(n1 / dt1, 4), "unit": "seq/s", "cores": 1,
                            "sample": "the first %d sequences, %d of %d row-layers hit, %.1f s"
                                      % (n1, hits1, n1 * cfg.n_layers, dt1)}}


def bench_decoder(args, llmc, W, GatedStack, cfg, full_line):
    """GPT-2-small-shaped causal decoder: every query shares a prefix of random length (25-75 % of the sequence)
    with a bank source and continues with a fresh suffix."""
    import torch
    leg = Leg(cfg, args, llmc, W, GatedStack)
    ids, srcmap, _ = W.make_prefix_queries(cfg, leg.src, seed=2)
    h0 = leg.embed(ids)
    steps, warmup = max(5, args.steps // 2), max(2, args.warmup // 2)
    sweep = []
    leg.build("uncentred")
    dt, cnt = leg.run(h0, 0.95, steps, warmup)
    sweep.append(leg.row(0.95, dt, cnt))
    leg.build("centred")
    for tau in (0.5, 0.95, 2.0):
        dt, cnt = leg.run(h0, tau, steps, warmup)
        sweep.append(leg.row(tau, dt, cnt))
    head = sweep[-2]
    dial = [] if args.no_dial else leg.dial((0.5, 0.875), steps, warmup)
    # the same queries under keys that include the prefix attention statistics (Section IV-B): a query shares at
    # least its first quarter with its source, and a causal block's prefix feature depends on those tokens only
    leg.build("centred+prefix")
    for tau in (0.9, 0.95):
        dt, cnt = leg.run(h0, tau, steps, warmup)
        sweep.append(leg.row(tau, dt, cnt, prefix_tokens=leg.prefix_tokens))
    prof = None
    if full_line:
        prof, _ = leg.profile(h0, 2.0)
        show_profile("no-cache", prof)
    leg.close()
    del leg
    torch.cuda.empty_cache()
    res = {"workload": "%s causal decoder: %d layers, d=%d, batch %d x %d tokens, bank %d x k=%d per layer, each query = a "
                       "bank source's prefix of 25-75 %% of the tokens + a fresh suffix, static banks"
                       % (cfg.name, cfg.n_layers, cfg.d, cfg.B, cfg.S, cfg.n_bank, cfg.k),
           "sweep": sweep, "dial": dial}
    if not full_line:
        return res
    nc = [r for r in sweep if r["tau"] == "no-cache"][-1]
    return {"metric": METRIC, "value": head["seq_per_s"], "unit": "seq/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
            "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16", "data": "synthetic", "config": {"workload": res["workload"], "tau": 0.95, "variant": "centred",
                                                             "hit_rate": head["hit_rate"]},
            "sweep": sweep, "dial": dial, "no_cache_seq_per_s": nc["seq_per_s"], "kernels": {"no_cache": prof},
            "roofline": None, "cpu_baseline": None}


def bench_dynamic(args, llmc, W, GatedStack, cfg, full_line):
    """BERT-large-shaped stack with bank insertion and LRU eviction active: banks pre-filled to capacity by a
    warm-up stream, then segments of 50 successive batches of stem-sharing candidates (64 groups of 4 sequences
    sharing an 80-token stem).  A step is one batch through all 24 layers, inserts and evictions included."""
    import torch
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
    log("%s: banks pre-filled: %d batches x %d layers in %.1f s (%.1f seq/s all-miss with insertion)"
        % (cfg.name, cfg.n_bank // cfg.B, cfg.n_layers, fill_s, cfg.n_bank / fill_s))
    n_batches, segments = 50, []
    n_seg = 3 if full_line else 2
    # the last segment also uses within-batch reuse: candidates of one group whose stem makes them similar enough
    # follow the group's first candidate instead of being computed and stored again
    for seg in range(n_seg + 1):
        seg_flags = flags | (llmc.DEDUP if seg == n_seg else 0)
        hs = []
        for _ in range(n_batches):
            ids, _ = stream.next_batch()
            hs.append(W.embed(torch.from_numpy(ids).to(dev), tok, pos, cfg.torch_dtype))
        counters = []
        torch.cuda.synchronize()
        t = time.perf_counter()
        for h in hs:
            tick += 1
            st.forward(h, tau=args.tau, flags=seg_flags, tick=tick)
            counters.append(torch.stack([g.counters for g in st.gate]))      # device-side copy, no host sync
        torch.cuda.synchronize()
        dt = time.perf_counter() - t
        cnt = torch.stack(counters).cpu().numpy()                            # [batch, layer, word]
        hit_rate = cnt[:, :, llmc.CNT_HIT].sum(axis=1) / float(cfg.B * cfg.n_layers)
        segments.append({"batches": n_batches, "seconds": round(dt, 4), "seq_per_s": round(n_batches * cfg.B / dt, 2),
                         "hit_rate": round(float(hit_rate.mean()), 4),
                         "hit_rate_first_last_batch": [round(float(hit_rate[0]), 4), round(float(hit_rate[-1]), 4)],
                         "inserted": int(cnt[:, :, llmc.CNT_INSERTED].sum()),
                         "evicted": int(cnt[:, :, llmc.CNT_EVICTED].sum()),
                         "within_batch_reuse": seg == n_seg,
                         "followers": int(cnt[:, :, llmc.CNT_DEDUP].sum())})
        log("%s segment %d: %d batches in %.3f s -> %.1f seq/s, hit rate %.3f, %d inserts, %d evictions"
            % (cfg.name, seg, n_batches, dt, segments[-1]["seq_per_s"], segments[-1]["hit_rate"],
               segments[-1]["inserted"], segments[-1]["evicted"]))
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
    log("%s no-cache: %.1f seq/s" % (cfg.name, nocache))
    best = max(segments[:n_seg], key=lambda r: r["seq_per_s"])
    last = segments[n_seg - 1]
    st.close()
    del st
    torch.cuda.empty_cache()
    workload = ("%s encoder, dynamic banks: %d layers, d=%d, batch %d x %d tokens (64 groups of 4 candidates sharing an "
                "80-token stem, 512 recurring stems), bank %d x k=%d per layer pre-filled to capacity, INSERT_ON_MISS | "
                "UPDATE_LRU, every miss evicts; uncentred fingerprint; steps enqueued from Python"
                % (cfg.name, cfg.n_layers, cfg.d, cfg.B, cfg.S, cfg.n_bank, cfg.k))
    res = {"workload": workload, "tau": args.tau, "segments": segments, "no_cache_seq_per_s": round(nocache, 2),
           "best_segment_seq_per_s": best["seq_per_s"], "prefill_s": round(fill_s, 1)}
    if not full_line:
        return res
    return {"metric": METRIC, "value": last["seq_per_s"], "unit": "seq/s", "n_gpus": 1, "steps": n_batches, "warmup": 0,
            "ms_per_step": round(last["seconds"] / n_batches * 1e3, 4), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": workload, "tau": args.tau, "hit_rate": last["hit_rate"], "prefill_s": round(fill_s, 1)},
            "segments": segments, "no_cache_seq_per_s": round(nocache, 2), "best_segment_seq_per_s": best["seq_per_s"],
            "roofline": None, "cpu_baseline": None}


if __name__ == "__main__":
    main()
