// Compaction of the gate (Section III-D of the paper): per-row hit flags into ascending lists of reused rows and of
// rows to compute, with device-side counts; recency update of the entries that were hit (Section IV-D).
#pragma once
#include "common.h"

namespace llmc {

// Called by all 1024 threads of one workgroup, which walks the batch in ascending chunks; within a chunk a
// ballot + popcount gives each row its rank among the hits (and among the misses).
// Divergence monitor (Section IV-D): with reval_every = r >= 1 a hit row b with (tick + b) % r == 0
// is also appended, after all misses, to the list of rows to compute: miss_rows holds the misses in
// ascending order followed by those rows in ascending order; counters[COMPUTED] is the length of that
// list, counters[MISS] the number of real misses at its head.
__device__ __forceinline__ void compact_rows(const uint8_t* hit, const int32_t* __restrict__ idx,
                                                       const float* __restrict__ sim, const uint8_t* __restrict__ tie,
                                                       int B, float tau, int32_t* __restrict__ hit_rows,
                                                       int32_t* __restrict__ miss_rows, int32_t* __restrict__ counters,
                                                       uint64_t* last_used, uint32_t* hits, int touch, uint64_t tick,
                                                       int reval_every, int32_t* __restrict__ reval_tmp,
                                                       uint8_t* __restrict__ pooled_valid_out, int has_pool,
                                                       int32_t* __restrict__ ref_out,
                                                       const int32_t* __restrict__ act_slot) {
  __shared__ int wave_hits[16], wave_reval[16];
  __shared__ int base_hit, base_miss, base_reval, s_near_tau, s_near_tie, s_scanned;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) { base_hit = 0; base_miss = 0; base_reval = 0; s_near_tau = 0; s_near_tie = 0; s_scanned = 0; }
  __syncthreads();
  for (int c0 = 0; c0 < B; c0 += 1024) {
    const int b = c0 + tid;
    const bool in = b < B;
    const bool h = in && hit[b] != 0;
    const bool rv = h && reval_every > 0 && (tick + (uint64_t)b) % (uint64_t)reval_every == 0;
    const unsigned long long bal = __ballot(h), bal_rv = __ballot(rv);
    const unsigned long long below = (1ull << lane) - 1ull;
    const int before = __popcll(bal & below), before_rv = __popcll(bal_rv & below);
    if (lane == 0) { wave_hits[wave] = __popcll(bal); wave_reval[wave] = __popcll(bal_rv); }
    __syncthreads();
    int wbase = 0, total = 0, wbase_rv = 0, total_rv = 0;
    for (int w = 0; w < 16; ++w) {
      if (w < wave) { wbase += wave_hits[w]; wbase_rv += wave_reval[w]; }
      total += wave_hits[w];
      total_rv += wave_reval[w];
    }
    const int n_in = min(1024, B - c0);
    if (in) {
      const int hrank = wbase + before;
      // a row answered from the bank carries its stored token mean to the next layer; computed rows do not
      if (pooled_valid_out) pooled_valid_out[b] = (has_pool && h && !rv) ? 1 : 0;
      // deferred copy: a reused row is only a reference to the value row of its entry
      if (ref_out) {
        const int j = (h && !rv) ? idx[b] : -1;
        ref_out[b] = j < 0 ? -1 : (act_slot ? act_slot[j] : j);
      }
      if (h) {
        hit_rows[base_hit + hrank] = b;
        if (rv) reval_tmp[base_reval + wbase_rv + before_rv] = b;
        if (touch) {
          const int j = idx[b];
          last_used[j] = tick;            // several rows may name one slot: same value
          atomicAdd(&hits[j], 1u);
        }
      } else {
        miss_rows[base_miss + (tid - hrank)] = b;
      }
      if (sim && fabsf(sim[b] - tau) < 1e-3f) atomicAdd(&s_near_tau, 1);
      if (tie && tie[b]) atomicAdd(&s_near_tie, 1);
      if (tie && tie[b] > 1) atomicAdd(&s_scanned, 1);
    }
    __syncthreads();
    if (tid == 0) { base_hit += total; base_miss += n_in - total; base_reval += total_rv; }
    __syncthreads();
  }
  const int n_miss = base_miss, n_reval = base_reval;
  for (int i = tid; i < n_reval; i += 1024) miss_rows[n_miss + i] = reval_tmp[i];
  if (tid == 0) {
    counters[LLMC_CNT_HIT] = base_hit;
    counters[LLMC_CNT_MISS] = n_miss;
    counters[LLMC_CNT_NEAR_TAU] = s_near_tau;
    counters[LLMC_CNT_NEAR_TIE] = s_near_tie;
    counters[LLMC_CNT_INSERTED] = 0;
    counters[LLMC_CNT_EVICTED] = 0;
    counters[LLMC_CNT_DROPPED] = 0;
    counters[LLMC_CNT_COMPUTED] = n_miss + n_reval;
    counters[LLMC_CNT_REVALIDATED] = n_reval;
    counters[LLMC_CNT_DIVERGED] = 0;
    counters[LLMC_CNT_TIE_OVERFLOW] = s_scanned;
    counters[LLMC_CNT_DEDUP] = 0;
  }
}

}  // namespace llmc
