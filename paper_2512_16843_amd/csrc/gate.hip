// The decision gate (Section III-D of the paper): turn the per-row hit flags into
// compacted, ascending lists of hit rows and miss rows with device-side counts, record
// hits in the bank (Section IV-D: recency), and copy the cached outputs of the hit rows
// (Algorithm 1: h_l <- h').
#include "common.h"

namespace llmc {

// One workgroup of 1024 threads walks the batch in ascending chunks; within a chunk a
// ballot + popcount gives each row its rank among the hits (and among the misses).
__global__ __launch_bounds__(1024) void compact_kernel(const uint8_t* __restrict__ hit, const int32_t* __restrict__ idx,
                                                       const float* __restrict__ sim, const uint8_t* __restrict__ tie,
                                                       int B, float tau, int32_t* __restrict__ hit_rows,
                                                       int32_t* __restrict__ miss_rows, int32_t* __restrict__ counters,
                                                       uint64_t* last_used, uint32_t* hits, int touch, uint64_t tick) {
  __shared__ int wave_hits[16];
  __shared__ int base_hit, base_miss, s_near_tau, s_near_tie;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) { base_hit = 0; base_miss = 0; s_near_tau = 0; s_near_tie = 0; }
  __syncthreads();
  for (int c0 = 0; c0 < B; c0 += 1024) {
    const int b = c0 + tid;
    const bool in = b < B;
    const bool h = in && hit[b] != 0;
    const unsigned long long bal = __ballot(h);
    const int before = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) wave_hits[wave] = __popcll(bal);
    __syncthreads();
    int wbase = 0, total = 0;
    for (int w = 0; w < 16; ++w) {
      if (w < wave) wbase += wave_hits[w];
      total += wave_hits[w];
    }
    const int n_in = min(1024, B - c0);
    if (in) {
      const int hrank = wbase + before;
      if (h) {
        hit_rows[base_hit + hrank] = b;
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
    }
    __syncthreads();
    if (tid == 0) { base_hit += total; base_miss += n_in - total; }
    __syncthreads();
  }
  if (tid == 0) {
    counters[LLMC_CNT_HIT] = base_hit;
    counters[LLMC_CNT_MISS] = base_miss;
    counters[LLMC_CNT_NEAR_TAU] = s_near_tau;
    counters[LLMC_CNT_NEAR_TIE] = s_near_tie;
    counters[LLMC_CNT_INSERTED] = 0;
    counters[LLMC_CNT_EVICTED] = 0;
    counters[LLMC_CNT_DROPPED] = 0;
    counters[7] = 0;
  }
}

// uncached layer: every row is a miss
__global__ void all_miss_kernel(int B, int32_t* miss_rows, int32_t* counters, int32_t* idx, float* sim, uint8_t* hit) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) {
    miss_rows[b] = b;
    if (idx) idx[b] = -1;
    if (sim) sim[b] = -INFINITY;
    if (hit) hit[b] = 0;
  }
  if (b < LLMC_CNT_WORDS) counters[b] = b == LLMC_CNT_MISS ? B : 0;
}

// Copy of cached outputs: grid (chunks, n_max); every thread moves 16-byte vectors.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
constexpr int kGatherThreads = 256;
constexpr int kGatherVecPerThread = 4;   // 16 KiB per workgroup: the launch shape that streamed fastest

__global__ __launch_bounds__(kGatherThreads) void gather_kernel(const u32x4_t* __restrict__ act, const int32_t* act_slot,
                                                                const int32_t* __restrict__ idx,
                                                                const int32_t* __restrict__ rows,
                                                                const int32_t* __restrict__ count, int n_max,
                                                                size_t vec_per_seq, u32x4_t* __restrict__ out) {
  const int n = count ? min(*count, n_max) : n_max;
  const int i = blockIdx.y;
  if (i >= n) return;
  const int b = rows ? rows[i] : i;
  const int j = idx[b];
  if (j < 0) return;
  const int slot = act_slot ? act_slot[j] : j;
  const u32x4_t* src = act + (size_t)slot * vec_per_seq;
  u32x4_t* dst = out + (size_t)b * vec_per_seq;
  const size_t v0 = (size_t)blockIdx.x * (kGatherThreads * kGatherVecPerThread) + threadIdx.x;
  u32x4_t r[kGatherVecPerThread];
#pragma unroll
  for (int u = 0; u < kGatherVecPerThread; ++u) {
    const size_t v = v0 + (size_t)u * kGatherThreads;
    if (v < vec_per_seq) r[u] = __builtin_nontemporal_load(src + v);
  }
#pragma unroll
  for (int u = 0; u < kGatherVecPerThread; ++u) {
    const size_t v = v0 + (size_t)u * kGatherThreads;
    if (v < vec_per_seq) __builtin_nontemporal_store(r[u], dst + v);
  }
}

llmc_status_t launch_compact(const uint8_t* d_hit, const int32_t* d_idx, const float* d_sim, const uint8_t* d_near_tie,
                             int B, float tau, int32_t* d_hit_rows, int32_t* d_miss_rows, int32_t* d_counters,
                             llmc_bank* bank, uint32_t flags, uint64_t tick, hipStream_t st) {
  const int touch = (flags & LLMC_UPDATE_LRU) ? 1 : 0;
  { ProfScope ps_("compact_kernel", st); hipLaunchKernelGGL(compact_kernel, dim3(1), dim3(1024), 0, st, d_hit, d_idx, d_sim, d_near_tie, B, tau, d_hit_rows,
                     d_miss_rows, d_counters, bank->desc.d_last_used, bank->desc.d_hits, touch, tick); }
  LLMC_LAUNCH_CHECK("compact_kernel");
  return LLMC_OK;
}

llmc_status_t launch_all_miss(int B, int32_t* d_miss_rows, int32_t* d_counters, int32_t* d_idx, float* d_sim,
                              uint8_t* d_hit, hipStream_t st) {
  const int n = B > LLMC_CNT_WORDS ? B : LLMC_CNT_WORDS;
  { ProfScope ps_("all_miss_kernel", st); hipLaunchKernelGGL(all_miss_kernel, dim3((n + 255) / 256), dim3(256), 0, st, B, d_miss_rows, d_counters, d_idx, d_sim,
                     d_hit); }
  LLMC_LAUNCH_CHECK("all_miss_kernel");
  return LLMC_OK;
}

llmc_status_t launch_gather(const llmc_bank* bank, const int32_t* d_idx, const int32_t* d_rows, const int32_t* d_n,
                            int n_max, void* d_h_out, hipStream_t st) {
  const llmc_bank_desc_t& D = bank->desc;
  const size_t vec_per_seq = (size_t)D.S * D.d * elem_size(D.dtype) / 16;
  const size_t per_wg = (size_t)kGatherThreads * kGatherVecPerThread;
  dim3 grid((unsigned)((vec_per_seq + per_wg - 1) / per_wg), n_max);
  { ProfScope ps_("gather_kernel", st); hipLaunchKernelGGL(gather_kernel, grid, dim3(kGatherThreads), 0, st, (const u32x4_t*)D.d_act, D.d_act_slot, d_idx,
                     d_rows, d_n, n_max, vec_per_seq, (u32x4_t*)d_h_out); }
  LLMC_LAUNCH_CHECK("gather_kernel");
  return LLMC_OK;
}

}  // namespace llmc
