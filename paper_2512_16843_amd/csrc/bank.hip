// Bank updates run on the device as batched operations: Algorithm 1's store step
// C_l[f_X] <- h_l for all computed rows of a batch, and the least-recently-used
// replacement of Section IV-D of the paper.
//
// Slot selection orders the candidates by a 64-bit key
//     free slot:   (0              << 32) | slot
//     valid entry: ((last_used + 1) << 32) | slot
// so "free slots by ascending index, then entries by ascending (last_used, slot)" is the
// ascending order of distinct integers.  One workgroup finds the m-th smallest key with
// an 8-bit radix select (integer histograms only), collects the m keys not above it and
// ranks them by counting, so the result does not depend on thread timing.
#include "common.h"

namespace llmc {

constexpr int kSelThreads = 1024;

__global__ void refresh_kernel(const uint8_t* __restrict__ valid, const float* __restrict__ inv_norm, int N, int n_pad,
                               float* __restrict__ binv_eff) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < n_pad) binv_eff[j] = (j < N && valid[j]) ? inv_norm[j] : NAN;
}

__device__ __forceinline__ bool sel_key(const uint8_t* valid, const uint64_t* last_used, int j, int mode_evict,
                                        int allow_replace, uint64_t* key) {
  const bool v = valid[j] != 0;
  if (v) {
    if (!allow_replace) return false;
    *key = ((last_used[j] + 1ull) << 32) | (uint32_t)j;
    return true;
  }
  if (mode_evict) return false;
  *key = (uint64_t)(uint32_t)j;
  return true;
}

// mode_evict = 0: slots for insertion (free first, then LRU victims if allow_replace)
// mode_evict = 1: LRU victims among valid entries; they are invalidated here
__global__ __launch_bounds__(kSelThreads) void select_kernel(uint8_t* valid, const uint64_t* __restrict__ last_used,
                                                             int N, const int32_t* d_m, int m_max, int mode_evict,
                                                             int allow_replace, int32_t* __restrict__ slots_out,
                                                             float* binv_eff) {
  extern __shared__ uint64_t list[];      // [m_max]
  __shared__ unsigned hist[256];
  __shared__ unsigned s_total, s_count;
  __shared__ uint64_t s_prefix, s_mask;
  __shared__ unsigned s_remaining;
  const int tid = threadIdx.x;
  int m = d_m ? *d_m : m_max;
  m = max(0, min(m, m_max));
  if (tid == 0) { s_total = 0; s_count = 0; }
  __syncthreads();
  unsigned mine = 0;
  for (int j = tid; j < N; j += kSelThreads) {
    uint64_t key;
    if (sel_key(valid, last_used, j, mode_evict, allow_replace, &key)) ++mine;
  }
  if (mine) atomicAdd(&s_total, mine);
  __syncthreads();
  const int m_eff = min(m, (int)s_total);
  for (int i = m_eff + tid; i < m_max; i += kSelThreads) slots_out[i] = -1;
  if (m_eff == 0) return;
  if (tid == 0) { s_prefix = 0; s_mask = 0; s_remaining = (unsigned)m_eff; }
  for (int pass = 7; pass >= 0; --pass) {
    const int shift = pass * 8;
    for (int i = tid; i < 256; i += kSelThreads) hist[i] = 0;
    __syncthreads();
    const uint64_t prefix = s_prefix, mask = s_mask;
    for (int j = tid; j < N; j += kSelThreads) {
      uint64_t key;
      if (sel_key(valid, last_used, j, mode_evict, allow_replace, &key) && (key & mask) == prefix)
        atomicAdd(&hist[(unsigned)(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (tid == 0) {
      unsigned cum = 0, rem = s_remaining;
      int dsel = 255;
      for (int dgt = 0; dgt < 256; ++dgt) {
        if (cum + hist[dgt] >= rem) { dsel = dgt; break; }
        cum += hist[dgt];
      }
      s_remaining = rem - cum;
      s_prefix = prefix | ((uint64_t)dsel << shift);
      s_mask = mask | (0xFFull << shift);
    }
    __syncthreads();
  }
  const uint64_t kth = s_prefix;
  for (int j = tid; j < N; j += kSelThreads) {
    uint64_t key;
    if (sel_key(valid, last_used, j, mode_evict, allow_replace, &key) && key <= kth) {
      const unsigned p = atomicAdd(&s_count, 1u);
      if (p < (unsigned)m_max) list[p] = key;
    }
  }
  __syncthreads();
  const int n = min((int)s_count, m_eff);
  for (int i = tid; i < n; i += kSelThreads) {
    const uint64_t key = list[i];
    int rank = 0;
    for (int o = 0; o < n; ++o) rank += list[o] < key ? 1 : 0;
    const int slot = (int)(uint32_t)key;
    slots_out[rank] = slot;
    if (mode_evict) {
      valid[slot] = 0;
      binv_eff[slot] = NAN;
    }
  }
}

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
constexpr int kCopyThreads = 256;
constexpr int kCopyVecPerThread = 4;

// grid (chunks, m_max): entry i stores row r = rows[i] (or i) of fp / inv_norm / act into slots[i]
__global__ __launch_bounds__(kCopyThreads) void insert_kernel(
    const u32x4_t* __restrict__ fp_src, const float* __restrict__ inv_src, const u32x4_t* __restrict__ act_src,
    const int32_t* __restrict__ rows, const int32_t* d_m, int m_max, const int32_t* __restrict__ slots,
    u32x4_t* __restrict__ bank_fp, float* bank_inv, u32x4_t* __restrict__ bank_act, const int32_t* act_slot,
    uint64_t* last_used, uint32_t* hits, uint8_t* valid, float* binv_eff, size_t vec_per_key, size_t vec_per_seq,
    uint64_t tick, int32_t* counters) {
  int m = d_m ? *d_m : m_max;
  m = max(0, min(m, m_max));
  const int i = blockIdx.y;
  if (i >= m) return;
  const int slot = slots[i];
  const bool first = blockIdx.x == 0;
  if (slot < 0) {
    if (first && threadIdx.x == 0 && counters) atomicAdd(&counters[LLMC_CNT_DROPPED], 1);
    return;
  }
  const int r = rows ? rows[i] : i;
  const int vslot = act_slot ? act_slot[slot] : slot;
  const u32x4_t* src = act_src + (size_t)r * vec_per_seq;
  u32x4_t* dst = bank_act + (size_t)vslot * vec_per_seq;
  const size_t v0 = (size_t)blockIdx.x * (kCopyThreads * kCopyVecPerThread) + threadIdx.x;
  u32x4_t regs[kCopyVecPerThread];
#pragma unroll
  for (int u = 0; u < kCopyVecPerThread; ++u) {
    const size_t v = v0 + (size_t)u * kCopyThreads;
    if (v < vec_per_seq) regs[u] = src[v];
  }
#pragma unroll
  for (int u = 0; u < kCopyVecPerThread; ++u) {
    const size_t v = v0 + (size_t)u * kCopyThreads;
    if (v < vec_per_seq) __builtin_nontemporal_store(regs[u], dst + v);
  }
  if (first) {
    for (size_t v = threadIdx.x; v < vec_per_key; v += kCopyThreads)
      bank_fp[(size_t)slot * vec_per_key + v] = fp_src[(size_t)r * vec_per_key + v];
    if (threadIdx.x == 0) {
      const float inv = inv_src[r];
      const bool was = valid[slot] != 0;
      bank_inv[slot] = inv;
      binv_eff[slot] = inv;
      last_used[slot] = tick;
      hits[slot] = 0;
      valid[slot] = 1;
      if (counters) {
        atomicAdd(&counters[LLMC_CNT_INSERTED], 1);
        if (was) atomicAdd(&counters[LLMC_CNT_EVICTED], 1);
      }
    }
  }
}

llmc_status_t launch_bank_refresh(llmc_bank* bank, hipStream_t st) {
  const int N = bank->desc.n_slots;
  const int n_pad = (int)align_up((size_t)N, 256);
  { ProfScope ps_("refresh_kernel", st); hipLaunchKernelGGL(refresh_kernel, dim3((n_pad + 255) / 256), dim3(256), 0, st, bank->desc.d_valid,
                     bank->desc.d_inv_norm, N, n_pad, bank->d_binv_eff); }
  LLMC_LAUNCH_CHECK("refresh_kernel");
  return LLMC_OK;
}

llmc_status_t launch_bank_insert(llmc_bank* bank, const void* d_fp, const float* d_inv, const void* d_act,
                                 const int32_t* d_rows, const int32_t* d_m, int m_max, uint64_t tick,
                                 int32_t* d_slots_out, int32_t* d_counters, hipStream_t st) {
  const llmc_bank_desc_t& D = bank->desc;
  { ProfScope ps_("select_kernel", st); hipLaunchKernelGGL(select_kernel, dim3(1), dim3(kSelThreads), (size_t)m_max * sizeof(uint64_t), st, D.d_valid,
                     D.d_last_used, D.n_slots, d_m, m_max, 0, D.policy == LLMC_EVICT_LRU ? 1 : 0, d_slots_out,
                     bank->d_binv_eff); }
  LLMC_LAUNCH_CHECK("select_kernel");
  const size_t e = elem_size(D.dtype);
  const size_t vec_per_seq = (size_t)D.S * D.d * e / 16, vec_per_key = (size_t)D.k * e / 16;
  const size_t per_wg = (size_t)kCopyThreads * kCopyVecPerThread;
  dim3 grid((unsigned)((vec_per_seq + per_wg - 1) / per_wg), m_max);
  { ProfScope ps_("insert_kernel", st); hipLaunchKernelGGL(insert_kernel, grid, dim3(kCopyThreads), 0, st, (const u32x4_t*)d_fp, d_inv, (const u32x4_t*)d_act,
                     d_rows, d_m, m_max, d_slots_out, (u32x4_t*)D.d_fp, D.d_inv_norm, (u32x4_t*)D.d_act, D.d_act_slot,
                     D.d_last_used, D.d_hits, D.d_valid, bank->d_binv_eff, vec_per_key, vec_per_seq, tick, d_counters); }
  LLMC_LAUNCH_CHECK("insert_kernel");
  return LLMC_OK;
}

llmc_status_t launch_bank_evict(llmc_bank* bank, const int32_t* d_m, int m_max, int32_t* d_victims, hipStream_t st) {
  const llmc_bank_desc_t& D = bank->desc;
  { ProfScope ps_("select_kernel", st); hipLaunchKernelGGL(select_kernel, dim3(1), dim3(kSelThreads), (size_t)m_max * sizeof(uint64_t), st, D.d_valid,
                     D.d_last_used, D.n_slots, d_m, m_max, 1, 1, d_victims, bank->d_binv_eff); }
  LLMC_LAUNCH_CHECK("select_kernel");
  return LLMC_OK;
}

}  // namespace llmc
