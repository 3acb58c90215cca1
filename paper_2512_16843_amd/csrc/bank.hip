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
#include <algorithm>
#include "common.h"

namespace llmc {

constexpr int kSelThreads = 1024;

// The library's per-slot mirror: for real-valued keys the inverse norm of a valid slot and NaN for a free one;
// for sign-bit keys the start value of the popcount chain, 0 for a valid slot and kBitsFreePenalty for a free one.
constexpr uint32_t kBitsFreePenalty = 2048;

__global__ void refresh_kernel(const uint8_t* __restrict__ valid, const float* __restrict__ inv_norm, int N, int n_pad,
                               float* __restrict__ binv_eff, int key_bits) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n_pad) return;
  const bool v = j < N && valid[j];
  if (key_bits) reinterpret_cast<uint32_t*>(binv_eff)[j] = v ? 0u : kBitsFreePenalty;
  else binv_eff[j] = v ? inv_norm[j] : NAN;
}

// policy 2 (decayed hits): (min(hits, 65535) << 48) | ((last_used + 1) << 24) | slot, with n_slots <= 2^24 and
// last_used + 1 < 2^24; otherwise ((last_used + 1) << 32) | slot.  Free slots: their number alone.
__device__ __forceinline__ bool sel_key(const uint8_t* valid, const uint64_t* last_used, const uint32_t* hits, int j,
                                        int mode_evict, int allow_replace, int by_hits, uint64_t* key) {
  const bool v = valid[j] != 0;
  if (v) {
    if (!allow_replace) return false;
    if (by_hits)
      *key = ((uint64_t)min(hits[j], 65535u) << 48) | ((last_used[j] + 1ull) << 24) | (uint32_t)j;
    else
      *key = ((last_used[j] + 1ull) << 32) | (uint32_t)j;
    return true;
  }
  if (mode_evict) return false;
  *key = (uint64_t)(uint32_t)j;
  return true;
}

// basis [r, d] -> transposed copy [d, r] (element size e bytes, 2 or 4)
__global__ void transpose_kernel(const uint8_t* __restrict__ in, uint8_t* __restrict__ out, int r, int d, int e) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= r * d) return;
  const int a = i / d, b = i % d;
  for (int x = 0; x < e; ++x) out[((size_t)b * r + a) * e + x] = in[(size_t)i * e + x];
}

llmc_status_t launch_transpose(const void* in, void* out, int r, int d, int e, hipStream_t st) {
  LLMC_KERNEL_GGL(transpose_kernel, dim3((r * d + 255) / 256), dim3(256), 0, st, (const uint8_t*)in, (uint8_t*)out, r, d, e);
  LLMC_LAUNCH_CHECK("transpose_kernel");
  return LLMC_OK;
}

// hits[j] >>= shift for every slot (free slots too: their counts are reset on insertion)
__global__ void decay_kernel(uint32_t* __restrict__ hits, int N, int shift) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < N) hits[j] >>= shift;
}

// mode_evict = 0: slots for insertion (free first, then LRU victims if allow_replace)
// mode_evict = 1: LRU victims among valid entries; they are invalidated here
// KPT > 0: every thread keeps its KPT candidate keys in registers (N <= KPT * 1024), so the bank's
// metadata is read once; KPT == 0: keys are re-read from memory in every pass (any N).
//
// Radix select over the bits that actually differ between candidate keys (ticks and slot numbers are
// small integers, so most of the 64 bits are the same in every key): OR and AND of all keys give the
// varying bits; digits of up to 11 bits are cut from the highest varying bit downwards.  A wavefront
// whose lanes all hold the same digit (many entries of one tick) adds its count with one atomic.
constexpr int kSelDigitBits = 11, kSelBins = 1 << kSelDigitBits;

template <int KPT>
__global__ __launch_bounds__(kSelThreads) void select_kernel(uint8_t* valid, const uint64_t* __restrict__ last_used,
                                                             const uint32_t* __restrict__ hits, int by_hits,
                                                             int N, const int32_t* d_m, int m_max, int mode_evict,
                                                             int allow_replace, int32_t* __restrict__ slots_out,
                                                             float* binv_eff, uint32_t free_mark) {
  extern __shared__ uint64_t list[];      // [m_max]
  __shared__ unsigned hist[kSelBins];
  __shared__ unsigned wave_tot[kSelThreads / 64];
  __shared__ unsigned s_total, s_count, s_or_lo, s_or_hi, s_and_lo, s_and_hi;
  __shared__ uint64_t s_prefix;
  __shared__ unsigned s_remaining;
  constexpr uint64_t kAbsent = ~0ull;     // larger than every candidate key
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int m = d_m ? *d_m : m_max;
  m = max(0, min(m, m_max));
  if (m == 0) {                           // nothing to place: the bank's metadata is not even read
    for (int i = tid; i < m_max; i += kSelThreads) slots_out[i] = -1;
    return;
  }
  if (tid == 0) { s_total = 0; s_count = 0; s_or_lo = 0; s_or_hi = 0; s_and_lo = ~0u; s_and_hi = ~0u; }
  __syncthreads();
  const int n_iter = KPT > 0 ? KPT : (N + kSelThreads - 1) / kSelThreads;
  uint64_t cached[KPT > 0 ? KPT : 1];
  auto key_at = [&](int u) -> uint64_t {
    if (KPT > 0) return cached[u];
    const int j = tid + u * kSelThreads;
    uint64_t key;
    return (j < N && sel_key(valid, last_used, hits, j, mode_evict, allow_replace, by_hits, &key)) ? key : kAbsent;
  };
  if (KPT > 0) {
#pragma unroll
    for (int u = 0; u < (KPT > 0 ? KPT : 1); ++u) {
      const int j = tid + u * kSelThreads;
      uint64_t key;
      cached[u] = (j < N && sel_key(valid, last_used, hits, j, mode_evict, allow_replace, by_hits, &key)) ? key : kAbsent;
    }
  }
  unsigned mine = 0;
  uint64_t or_k = 0, and_k = ~0ull;
  for (int u = 0; u < n_iter; ++u) {
    const uint64_t key = key_at(u);
    if (key != kAbsent) { ++mine; or_k |= key; and_k &= key; }
  }
  // wavefront reduction first: one set of atomics per wavefront
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    mine += __shfl_xor(mine, o, 64);
    or_k |= ((uint64_t)__shfl_xor((unsigned)(or_k >> 32), o, 64) << 32) | __shfl_xor((unsigned)or_k, o, 64);
    and_k &= ((uint64_t)__shfl_xor((unsigned)(and_k >> 32), o, 64) << 32) | __shfl_xor((unsigned)and_k, o, 64);
  }
  if (lane == 0 && mine) {
    atomicAdd(&s_total, mine);
    atomicOr(&s_or_lo, (unsigned)or_k); atomicOr(&s_or_hi, (unsigned)(or_k >> 32));
    atomicAnd(&s_and_lo, (unsigned)and_k); atomicAnd(&s_and_hi, (unsigned)(and_k >> 32));
  }
  __syncthreads();
  const int m_eff = min(m, (int)s_total);
  for (int i = m_eff + tid; i < m_max; i += kSelThreads) slots_out[i] = -1;
  if (m_eff == 0) return;
  const uint64_t or_all = ((uint64_t)s_or_hi << 32) | s_or_lo, and_all = ((uint64_t)s_and_hi << 32) | s_and_lo;
  uint64_t varying = or_all ^ and_all;   // bits on which candidate keys differ
  uint64_t mask = 0;                     // bits decided so far
  if (tid == 0) { s_prefix = 0; s_remaining = (unsigned)m_eff; }
  __syncthreads();
  while (varying) {
    const int hi = 63 - __clzll((long long)varying);
    const int lo = max(0, hi - kSelDigitBits + 1);
    const uint64_t field = ((hi - lo + 1 >= 64) ? ~0ull : ((1ull << (hi - lo + 1)) - 1ull)) << lo;
    for (int i = tid; i < kSelBins; i += kSelThreads) hist[i] = 0;
    __syncthreads();
    const uint64_t prefix = s_prefix;
    for (int u = 0; u < n_iter; ++u) {
      const uint64_t key = key_at(u);
      const bool in = key != kAbsent && (key & mask) == prefix;
      const unsigned dgt = (unsigned)((key & field) >> lo);
      // one atomic for a wavefront whose participating lanes all hold the same digit
      const unsigned long long act = __ballot(in);
      if (act) {
        const int leader = __ffsll((long long)act) - 1;
        const unsigned d0 = (unsigned)__builtin_amdgcn_readlane((int)dgt, leader);
        const unsigned long long same = __ballot(in && dgt == d0);
        if (same == act) {
          if (lane == leader) atomicAdd(&hist[d0], (unsigned)__popcll(act));
        } else if (in) {
          atomicAdd(&hist[dgt], 1u);
        }
      }
    }
    __syncthreads();
    {
      // digit whose cumulative count first reaches the remaining rank: 2 bins per thread, scan over the workgroup
      const unsigned h0 = hist[2 * tid], h1 = hist[2 * tid + 1];
      const unsigned own = h0 + h1;
      unsigned incl = own;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const unsigned v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
      }
      if (lane == 63) wave_tot[wave] = incl;
      __syncthreads();
      unsigned base = 0;
      for (int w = 0; w < wave; ++w) base += wave_tot[w];
      incl += base;
      const unsigned rem = s_remaining, before = incl - own;
      __syncthreads();                                       // everyone has read s_remaining
      if (before < rem && incl >= rem) {                     // exactly one thread: counts are cumulative
        const bool first = before + h0 >= rem;
        s_remaining = rem - (first ? before : before + h0);
        s_prefix = prefix | ((uint64_t)(2 * tid + (first ? 0 : 1)) << lo);
      }
    }
    mask |= field;
    varying &= ~field;
    __syncthreads();
  }
  // bits never examined are the same in every candidate key
  const uint64_t kth = s_prefix | (and_all & ~mask);
  for (int u = 0; u < n_iter; ++u) {
    const uint64_t key = key_at(u);
    if (key != kAbsent && key <= kth) {
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
    const int slot = by_hits ? (int)(key & 0xFFFFFFull) : (int)(uint32_t)key;
    slots_out[rank] = slot;
    if (mode_evict) {
      valid[slot] = 0;
      reinterpret_cast<uint32_t*>(binv_eff)[slot] = free_mark;     // NaN, or the popcount penalty of a free slot
    }
  }
}

static void launch_select(const llmc_bank* bank, const int32_t* d_m, int m_max, int mode_evict, int allow_replace,
                          int32_t* slots_out, hipStream_t st) {
  const llmc_bank_desc_t& D = bank->desc;
  const int N = D.n_slots, by_hits = D.policy == LLMC_EVICT_DECAYED_HITS ? 1 : 0;
  const size_t lds = (size_t)m_max * sizeof(uint64_t);
#define LLMC_SELECT(KPT_) LLMC_KERNEL_GGL(select_kernel<KPT_>, dim3(1), dim3(kSelThreads), lds, st, D.d_valid,         \
                                             D.d_last_used, D.d_hits, by_hits, N, d_m, m_max, mode_evict, allow_replace, \
                                             slots_out, bank->d_binv_eff, D.key_bits ? kBitsFreePenalty : 0x7FC00000u)
  if (N <= 4 * kSelThreads) LLMC_SELECT(4);
  else if (N <= 16 * kSelThreads) LLMC_SELECT(16);
  else if (N <= 48 * kSelThreads) LLMC_SELECT(48);
  else LLMC_SELECT(0);
#undef LLMC_SELECT
}

llmc_status_t launch_bank_advance(llmc_bank* bank, uint64_t tick, hipStream_t st) {
  const llmc_bank_desc_t& D = bank->desc;
  if (D.policy != LLMC_EVICT_DECAYED_HITS || D.half_life <= 0) return LLMC_OK;
  const int64_t e = (int64_t)(tick / (uint64_t)D.half_life);
  if (e <= bank->epoch) return LLMC_OK;
  const int shift = (int)std::min<int64_t>(31, e - bank->epoch);
  bank->epoch = e;
  { ProfScope ps_("decay_kernel", st);
    LLMC_KERNEL_GGL(decay_kernel, dim3((D.n_slots + 255) / 256), dim3(256), 0, st, D.d_hits, D.n_slots, shift); }
  LLMC_LAUNCH_CHECK("decay_kernel");
  return LLMC_OK;
}

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
constexpr int kCopyThreads = 1024;          // the gather's launch shape, see gate.hip
constexpr int kCopyVecPerThread = 6;

// grid (chunks, m_max): entry i stores row r = rows[i] (or i) of fp / inv_norm / act into slots[i]
__global__ __launch_bounds__(kCopyThreads) void insert_kernel(
    const u32x4_t* __restrict__ fp_src, const float* __restrict__ inv_src, const u32x4_t* __restrict__ act_src,
    const int32_t* __restrict__ rows, const int32_t* d_m, int m_max, const int32_t* __restrict__ slots,
    u32x4_t* __restrict__ bank_fp, float* bank_inv, u32x4_t* __restrict__ bank_act, const int32_t* act_slot,
    uint64_t* last_used, uint32_t* hits, uint8_t* valid, float* binv_eff, size_t words_per_key, size_t vec_per_seq,
    uint64_t tick, int32_t* counters, int key_bits) {
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
    const uint32_t* ksrc = reinterpret_cast<const uint32_t*>(fp_src) + (size_t)r * words_per_key;
    uint32_t* kdst = reinterpret_cast<uint32_t*>(bank_fp) + (size_t)slot * words_per_key;
    for (size_t v = threadIdx.x; v < words_per_key; v += kCopyThreads) kdst[v] = ksrc[v];
    if (threadIdx.x == 0) {
      const bool was = valid[slot] != 0;
      if (key_bits) {
        reinterpret_cast<uint32_t*>(binv_eff)[slot] = 0u;
      } else {
        const float inv = inv_src[r];
        bank_inv[slot] = inv;
        binv_eff[slot] = inv;
      }
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

// the bucket index of a bank of sign-bit keys follows every change of keys or validity; `changed` (device, optional)
// lets the kernels leave at once when a batch changed nothing
static llmc_status_t rebuild_lsh_index(const llmc_bank* bank, hipStream_t st, const int32_t* changed) {
  const llmc_bank_desc_t& D = bank->desc;
  if (!D.key_bits || !D.d_lsh_index) return LLMC_OK;
  return launch_lsh_build((const uint32_t*)D.d_fp, D.d_valid, D.n_slots, D.k, D.d_lsh_index, st, changed);
}

llmc_status_t launch_bank_refresh(llmc_bank* bank, hipStream_t st) {
  const int N = bank->desc.n_slots;
  const int n_pad = (int)align_up((size_t)N + 8, 256);      // the mirror's allocated length
  { ProfScope ps_("refresh_kernel", st); LLMC_KERNEL_GGL(refresh_kernel, dim3((n_pad + 255) / 256), dim3(256), 0, st, bank->desc.d_valid,
                     bank->desc.d_inv_norm, N, n_pad, bank->d_binv_eff, bank->desc.key_bits); }
  LLMC_LAUNCH_CHECK("refresh_kernel");
  return rebuild_lsh_index(bank, st, nullptr);
}

llmc_status_t launch_bank_insert(llmc_bank* bank, const void* d_fp, const float* d_inv, const void* d_act,
                                 const int32_t* d_rows, const int32_t* d_m, int m_max, uint64_t tick,
                                 int32_t* d_slots_out, int32_t* d_counters, hipStream_t st) {
  const llmc_bank_desc_t& D = bank->desc;
  LLMC_TRY(launch_bank_advance(bank, tick, st));
  { ProfScope ps_("select_kernel", st);
    launch_select(bank, d_m, m_max, 0, D.policy != LLMC_EVICT_NONE ? 1 : 0, d_slots_out, st); }
  LLMC_LAUNCH_CHECK("select_kernel");
  const size_t e = elem_size(D.dtype);
  if (D.rank > 0) {
    // compressed values: C = h U^T straight into the slots' value rows (every listed row has a slot: the policy
    // replaces, and the call places at most n_slots rows)
    LLMC_TRY(launch_linear(d_act, D.d, d_rows, D.d_basis, nullptr, D.rank, D.d, D.d_act, D.rank, d_slots_out, D.S, d_m,
                           m_max, D.dtype, st));
  }
  const size_t vec_per_seq = D.rank > 0 ? 0 : (size_t)D.S * D.d * e / 16;
  const size_t words_per_key = D.key_bits ? (size_t)D.k / 32 : (size_t)D.k * e / 4;
  const size_t per_wg = (size_t)kCopyThreads * kCopyVecPerThread;
  dim3 grid((unsigned)std::max<size_t>(1, (vec_per_seq + per_wg - 1) / per_wg), m_max);
  { ProfScope ps_("insert_kernel", st); LLMC_KERNEL_GGL(insert_kernel, grid, dim3(kCopyThreads), 0, st, (const u32x4_t*)d_fp, d_inv, (const u32x4_t*)d_act,
                     d_rows, d_m, m_max, d_slots_out, (u32x4_t*)D.d_fp, D.d_inv_norm, (u32x4_t*)D.d_act, D.d_act_slot,
                     D.d_last_used, D.d_hits, D.d_valid, bank->d_binv_eff, words_per_key, vec_per_seq, tick, d_counters,
                     D.key_bits); }
  LLMC_LAUNCH_CHECK("insert_kernel");
  // the token mean of every stored output, kept beside it (dropped rows have slot -1 and are skipped)
  if (D.d_act_pool)
    LLMC_TRY(launch_pool_rows(d_act, m_max, D.S, D.d, D.dtype, d_rows, d_m, d_slots_out, D.d_act_pool, st));
  // ... and the key under which the next layer will look it up
  if (D.d_next_fp)
    LLMC_TRY(launch_project_rows(D.d_act_pool, m_max, D.d, D.dtype, D.d_next_proj, D.d_next_bias, D.next_k, d_slots_out,
                                 d_m, D.d_next_fp, D.d_next_inv, st));
  return rebuild_lsh_index(bank, st, d_m);
}

llmc_status_t launch_bank_evict(llmc_bank* bank, const int32_t* d_m, int m_max, int32_t* d_victims, hipStream_t st) {
  { ProfScope ps_("select_kernel", st);
    launch_select(bank, d_m, m_max, 1, 1, d_victims, st); }
  LLMC_LAUNCH_CHECK("select_kernel");
  return rebuild_lsh_index(bank, st, d_m);
}

}  // namespace llmc
