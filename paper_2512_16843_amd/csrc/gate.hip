// The decision gate (Section III-D of the paper): turn the per-row hit flags into
// compacted, ascending lists of hit rows and miss rows with device-side counts, record
// hits in the bank (Section IV-D: recency), and copy the cached outputs of the hit rows
// (Algorithm 1: h_l <- h').
#include "common.h"
#include "compact.h"

namespace llmc {

// the stand-alone compaction: one workgroup of 1024 threads
__global__ __launch_bounds__(1024) void compact_kernel(const uint8_t* __restrict__ hit, const int32_t* __restrict__ idx,
                                                       const float* __restrict__ sim, const uint8_t* __restrict__ tie,
                                                       int B, float tau, int32_t* __restrict__ hit_rows,
                                                       int32_t* __restrict__ miss_rows, int32_t* __restrict__ counters,
                                                       uint64_t* last_used, uint32_t* hits, int touch, uint64_t tick,
                                                       int reval_every, int32_t* __restrict__ reval_tmp,
                                                       uint8_t* __restrict__ pooled_valid_out, int has_pool,
                                                       int32_t* __restrict__ ref_out,
                                                       const int32_t* __restrict__ act_slot) {
  compact_rows(hit, idx, sim, tie, B, tau, hit_rows, miss_rows, counters, last_used, hits, touch, tick, reval_every,
               reval_tmp, pooled_valid_out, has_pool, ref_out, act_slot);
}

// Divergence monitor, second half: workgroup i takes the i-th recomputed hit row.  It compares the fresh output
// (already in h_out) with the cached value, max|fresh - cached| / max|cached|, and replaces the cached value when
// the ratio exceeds the bound -- unless a lower recomputed row of this batch matched the same entry, which then
// decides alone.  grid (B).
template <typename T>
__global__ __launch_bounds__(1024) void divergence_kernel(const T* __restrict__ h_out, T* __restrict__ act,
                                                          const int32_t* __restrict__ act_slot,
                                                          const int32_t* __restrict__ idx,
                                                          const int32_t* __restrict__ rows, int32_t* counters,
                                                          size_t elems_per_seq, float bound) {
  constexpr int VEC = Vec16<T>::N;
  __shared__ float red_d[16], red_c[16];
  __shared__ int s_owner;
  const int n_miss = counters[LLMC_CNT_MISS], n_reval = counters[LLMC_CNT_REVALIDATED];
  const int i = blockIdx.x;
  if (i >= n_reval) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = rows[n_miss + i];
  const int slot = idx[row];
  if (tid == 0) s_owner = 1;
  __syncthreads();
  for (int o = tid; o < i; o += 1024)
    if (idx[rows[n_miss + o]] == slot) s_owner = 0;
  __syncthreads();
  if (!s_owner) return;
  const int vslot = act_slot ? act_slot[slot] : slot;
  const T* fresh = h_out + (size_t)row * elems_per_seq;
  T* cached = act + (size_t)vslot * elems_per_seq;
  float md = 0.f, mc = 0.f;
  for (size_t e = (size_t)tid * VEC; e < elems_per_seq; e += (size_t)1024 * VEC) {
    float f[VEC], c[VEC];
    Vec16<T>::load(fresh + e, f);
    Vec16<T>::load(cached + e, c);
#pragma unroll
    for (int u = 0; u < VEC; ++u) {
      md = fmaxf(md, fabsf(f[u] - c[u]));
      mc = fmaxf(mc, fabsf(c[u]));
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    md = fmaxf(md, __shfl_xor(md, o, 64));
    mc = fmaxf(mc, __shfl_xor(mc, o, 64));
  }
  if (lane == 0) { red_d[wave] = md; red_c[wave] = mc; }
  __syncthreads();
  md = 0.f; mc = 0.f;
  for (int w = 0; w < 16; ++w) { md = fmaxf(md, red_d[w]); mc = fmaxf(mc, red_c[w]); }
  const float div = md / fmaxf(mc, 1e-30f);
  if (!(div > bound)) return;
  for (size_t e = (size_t)tid * VEC; e < elems_per_seq; e += (size_t)1024 * VEC) {
    float f[VEC];
    Vec16<T>::load(fresh + e, f);
    Vec16<T>::store(cached + e, f);
  }
  if (tid == 0) atomicAdd(&counters[LLMC_CNT_DIVERGED], 1);
}

// uncached layer: every row is a miss
__global__ void all_miss_kernel(int B, int32_t* miss_rows, int32_t* counters, int32_t* idx, float* sim, uint8_t* hit,
                                uint8_t* pooled_valid_out) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) {
    miss_rows[b] = b;
    if (pooled_valid_out) pooled_valid_out[b] = 0;
    if (idx) idx[b] = -1;
    if (sim) sim[b] = -INFINITY;
    if (hit) hit[b] = 0;
  }
  if (b < LLMC_CNT_WORDS) counters[b] = (b == LLMC_CNT_MISS || b == LLMC_CNT_COMPUTED) ? B : 0;
}

// Copy of cached outputs: grid (chunks, n_max); every thread moves 16-byte vectors.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
// 1024 threads x 6 vectors = 96 KiB per workgroup: of the launch shapes swept at 2,048 and 4,096 rows of 576 KiB this
// one streamed fastest (74 % of the HBM peak against 70-72 % for 256 threads x 4 vectors)
constexpr int kGatherThreads = 1024;
constexpr int kGatherVecPerThread = 6;

__device__ __forceinline__ void gather_body(const u32x4_t* __restrict__ act, const int32_t* act_slot,
                                                                const int32_t* __restrict__ idx,
                                                                const int32_t* __restrict__ rows,
                                                                const int32_t* __restrict__ count, int n_max,
                                                                size_t vec_per_seq, u32x4_t* __restrict__ out,
                                                                const float* __restrict__ act_pool,
                                                                float* __restrict__ pooled_out, int d,
                                                                const uint32_t* __restrict__ next_fp,
                                                                const float* __restrict__ next_inv,
                                                                uint32_t* __restrict__ key_out,
                                                                float* __restrict__ key_inv_out, int key_words) {
  const int n = count ? min(*count, n_max) : n_max;
  const int i = blockIdx.y;
  if (i >= n) return;
  const int b = rows ? rows[i] : i;
  const int j = idx[b];
  if (j < 0) return;
  const int slot = act_slot ? act_slot[j] : j;
  if (pooled_out && blockIdx.x == 0)       // the stored token mean of the cached output rides along
    for (int c = threadIdx.x; c < d; c += kGatherThreads) pooled_out[(size_t)b * d + c] = act_pool[(size_t)slot * d + c];
  if (key_out && blockIdx.x == 0) {        // ... and so does the key under which the next layer looks it up
    for (int c = threadIdx.x; c < key_words; c += kGatherThreads)
      key_out[(size_t)b * key_words + c] = next_fp[(size_t)slot * key_words + c];
    if (threadIdx.x == 0) key_inv_out[b] = next_inv[slot];
  }
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
                             int B, float tau, int32_t* d_hit_rows, int32_t* d_miss_rows, int32_t* d_reval_tmp,
                             int32_t* d_counters, llmc_bank* bank, uint32_t flags, uint64_t tick, hipStream_t st,
                             uint8_t* d_pooled_valid_out, int has_pool, int32_t* d_ref_out) {
  const int touch = (flags & LLMC_UPDATE_LRU) ? 1 : 0;
  const int reval_every = (flags & LLMC_REVALIDATE) ? bank->desc.reval_every : 0;
  { ProfScope ps_("compact_kernel", st); LLMC_KERNEL_GGL(compact_kernel, dim3(1), dim3(1024), 0, st, d_hit, d_idx, d_sim, d_near_tie, B, tau, d_hit_rows,
                     d_miss_rows, d_counters, bank->desc.d_last_used, bank->desc.d_hits, touch, tick, reval_every,
                     d_reval_tmp, d_pooled_valid_out, has_pool, d_ref_out, bank->desc.d_act_slot); }
  LLMC_LAUNCH_CHECK("compact_kernel");
  return LLMC_OK;
}

llmc_status_t launch_divergence(llmc_bank* bank, const void* d_h_out, const int32_t* d_idx, const int32_t* d_rows,
                                int32_t* d_counters, int B, hipStream_t st) {
  const llmc_bank_desc_t& D = bank->desc;
  const size_t elems = (size_t)D.S * D.d;
  ProfScope ps_("divergence_kernel", st);
  if (D.dtype == LLMC_F32)
    LLMC_KERNEL_GGL(divergence_kernel<float>, dim3(B), dim3(1024), 0, st, (const float*)d_h_out, (float*)D.d_act,
                       D.d_act_slot, d_idx, d_rows, d_counters, elems, D.drift_bound);
  else
    LLMC_KERNEL_GGL(divergence_kernel<bf16_t>, dim3(B), dim3(1024), 0, st, (const bf16_t*)d_h_out, (bf16_t*)D.d_act,
                       D.d_act_slot, d_idx, d_rows, d_counters, elems, D.drift_bound);
  LLMC_LAUNCH_CHECK("divergence_kernel");
  return LLMC_OK;
}

llmc_status_t launch_all_miss(int B, int32_t* d_miss_rows, int32_t* d_counters, int32_t* d_idx, float* d_sim,
                              uint8_t* d_hit, hipStream_t st, uint8_t* d_pooled_valid_out) {
  const int n = B > LLMC_CNT_WORDS ? B : LLMC_CNT_WORDS;
  { ProfScope ps_("all_miss_kernel", st); LLMC_KERNEL_GGL(all_miss_kernel, dim3((n + 255) / 256), dim3(256), 0, st, B, d_miss_rows, d_counters, d_idx, d_sim,
                     d_hit, d_pooled_valid_out); }
  LLMC_LAUNCH_CHECK("all_miss_kernel");
  return LLMC_OK;
}

#define LLMC_GATHER_PARAMS                                                                                         \
  const u32x4_t *__restrict__ act, const int32_t *act_slot, const int32_t *__restrict__ idx,                       \
      const int32_t *__restrict__ rows, const int32_t *__restrict__ count, int n_max, size_t vec_per_seq,           \
      u32x4_t *__restrict__ out, const float *__restrict__ act_pool, float *__restrict__ pooled_out, int d,         \
      const uint32_t *__restrict__ next_fp, const float *__restrict__ next_inv, uint32_t *__restrict__ key_out,     \
      float *__restrict__ key_inv_out, int key_words
#define LLMC_GATHER_ARGS                                                                                             \
  act, act_slot, idx, rows, count, n_max, vec_per_seq, out, act_pool, pooled_out, d, next_fp, next_inv, key_out,   \
      key_inv_out, key_words
// the reuse step of a call: copies of cached outputs for the rows answered from the bank
__global__ __launch_bounds__(kGatherThreads) void gather_kernel(LLMC_GATHER_PARAMS) { gather_body(LLMC_GATHER_ARGS); }
// the same copy for rows that arrived as references (deferred copies): a separate name, so that traces tell the
// usually empty just-in-time copies from the reuse step
__global__ __launch_bounds__(kGatherThreads) void materialize_kernel(LLMC_GATHER_PARAMS) { gather_body(LLMC_GATHER_ARGS); }

// value row of the i-th listed hit: act_slot[idx[rows[i]]]
__global__ void hit_slots_kernel(const int32_t* __restrict__ idx, const int32_t* __restrict__ rows,
                                 const int32_t* __restrict__ act_slot, const int32_t* count, int n_max,
                                 int32_t* __restrict__ out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  const int n = count ? min(*count, n_max) : n_max;
  if (i >= n) return;
  const int j = max(idx[rows ? rows[i] : i], 0);
  out[i] = act_slot ? act_slot[j] : j;
}

llmc_status_t launch_gather(const llmc_bank* bank, const int32_t* d_idx, const int32_t* d_rows, const int32_t* d_n,
                            int n_max, void* d_h_out, hipStream_t st, float* d_pooled_out, void* d_key_out,
                            float* d_key_inv_out) {
  const llmc_bank_desc_t& D = bank->desc;
  if (D.rank > 0) {
    // compressed values: h_out[rows[i]] = C[value row] * U, one GEMM with K = rank over the listed hits
    { ProfScope ps_("hit_slots_kernel", st);
      LLMC_KERNEL_GGL(hit_slots_kernel, dim3((n_max + 255) / 256), dim3(256), 0, st, d_idx, d_rows, D.d_act_slot, d_n,
                         n_max, bank->d_hit_slots); }
    LLMC_LAUNCH_CHECK("hit_slots_kernel");
    return launch_linear(D.d_act, D.rank, bank->d_hit_slots, bank->d_basis_t, nullptr, D.d, D.rank, d_h_out, D.d, d_rows,
                         D.S, d_n, n_max, D.dtype, st);
  }
  const size_t vec_per_seq = (size_t)D.S * D.d * elem_size(D.dtype) / 16;
  const size_t per_wg = (size_t)kGatherThreads * kGatherVecPerThread;
  dim3 grid((unsigned)((vec_per_seq + per_wg - 1) / per_wg), n_max);
  { ProfScope ps_("gather_kernel", st); LLMC_KERNEL_GGL(gather_kernel, grid, dim3(kGatherThreads), 0, st, (const u32x4_t*)D.d_act, D.d_act_slot, d_idx,
                     d_rows, d_n, n_max, vec_per_seq, (u32x4_t*)d_h_out, D.d_act_pool,
                     D.d_act_pool ? d_pooled_out : nullptr, D.d, (const uint32_t*)D.d_next_fp, D.d_next_inv,
                     (D.d_next_fp && d_key_inv_out) ? (uint32_t*)d_key_out : nullptr, d_key_inv_out,
                     (int)((size_t)D.next_k * elem_size(D.dtype) / 4)); }
  LLMC_LAUNCH_CHECK("gather_kernel");
  return LLMC_OK;
}

// ---- within-batch reuse (Algorithm 1 applied to the rows of a batch one after the other) ----------------------
// The rows that missed the bank are listed in ascending order in miss_rows[0 .. m).  Three steps:
//   pairs:   S[i][j] = cosine of the stored keys of listed rows i and j (j < i), fp64, one thread per pair;
//   resolve: one wavefront walks i = 0 .. m - 1: row i FOLLOWS the most similar earlier LEADER with S > tau (the
//            earliest among equals), else it is a leader itself; the list of rows to compute is rewritten in place to
//            the leaders, and the counters follow (MISS = COMPUTED = leaders, HIT += followers, DEDUP = followers);
//   finish:  after the dense block and the insertion, every follower copies its leader's output row and is reported
//            as a hit on the slot the leader was stored in.
// Scratch layout (dedup_ws_bytes): S [B * B] fp64 | src_row [B] | fol_rows [B] | fol_rank [B] | fol_sim [B] | n_fol.
struct DedupWs {
  double* S;
  int32_t *src_row, *fol_rows, *fol_rank;
  float* fol_sim;
  int32_t* n_fol;
};
static DedupWs dedup_ws(void* ws, int B) {
  char* p = (char*)ws;
  DedupWs w;
  w.S = (double*)p;         p += align_up((size_t)B * B * sizeof(double), 256);
  w.src_row = (int32_t*)p;  p += align_up((size_t)B * 4, 256);
  w.fol_rows = (int32_t*)p; p += align_up((size_t)B * 4, 256);
  w.fol_rank = (int32_t*)p; p += align_up((size_t)B * 4, 256);
  w.fol_sim = (float*)p;    p += align_up((size_t)B * 4, 256);
  w.n_fol = (int32_t*)p;
  return w;
}
size_t dedup_ws_bytes(int B) {
  if (B > LLMC_MAX_DEDUP_ROWS) return 0;
  return align_up((size_t)B * B * sizeof(double), 256) + 4 * align_up((size_t)B * 4, 256) + 256;
}

// grid (ceil(m_max / 256), m_max): block y is listed row i, thread x is listed row j < i
template <typename T>
__global__ __launch_bounds__(256) void dedup_pairs_kernel(const T* __restrict__ keys, const float* __restrict__ inv,
                                                          int k, const int32_t* __restrict__ rows,
                                                          const int32_t* __restrict__ counters, int m_max,
                                                          double* __restrict__ S) {
  constexpr int VEC = Vec16<T>::N;
  const int m = min(counters[LLMC_CNT_MISS], m_max);
  const int i = blockIdx.y, j = blockIdx.x * 256 + threadIdx.x;
  if (i >= m || j >= i) return;
  const int bi = rows[i], bj = rows[j];
  const T* a = keys + (size_t)bi * k;
  const T* b = keys + (size_t)bj * k;
  double acc = 0.0;
  for (int e = 0; e < k; e += VEC) {
    float x[VEC], y[VEC];
    Vec16<T>::load(a + e, x);
    Vec16<T>::load(b + e, y);
#pragma unroll
    for (int u = 0; u < VEC; ++u) acc += (double)x[u] * (double)y[u];
  }
  S[(size_t)i * m_max + j] = acc * (double)inv[bi] * (double)inv[bj];
}

// one wavefront; see above
__global__ __launch_bounds__(64) void dedup_resolve_kernel(const double* __restrict__ S, int m_max, float tau,
                                                           int32_t* miss_rows, int32_t* counters,
                                                           int32_t* __restrict__ src_row, int32_t* __restrict__ fol_rows,
                                                           int32_t* __restrict__ fol_rank, float* __restrict__ fol_sim,
                                                           int32_t* __restrict__ n_fol_out) {
  __shared__ int16_t lead_pos[LLMC_MAX_DEDUP_ROWS];     // position among the leaders, -1 for a follower
  const int lane = threadIdx.x;
  const int m = min(counters[LLMC_CNT_MISS], m_max);
  int n_lead = 0, n_fol = 0;
  for (int i = 0; i < m; ++i) {
    double best = -INFINITY;
    int best_j = -1;
    for (int j = lane; j < i; j += 64) {
      const double s = S[(size_t)i * m_max + j];
      if (lead_pos[j] >= 0 && s > (double)tau && (s > best)) { best = s; best_j = j; }     // ascending j: earliest among equals
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const double os = __shfl_xor(best, o, 64);
      const int oj = __shfl_xor(best_j, o, 64);
      if (oj >= 0 && (best_j < 0 || os > best || (os == best && oj < best_j))) { best = os; best_j = oj; }
    }
    const int row = miss_rows[i];                       // read before the slot may be overwritten below
    if (best_j < 0) {
      if (lane == 0) { lead_pos[i] = (int16_t)n_lead; miss_rows[n_lead] = row; }      // n_lead <= i: in place
      ++n_lead;
    } else {
      if (lane == 0) {
        lead_pos[i] = -1;
        fol_rows[n_fol] = row;
        fol_rank[n_fol] = lead_pos[best_j];
        fol_sim[n_fol] = (float)best;
        src_row[row] = miss_rows[lead_pos[best_j]];     // leaders already sit at their final positions
      }
      ++n_fol;
    }
    __builtin_amdgcn_s_waitcnt(0);                      // this wavefront's LDS and memory writes land before the next row reads them
    __builtin_amdgcn_wave_barrier();
  }
  if (lane == 0) {
    *n_fol_out = n_fol;
    counters[LLMC_CNT_MISS] = n_lead;
    counters[LLMC_CNT_COMPUTED] = n_lead;
    counters[LLMC_CNT_HIT] += n_fol;
    counters[LLMC_CNT_DEDUP] = n_fol;
  }
}

// grid (chunks, B): entry i < n_fol copies the output row of follower i's leader and records the hit
__global__ __launch_bounds__(kGatherThreads) void dedup_finish_kernel(
    u32x4_t* __restrict__ h_out, size_t vec_per_seq, const int32_t* __restrict__ n_fol, int n_max,
    const int32_t* __restrict__ src_row, const int32_t* __restrict__ fol_rows, const int32_t* __restrict__ fol_rank,
    const float* __restrict__ fol_sim, const int32_t* __restrict__ slots, int32_t* __restrict__ idx,
    float* __restrict__ sim, uint8_t* __restrict__ hit, uint32_t* hits, int touch) {
  const int n = min(*n_fol, n_max);
  const int i = blockIdx.y;
  if (i >= n) return;
  const int b = fol_rows[i];
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    const int slot = slots[fol_rank[i]];
    idx[b] = slot;
    if (sim) sim[b] = fol_sim[i];
    if (hit) hit[b] = 1;
    if (touch && slot >= 0) atomicAdd(&hits[slot], 1u);
  }
  const u32x4_t* src = h_out + (size_t)src_row[b] * vec_per_seq;
  u32x4_t* dst = h_out + (size_t)b * vec_per_seq;
  const size_t v0 = (size_t)blockIdx.x * (kGatherThreads * kGatherVecPerThread) + threadIdx.x;
  u32x4_t r[kGatherVecPerThread];
#pragma unroll
  for (int u = 0; u < kGatherVecPerThread; ++u) {
    const size_t v = v0 + (size_t)u * kGatherThreads;
    if (v < vec_per_seq) r[u] = src[v];
  }
#pragma unroll
  for (int u = 0; u < kGatherVecPerThread; ++u) {
    const size_t v = v0 + (size_t)u * kGatherThreads;
    if (v < vec_per_seq) __builtin_nontemporal_store(r[u], dst + v);
  }
}

llmc_status_t launch_dedup_resolve(const void* d_keys, const float* d_inv, int k, int dtype, int B, float tau,
                                   int32_t* d_miss_rows, int32_t* d_counters, void* ws, hipStream_t st) {
  const DedupWs w = dedup_ws(ws, B);
  dim3 grid((B + 255) / 256, B);
  { ProfScope ps_("dedup_pairs_kernel", st);
    if (dtype == LLMC_F32)
      LLMC_KERNEL_GGL(dedup_pairs_kernel<float>, grid, dim3(256), 0, st, (const float*)d_keys, d_inv, k, d_miss_rows,
                      d_counters, B, w.S);
    else
      LLMC_KERNEL_GGL(dedup_pairs_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)d_keys, d_inv, k, d_miss_rows,
                      d_counters, B, w.S); }
  LLMC_LAUNCH_CHECK("dedup_pairs_kernel");
  { ProfScope ps_("dedup_resolve_kernel", st);
    LLMC_KERNEL_GGL(dedup_resolve_kernel, dim3(1), dim3(64), 0, st, w.S, B, tau, d_miss_rows, d_counters, w.src_row,
                    w.fol_rows, w.fol_rank, w.fol_sim, w.n_fol); }
  LLMC_LAUNCH_CHECK("dedup_resolve_kernel");
  return LLMC_OK;
}

llmc_status_t launch_dedup_finish(llmc_bank* bank, void* d_h_out, int B, const int32_t* d_slots, int32_t* d_idx,
                                  float* d_sim, uint8_t* d_hit, int32_t* d_counters, uint32_t flags, void* ws,
                                  hipStream_t st) {
  const llmc_bank_desc_t& D = bank->desc;
  const DedupWs w = dedup_ws(ws, B);
  const size_t vec_per_seq = (size_t)D.S * D.d * elem_size(D.dtype) / 16;
  const size_t per_wg = (size_t)kGatherThreads * kGatherVecPerThread;
  dim3 grid((unsigned)((vec_per_seq + per_wg - 1) / per_wg), B);
  { ProfScope ps_("dedup_finish_kernel", st);
    LLMC_KERNEL_GGL(dedup_finish_kernel, grid, dim3(kGatherThreads), 0, st, (u32x4_t*)d_h_out, vec_per_seq, w.n_fol, B,
                    w.src_row, w.fol_rows, w.fol_rank, w.fol_sim, d_slots, d_idx, d_sim, d_hit, D.d_hits,
                    (flags & LLMC_UPDATE_LRU) ? 1 : 0); }
  LLMC_LAUNCH_CHECK("dedup_finish_kernel");
  return LLMC_OK;
}

// copy of referenced value rows: out[rows[i] or i] = act[ref[...]] for the listed rows whose reference is >= 0
llmc_status_t launch_materialize(const llmc_bank* bank, const int32_t* d_ref, const int32_t* d_rows, const int32_t* d_n,
                                 int n_max, void* d_h, hipStream_t st) {
  const llmc_bank_desc_t& D = bank->desc;
  const size_t vec_per_seq = (size_t)D.S * D.d * elem_size(D.dtype) / 16;
  const size_t per_wg = (size_t)kGatherThreads * kGatherVecPerThread;
  dim3 grid((unsigned)((vec_per_seq + per_wg - 1) / per_wg), n_max);
  { ProfScope ps_("materialize_kernel", st);
    LLMC_KERNEL_GGL(materialize_kernel, grid, dim3(kGatherThreads), 0, st, (const u32x4_t*)D.d_act,
                       (const int32_t*)nullptr, d_ref, d_rows, d_n, n_max, vec_per_seq, (u32x4_t*)d_h, (const float*)nullptr,
                       (float*)nullptr, D.d, (const uint32_t*)nullptr, (const float*)nullptr, (uint32_t*)nullptr,
                       (float*)nullptr, 0); }
  LLMC_LAUNCH_CHECK("materialize_kernel");
  return LLMC_OK;
}

}  // namespace llmc
