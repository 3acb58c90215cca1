// Bucketed lookup of sign-bit keys (Section IV-B: keys are compared by cosine similarity or by LSH;
// Section III-A: hashing is there to keep the comparison cost below linear in the bank size).
//
// A k-bit key is cut into k / 16 bands of 16 bits (band b = bits 16 b .. 16 b + 15).  The index holds, per
// band, the valid slots grouped by the band's value: start[b][v] .. start[b][v + 1] is the range of
// order[b][*] that lists the slots whose band b equals v.  A query compares itself (XOR + popcount) only with
// the members of the k / 16 buckets it falls into, so the work per query is the size of those buckets and not
// the size of the bank.  The answer is the nearest CANDIDATE (lowest slot among equals); it equals the exact
// nearest neighbour whenever that neighbour shares one whole band with the query.
//
// Build: histogram of band values (atomics), exclusive scan per band (one workgroup each), scatter through
// per-bucket cursors (atomics).  The order of slots inside a bucket depends on timing; the lookup takes a
// minimum over the bucket, so its result does not.
#include "common.h"

namespace llmc {

constexpr int kLshValues = 65536;

struct LshLayout {
  size_t off_start, off_cursor, off_order, bytes;
  int bands;
};

static LshLayout lsh_layout(int N, int k) {
  LshLayout L;
  L.bands = k / 16;
  L.off_start = 0;
  L.off_cursor = align_up((size_t)L.bands * (kLshValues + 1) * sizeof(uint32_t), 256);
  L.off_order = L.off_cursor + align_up((size_t)L.bands * kLshValues * sizeof(uint32_t), 256);
  L.bytes = L.off_order + align_up((size_t)L.bands * N * sizeof(int32_t), 256);
  return L;
}

size_t lsh_index_bytes(int N, int k) { return lsh_layout(N, k).bytes; }

__device__ __forceinline__ uint32_t band_value(const uint32_t* key, int band) {
  return (key[band >> 1] >> (16 * (band & 1))) & 0xFFFFu;
}

__global__ void lsh_zero_kernel(uint32_t* p, size_t n, const int32_t* __restrict__ changed) {
  if (changed && *changed == 0) return;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// grid over (slot, band): counts[band][value] += 1 for valid slots
__global__ void lsh_count_kernel(const uint32_t* __restrict__ bank, const uint8_t* __restrict__ valid, int N, int W,
                                 int bands, uint32_t* __restrict__ counts, const int32_t* __restrict__ changed) {
  if (changed && *changed == 0) return;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)N * bands) return;
  const int j = (int)(i / bands), b = (int)(i % bands);
  if (!valid[j]) return;
  atomicAdd(&counts[(size_t)b * kLshValues + band_value(bank + (size_t)j * W, b)], 1u);
}

// one workgroup of 1024 threads per band: start[b][v] = number of slots with a smaller value; cursor = start
__global__ __launch_bounds__(1024) void lsh_scan_kernel(uint32_t* __restrict__ cursor, uint32_t* __restrict__ start,
                                                        const int32_t* __restrict__ changed) {
  __shared__ uint32_t wave_tot[16];
  __shared__ uint32_t carry;
  if (changed && *changed == 0) return;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint32_t* cnt = cursor + (size_t)b * kLshValues;          // counts arrive in the cursor array
  uint32_t* st = start + (size_t)b * (kLshValues + 1);
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int base = 0; base < kLshValues; base += 1024 * 4) {
    const int v0 = base + tid * 4;
    const uint32_t c0 = cnt[v0], c1 = cnt[v0 + 1], c2 = cnt[v0 + 2], c3 = cnt[v0 + 3];
    const uint32_t own = c0 + c1 + c2 + c3;
    uint32_t incl = own;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t x = __shfl_up(incl, o, 64);
      if (lane >= o) incl += x;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = carry;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
    const uint32_t e0 = before + incl - own;
    st[v0] = e0; st[v0 + 1] = e0 + c0; st[v0 + 2] = e0 + c0 + c1; st[v0 + 3] = e0 + c0 + c1 + c2;
    cnt[v0] = e0; cnt[v0 + 1] = e0 + c0; cnt[v0 + 2] = e0 + c0 + c1; cnt[v0 + 3] = e0 + c0 + c1 + c2;
    __syncthreads();
    if (tid == 1023) carry = before + incl;
    __syncthreads();
  }
  if (tid == 0) st[kLshValues] = carry;
}

__global__ void lsh_scatter_kernel(const uint32_t* __restrict__ bank, const uint8_t* __restrict__ valid, int N, int W,
                                   int bands, uint32_t* __restrict__ cursor, int32_t* __restrict__ order,
                                   const int32_t* __restrict__ changed) {
  if (changed && *changed == 0) return;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)N * bands) return;
  const int j = (int)(i / bands), b = (int)(i % bands);
  if (!valid[j]) return;
  const uint32_t pos = atomicAdd(&cursor[(size_t)b * kLshValues + band_value(bank + (size_t)j * W, b)], 1u);
  order[(size_t)b * N + pos] = j;
}

// one wavefront per query: lanes walk the members of the query's bucket in every band
template <int W>
__global__ __launch_bounds__(256) void lsh_match_kernel(const uint32_t* __restrict__ bank, int N,
                                                        const uint32_t* __restrict__ start,
                                                        const int32_t* __restrict__ order,
                                                        const uint32_t* __restrict__ queries, int B, int max_hamming,
                                                        int32_t* __restrict__ idx_out, int32_t* __restrict__ dist_out,
                                                        uint8_t* __restrict__ hit_out, int32_t* __restrict__ compared_out,
                                                        float* __restrict__ sim_out) {
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (b >= B) return;
  const int lane = threadIdx.x & 63;
  uint32_t q[W];
#pragma unroll
  for (int w = 0; w < W; ++w) q[w] = queries[(size_t)b * W + w];
  unsigned long long best = ~0ull;        // (distance << 32) | slot: the minimum is the nearest, lowest slot among equals
  int compared = 0;
  for (int band = 0; band < 2 * W; ++band) {
    const uint32_t v = (q[band >> 1] >> (16 * (band & 1))) & 0xFFFFu;
    const uint32_t* st = start + (size_t)band * (kLshValues + 1);
    const uint32_t lo = st[v], hi = st[v + 1];
    compared += (int)(hi - lo);
    for (uint32_t p = lo + lane; p < hi; p += 64) {
      const int j = order[(size_t)band * N + p];
      const uint32_t* key = bank + (size_t)j * W;
      uint32_t h = 0;
#pragma unroll
      for (int w = 0; w < W; ++w) h += __builtin_popcount(q[w] ^ key[w]);
      const unsigned long long cand = ((unsigned long long)h << 32) | (uint32_t)j;
      best = cand < best ? cand : best;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const unsigned long long other = ((unsigned long long)__shfl_xor((uint32_t)(best >> 32), o, 64) << 32) |
                                     __shfl_xor((uint32_t)best, o, 64);
    best = other < best ? other : best;
  }
  if (lane == 0) {
    const bool found = best != ~0ull;
    const int32_t h = (int32_t)(best >> 32);
    idx_out[b] = found ? (int32_t)(uint32_t)best : -1;
    if (dist_out) dist_out[b] = found ? h : 0x7FFFFFFF;
    if (hit_out) hit_out[b] = (found && h <= max_hamming) ? 1 : 0;
    // the cosine that the distance stands for, as the full comparison reports it
    if (sim_out) sim_out[b] = found ? cosf(3.14159265358979323846f * (float)h / (float)(32 * W)) : -INFINITY;
    if (compared_out) compared_out[b] = compared;       // bucket members visited (a slot in several buckets counts each time)
  }
}

llmc_status_t launch_lsh_build(const uint32_t* d_bank_bits, const uint8_t* d_valid, int N, int k, void* d_index,
                               hipStream_t st, const int32_t* d_changed) {
  const LshLayout L = lsh_layout(N, k);
  uint32_t* start = (uint32_t*)((char*)d_index + L.off_start);
  uint32_t* cursor = (uint32_t*)((char*)d_index + L.off_cursor);
  int32_t* order = (int32_t*)((char*)d_index + L.off_order);
  const size_t n_cnt = (size_t)L.bands * kLshValues, n_pairs = (size_t)N * L.bands;
  const int W = k / 32;
  { ProfScope ps_("lsh_zero_kernel", st);
    LLMC_KERNEL_GGL(lsh_zero_kernel, dim3((unsigned)((n_cnt + 255) / 256)), dim3(256), 0, st, cursor, n_cnt, d_changed); }
  LLMC_LAUNCH_CHECK("lsh_zero_kernel");
  { ProfScope ps_("lsh_count_kernel", st);
    LLMC_KERNEL_GGL(lsh_count_kernel, dim3((unsigned)((n_pairs + 255) / 256)), dim3(256), 0, st, d_bank_bits, d_valid, N,
                       W, L.bands, cursor, d_changed); }
  LLMC_LAUNCH_CHECK("lsh_count_kernel");
  { ProfScope ps_("lsh_scan_kernel", st);
    LLMC_KERNEL_GGL(lsh_scan_kernel, dim3(L.bands), dim3(1024), 0, st, cursor, start, d_changed); }
  LLMC_LAUNCH_CHECK("lsh_scan_kernel");
  { ProfScope ps_("lsh_scatter_kernel", st);
    LLMC_KERNEL_GGL(lsh_scatter_kernel, dim3((unsigned)((n_pairs + 255) / 256)), dim3(256), 0, st, d_bank_bits, d_valid,
                       N, W, L.bands, cursor, order, d_changed); }
  LLMC_LAUNCH_CHECK("lsh_scatter_kernel");
  return LLMC_OK;
}

llmc_status_t launch_lsh_match(const uint32_t* d_bank_bits, int N, int k, const void* d_index,
                               const uint32_t* d_query_bits, int B, int max_hamming, int32_t* d_idx, int32_t* d_dist,
                               uint8_t* d_hit, int32_t* d_compared, hipStream_t st, float* d_sim) {
  const LshLayout L = lsh_layout(N, k);
  const uint32_t* start = (const uint32_t*)((const char*)d_index + L.off_start);
  const int32_t* order = (const int32_t*)((const char*)d_index + L.off_order);
  const dim3 grid((B + 3) / 4), block(256);
  ProfScope ps_("lsh_match_kernel", st);
#define LLMC_LSH_CASE(W_) LLMC_KERNEL_GGL(lsh_match_kernel<W_>, grid, block, 0, st, d_bank_bits, N, start, order, \
                                             d_query_bits, B, max_hamming, d_idx, d_dist, d_hit, d_compared, d_sim)
  switch (k / 32) {
    case 2: LLMC_LSH_CASE(2); break;
    case 4: LLMC_LSH_CASE(4); break;
    case 8: LLMC_LSH_CASE(8); break;
    case 16: LLMC_LSH_CASE(16); break;
    default: return set_error(LLMC_ERR_SHAPE, "bucketed lookup supports k = 64, 128, 256 or 512 bits");
  }
#undef LLMC_LSH_CASE
  LLMC_LAUNCH_CHECK("lsh_match_kernel");
  return LLMC_OK;
}

}  // namespace llmc
