// Fingerprint of a layer input (Section IV-B of the paper): the average of the token
// vectors, a linear dimensionality reduction, and normalisation to the fixed-length
// key that the bank stores (Section III-A).
//
// Two kernels.  pool_kernel streams h once (HBM-bound): a workgroup owns one
// (sequence, 64-token chunk) and leaves an fp32 partial sum per feature.
// project_kernel adds the partials in chunk order, applies P and c, normalises,
// rounds to the bank's element type and stores 1/|rounded key|.
// Every reduction order depends on S, d and k only, so a sequence's key is the same
// bits wherever it sits in whatever batch.
#include <algorithm>
#include "common.h"

namespace llmc {

constexpr int kTokChunk = 64;   // tokens per pooling workgroup

// token rows of a chunk are dealt to R thread groups (row t goes to group t % R); R depends on d and the element
// type only, so the summation order -- and with it every key -- does not depend on the batch
static inline int pool_row_groups(int G) { return std::max(1, std::min(8, 1024 / G)); }

static inline int pool_chunks(int S) { return (S + kTokChunk - 1) / kTokChunk; }

// grid (chunks, B); block G*R threads, G = d / VEC column groups, R rows in flight.
// Entry b of the grid pools sequence rows[b] (or b) of h; entries beyond *count (if given) and sequences with
// skip[sequence] != 0 (their mean is supplied by the caller) leave at once.  Partials are indexed by entry.
template <typename T>
__global__ void pool_kernel(const T* __restrict__ h, int S, int d, int G, int R, float* __restrict__ partial,
                            int n_chunks, const uint8_t* __restrict__ skip, const int32_t* __restrict__ rows,
                            const int32_t* __restrict__ count, const int32_t* __restrict__ skip_ref) {
  constexpr int VEC = Vec16<T>::N;
  extern __shared__ float red[];  // [R][d]
  const int b = blockIdx.y, chunk = blockIdx.x;
  if (count && b >= *count) return;
  const int seq = rows ? rows[b] : b;
  if (skip && skip[seq]) return;
  if (skip_ref && skip_ref[seq] >= 0) return;      // the row is a reference to a cached output, its key is stored
  const int g = threadIdx.x % G, r = threadIdx.x / G;
  const int t0 = chunk * kTokChunk;
  const int t1 = min(S, t0 + kTokChunk);
  const T* base = h + ((size_t)seq * S) * d + (size_t)g * VEC;
  float acc[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
  int t = t0 + r;
  // eight rows in flight per thread, added in ascending token order
  constexpr int U = 8;
  for (; t + (U - 1) * R < t1; t += U * R) {
    float v[U][VEC];
#pragma unroll
    for (int u = 0; u < U; ++u) Vec16<T>::load(base + (size_t)(t + u * R) * d, v[u]);
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] += v[u][i];
  }
  for (; t < t1; t += R) {
    float v0[VEC];
    Vec16<T>::load(base + (size_t)t * d, v0);
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] += v0[i];
  }
#pragma unroll
  for (int i = 0; i < VEC; ++i) red[(size_t)r * d + g * VEC + i] = acc[i];
  __syncthreads();
  if (r == 0) {
    float* out = partial + ((size_t)b * n_chunks + chunk) * d + g * VEC;
    float s[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      s[i] = acc[i];
      for (int rr = 1; rr < R; ++rr) s[i] += red[(size_t)rr * d + g * VEC + i];
    }
#pragma unroll
    for (int i = 0; i < VEC; i += 4) *reinterpret_cast<float4*>(out + i) = make_float4(s[i], s[i + 1], s[i + 2], s[i + 3]);
  }
}

// Sum over the tokens of one whole sequence with the arithmetic of pool_kernel + the projection's chunk sum, by one
// workgroup and without a partials buffer: chunk after chunk, each thread sums its tokens of the chunk, the row
// groups are combined, and the chunk sums are added in ascending order.  Every thread of the workgroup must call
// it (it contains barriers); threads tid >= G * R only take part in those.  On return the threads of row group 0
// (tid < G) hold in `total` the sums of their column group.  red: LDS, R * d floats.
template <typename T>
__device__ __forceinline__ void pool_sequence(const T* __restrict__ seq, int S, int d, int G, int R, float* red,
                                              float (&total)[Vec16<T>::N]) {
  constexpr int VEC = Vec16<T>::N;
  const int tid = threadIdx.x;
  const bool active = tid < G * R;
  const int g = tid % G, r = tid / G;
  const T* base = seq + (size_t)g * VEC;
#pragma unroll
  for (int i = 0; i < VEC; ++i) total[i] = 0.f;
  for (int t0 = 0; t0 < S; t0 += kTokChunk) {
    const int t1 = min(S, t0 + kTokChunk);
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
    if (active) {
      int t = t0 + r;
      constexpr int U = 8;
      for (; t + (U - 1) * R < t1; t += U * R) {
        float v[U][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u) Vec16<T>::load(base + (size_t)(t + u * R) * d, v[u]);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int i = 0; i < VEC; ++i) acc[i] += v[u][i];
      }
      for (; t < t1; t += R) {
        float v0[VEC];
        Vec16<T>::load(base + (size_t)t * d, v0);
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] += v0[i];
      }
    }
    __syncthreads();                     // the previous chunk's readers are done
    if (active) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) red[(size_t)r * d + g * VEC + i] = acc[i];
    }
    __syncthreads();
    if (active && r == 0) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) {
        float s = acc[i];
        for (int rr = 1; rr < R; ++rr) s += red[(size_t)rr * d + g * VEC + i];
        total[i] += s;
      }
    }
  }
}

// grid (B); block CG * PARTS threads: thread (cg, part) owns the four output columns 4*cg .. 4*cg+3
// over the part-th slice of d; slices are then added in ascending order.
template <typename T>
__global__ __launch_bounds__(1024) void project_kernel(const float* __restrict__ partial, int n_chunks, int S, int d,
                                                       const T* __restrict__ P, const float* __restrict__ bias, int k,
                                                       int parts, T* __restrict__ fp_out, float* __restrict__ inv_out,
                                                       uint32_t* __restrict__ bits_out,
                                                       const float* __restrict__ pooled_in,
                                                       const uint8_t* __restrict__ pooled_valid,
                                                       const T* __restrict__ key_in, const float* __restrict__ key_inv_in,
                                                       const int32_t* __restrict__ row_map,
                                                       const int32_t* __restrict__ count,
                                                       const T* __restrict__ h_inline, int G, int R,
                                                       const int32_t* __restrict__ key_index) {
  // With h_inline (needs blockDim >= G * R and LDS for R * d more floats): a row whose mean is not supplied is
  // pooled here, by this workgroup, with pool_sequence -- no partials, no separate pooling launch.
  // Entry e = blockIdx.x works on row b = row_map[e] (or e) of the outputs.  Sources of the token mean of row b:
  // pooled_in[b] if pooled_in is given and either there are no flags (means kept elsewhere, e.g. beside a bank's
  // values, possibly through row_map) or pooled_valid[b] is set; else the chunk partials of entry e.  If key_in is given and pooled_valid[b], the finished key
  // itself was supplied: it is copied and nothing is computed.
  extern __shared__ float sm[];   // p[d] | v[parts][k]
  float* p = sm;
  float* vpart = sm + d;
  __shared__ double wsum[16];
  __shared__ float s_scale;
  const int entry = blockIdx.x;
  if (count && entry >= *count) return;
  const int b = row_map ? row_map[entry] : entry;
  if (b < 0) return;
  const int nthreads = blockDim.x;
  // key_index: row b is a reference to entry key_index[b] of a bank (negative: not a reference), and key_in /
  // key_inv_in are that bank's stored keys; without it, carried keys sit at row b and pooled_valid flags them
  const int ksrc = key_index ? key_index[b] : b;
  // flags: 1 = the row's mean (or key) is supplied; 2 = the chunk sums of the row are already in `partial` (left there
  // by the producing call's last LayerNorm), so the row was not pooled by this call but is projected as usual
  const bool given = !row_map && (key_index ? ksrc >= 0 : (pooled_valid && pooled_valid[b] == 1));
  const bool has_partials = !row_map && pooled_valid && pooled_valid[b] == 2;
  const bool from_means = pooled_in && (row_map || (!pooled_valid && !key_index) || (given && !key_index));
  if (given && key_in) {
    for (int i = threadIdx.x; i < k; i += nthreads) fp_out[(size_t)b * k + i] = key_in[(size_t)ksrc * k + i];
    if (threadIdx.x == 0) inv_out[b] = key_inv_in[ksrc];
    return;
  }
  const float inv_S = 1.0f / (float)S;
  if (from_means) {
    for (int i = threadIdx.x; i < d; i += nthreads) p[i] = pooled_in[(size_t)b * d + i];
  } else if (h_inline && !has_partials) {
    constexpr int VEC = Vec16<T>::N;
    float total[VEC];
    pool_sequence<T>(h_inline + ((size_t)b * S) * d, S, d, G, R, vpart + (size_t)parts * k, total);
    if ((int)threadIdx.x < G) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) p[threadIdx.x * VEC + i] = total[i] * inv_S;
    }
  } else
  for (int i = threadIdx.x; i < d; i += nthreads) {
    const float* src = partial + (size_t)entry * n_chunks * d + i;
    float s = 0.f;
    // eight chunk partials in flight; added in ascending chunk order
    constexpr int UC = 8;
    int c = 0;
    for (; c + UC <= n_chunks; c += UC) {
      float x[UC];
#pragma unroll
      for (int u = 0; u < UC; ++u) x[u] = src[(size_t)(c + u) * d];
#pragma unroll
      for (int u = 0; u < UC; ++u) s += x[u];
    }
    {
      float x[UC];
#pragma unroll
      for (int u = 0; u < UC; ++u) x[u] = c + u < n_chunks ? src[(size_t)(c + u) * d] : 0.f;
#pragma unroll
      for (int u = 0; u < UC; ++u)
        if (c + u < n_chunks) s += x[u];
    }
    p[i] = s * inv_S;
  }
  __syncthreads();
  {
    const int cgs = k / 4;
    const int cg = threadIdx.x % cgs, part = threadIdx.x / cgs;
    const int per = (d + parts - 1) / parts;
    const int i0 = part * per, i1 = min(d, i0 + per);
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    // sixteen rows of P in flight per thread; the sums run in ascending row order
    constexpr int U = 16;
    auto unpack = [](const T* src, float* w) {
      if (sizeof(T) == 2) {
        const uint2 u = *reinterpret_cast<const uint2*>(src);
        w[0] = __uint_as_float(u.x << 16); w[1] = __uint_as_float(u.x & 0xFFFF0000u);
        w[2] = __uint_as_float(u.y << 16); w[3] = __uint_as_float(u.y & 0xFFFF0000u);
      } else {
        const float4 u = *reinterpret_cast<const float4*>(src);
        w[0] = u.x; w[1] = u.y; w[2] = u.z; w[3] = u.w;
      }
    };
    const T* col = P + cg * 4;
    int i = i0;
    for (; i + U <= i1; i += U) {
      float w[U][4];
#pragma unroll
      for (int u = 0; u < U; ++u) unpack(col + (size_t)(i + u) * k, w[u]);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float pi = p[i + u];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = fmaf(pi, w[u][e], v[e]);
      }
    }
    for (; i < i1; ++i) {
      float w[4];
      unpack(col + (size_t)i * k, w);
      const float pi = p[i];
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = fmaf(pi, w[e], v[e]);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) vpart[part * k + cg * 4 + e] = v[e];
  }
  __syncthreads();
  const int j = threadIdx.x;
  const bool own = j < k;
  float v = 0.f;
  if (own) {
    v = vpart[j];
    for (int s = 1; s < parts; ++s) v += vpart[s * k + j];
    if (bias) v += bias[j];
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (bits_out) {
    // sign-bit key (Section IV-B, SimHash): bit j = (v_j >= 0), 32 per word, least significant first
    const unsigned long long m = __ballot(own && v >= 0.f);
    if (lane == 0 && wave * 64 < k) bits_out[(size_t)b * (k / 32) + wave * 2] = (uint32_t)m;
    if (lane == 32 && wave * 64 + 32 < k) bits_out[(size_t)b * (k / 32) + wave * 2 + 1] = (uint32_t)(m >> 32);
    return;
  }
  // |v|^2 in fp64: lanes of each wave, then waves in order
  const int n_waves_k = (k + 63) / 64;
  double sq = own ? (double)v * (double)v : 0.0;
  sq = wave_sum(sq);
  if (lane == 0 && wave < 16) wsum[wave] = sq;
  __syncthreads();
  if (threadIdx.x == 0) {
    double tot = 0.0;
    for (int w = 0; w < n_waves_k; ++w) tot += wsum[w];
    float nrm = (float)sqrt(tot);
    s_scale = 1.0f / fmaxf(nrm, 1e-12f);
  }
  __syncthreads();
  float q = 0.f;
  if (own) {
    q = Elem<T>::round(v * s_scale);
    Elem<T>::store(fp_out + (size_t)b * k + j, q);
  }
  double sq2 = own ? (double)q * (double)q : 0.0;
  sq2 = wave_sum(sq2);
  __syncthreads();
  if (lane == 0 && wave < 16) wsum[wave] = sq2;
  __syncthreads();
  if (threadIdx.x == 0) {
    double tot = 0.0;
    for (int w = 0; w < n_waves_k; ++w) tot += wsum[w];
    inv_out[b] = tot > 0.0 ? (float)(1.0 / sqrt(tot)) : 0.f;
  }
}

// one wavefront per key: 1/|key| with fp64 accumulation
template <typename T>
__global__ void inv_norm_kernel(const T* __restrict__ fp, int64_t n, int k, float* __restrict__ out) {
  const int64_t row = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (row >= n) return;
  const int lane = threadIdx.x & 63;
  double s = 0.0;
  for (int i = lane; i < k; i += 64) {
    double x = (double)Elem<T>::load(fp + row * k + i);
    s += x * x;
  }
  s = wave_sum(s);
  if (lane == 0) out[row] = s > 0.0 ? (float)(1.0 / sqrt(s)) : 0.f;
}

// Token means of whole sequences, one workgroup each.  Entry b pools sequence rows[b] (or b) into out[dst[b] or b];
// entries beyond *count, and negative destinations, are skipped.  grid (n_max); block G*R threads; LDS R*d floats.
template <typename T>
__global__ void pool_direct_kernel(const T* __restrict__ h, int S, int d, int G, int R, const int32_t* __restrict__ rows,
                                   const int32_t* __restrict__ count, const int32_t* __restrict__ dst,
                                   float* __restrict__ out, int ld_out) {
  constexpr int VEC = Vec16<T>::N;
  extern __shared__ float red[];  // [R][d]
  const int b = blockIdx.x;
  if (count && b >= *count) return;
  const int o = dst ? dst[b] : b;
  if (o < 0) return;
  const int seq = rows ? rows[b] : b;
  float total[VEC];
  pool_sequence<T>(h + ((size_t)seq * S) * d, S, d, G, R, red, total);
  if ((int)threadIdx.x < G) {
    const float inv_S = 1.0f / (float)S;
#pragma unroll
    for (int i = 0; i < VEC; ++i) out[(size_t)o * ld_out + threadIdx.x * VEC + i] = total[i] * inv_S;
  }
}

size_t fingerprint_ws_bytes(int B, int S, int d) {
  return align_up((size_t)B * pool_chunks(S) * d * sizeof(float), 256);
}

template <typename T>
static llmc_status_t fingerprint_t(const T* h, int B, int S, int d, const T* P, const float* bias, int k,
                                   T* fp, float* inv, uint32_t* bits, float* partial, const float* pooled_in,
                                   const uint8_t* pooled_valid, hipStream_t st, const T* key_in = nullptr,
                                   const float* key_inv_in = nullptr, bool few_uncarried = false,
                                   const int32_t* key_index = nullptr) {
  constexpr int VEC = Vec16<T>::N;
  const int G = d / VEC;
  const int R = pool_row_groups(G);
  const int n_chunks = pool_chunks(S);
  // slices of d per output column group; depends on k only.  k <= 1024 gives at least k threads.
  const int cgs = k / 4;
  const int parts = std::max(1, std::min(1024 / cgs, 16));
  const int threads = std::max(cgs * parts, k);
  // When the caller expects nearly every row to arrive with its mean or key (a carry from the producing call), the
  // projection's workgroups pool the few others themselves (same arithmetic, see pool_sequence) and the pooling
  // launch is dropped.  Otherwise every uncarried row is pooled by the dedicated, wider kernel.
  const bool inline_pool = few_uncarried && (pooled_valid != nullptr || key_index != nullptr) && threads >= G * R &&
                           (size_t)(d + parts * k + R * d) * sizeof(float) <= 64 * 1024;
  if (!inline_pool) {
    dim3 grid(n_chunks, B);
    { ProfScope ps_("pool_kernel", st); LLMC_KERNEL_GGL(pool_kernel<T>, grid, dim3(G * R), (size_t)R * d * sizeof(float), st, h, S, d, G, R, partial,
                       n_chunks, pooled_valid, (const int32_t*)nullptr, (const int32_t*)nullptr, key_index); }
    LLMC_LAUNCH_CHECK("pool_kernel");
  }
  {
    ProfScope ps_("project_kernel", st);
    LLMC_KERNEL_GGL(project_kernel<T>, dim3(B), dim3(threads),
                       (size_t)(d + parts * k + (inline_pool ? R * d : 0)) * sizeof(float), st, partial, n_chunks, S, d, P,
                       bias, k, parts, fp, inv, bits, pooled_in, pooled_valid, key_in, key_inv_in, (const int32_t*)nullptr,
                       (const int32_t*)nullptr, inline_pool ? h : (const T*)nullptr, G, R, key_index);
  }
  LLMC_LAUNCH_CHECK("project_kernel");
  return LLMC_OK;
}

llmc_status_t launch_fingerprint(const void* d_h, const int32_t*, int B, int S, int d, int dtype, const void* d_proj,
                                 const float* d_bias, int k, void* d_fp, float* d_inv, void* ws, hipStream_t st,
                                 const float* pooled_in, const uint8_t* pooled_valid, const void* key_in,
                                 const float* key_inv_in, bool few_uncarried, const int32_t* key_index) {
  if (dtype == LLMC_F32)
    return fingerprint_t<float>((const float*)d_h, B, S, d, (const float*)d_proj, d_bias, k, (float*)d_fp, d_inv,
                                nullptr, (float*)ws, pooled_in, pooled_valid, st, (const float*)key_in, key_inv_in,
                                few_uncarried, key_index);
  return fingerprint_t<bf16_t>((const bf16_t*)d_h, B, S, d, (const bf16_t*)d_proj, d_bias, k, (bf16_t*)d_fp, d_inv,
                               nullptr, (float*)ws, pooled_in, pooled_valid, st, (const bf16_t*)key_in, key_inv_in,
                               few_uncarried, key_index);
}

// token means of B whole sequences through the wide pooling kernel: chunk partials first, then one workgroup per
// sequence adds them in ascending chunk order (the arithmetic of the projection's own chunk sum, so the mean has
// the bits the fingerprint uses) and writes out[b * ld_out ..] [d]
__global__ void mean_from_partials_kernel(const float* __restrict__ partial, int n_chunks, int d, float inv_S,
                                          float* __restrict__ out, int ld_out) {
  const int b = blockIdx.x;
  for (int i = threadIdx.x; i < d; i += blockDim.x) {
    const float* src = partial + (size_t)b * n_chunks * d + i;
    float s = 0.f;
    for (int c = 0; c < n_chunks; ++c) s += src[(size_t)c * d];
    out[(size_t)b * ld_out + i] = s * inv_S;
  }
}

template <typename T>
static llmc_status_t pool_means_t(const T* h, int B, int S, int d, float* partial, float* out, int ld_out, hipStream_t st) {
  constexpr int VEC = Vec16<T>::N;
  const int G = d / VEC;
  const int R = pool_row_groups(G);
  const int n_chunks = pool_chunks(S);
  { ProfScope ps_("pool_kernel", st);
    LLMC_KERNEL_GGL(pool_kernel<T>, dim3(n_chunks, B), dim3(G * R), (size_t)R * d * sizeof(float), st, h, S, d, G, R, partial,
                    n_chunks, (const uint8_t*)nullptr, (const int32_t*)nullptr, (const int32_t*)nullptr,
                    (const int32_t*)nullptr); }
  LLMC_LAUNCH_CHECK("pool_kernel");
  { ProfScope ps_("mean_from_partials_kernel", st);
    LLMC_KERNEL_GGL(mean_from_partials_kernel, dim3(B), dim3(256), 0, st, partial, n_chunks, d, 1.0f / (float)S, out, ld_out); }
  LLMC_LAUNCH_CHECK("mean_from_partials_kernel");
  return LLMC_OK;
}

llmc_status_t launch_pool_means(const void* d_h, int B, int S, int d, int dtype, void* ws_partials, float* d_out,
                                int ld_out, hipStream_t st) {
  if (dtype == LLMC_F32) return pool_means_t<float>((const float*)d_h, B, S, d, (float*)ws_partials, d_out, ld_out, st);
  return pool_means_t<bf16_t>((const bf16_t*)d_h, B, S, d, (float*)ws_partials, d_out, ld_out, st);
}

// keys of token means kept elsewhere: entry e < *count (or n_max) projects means[rows[e]] into fp[rows[e]], inv[rows[e]]
template <typename T>
static llmc_status_t project_rows_t(const float* means, int n_max, int d, const T* P, const float* bias, int k,
                                    const int32_t* rows, const int32_t* count, T* fp, float* inv, hipStream_t st) {
  const int cgs = k / 4;
  const int parts = std::max(1, std::min(1024 / cgs, 16));
  ProfScope ps_("project_kernel", st);
  LLMC_KERNEL_GGL(project_kernel<T>, dim3(n_max), dim3(std::max(cgs * parts, k)),
                     (size_t)(d + parts * k) * sizeof(float), st, (const float*)nullptr, 0, 1, d, P, bias, k, parts, fp, inv,
                     (uint32_t*)nullptr, means, (const uint8_t*)nullptr, (const T*)nullptr, (const float*)nullptr, rows,
                     count, (const T*)nullptr, 0, 0, (const int32_t*)nullptr);
  LLMC_LAUNCH_CHECK("project_kernel");
  return LLMC_OK;
}

llmc_status_t launch_project_rows(const float* d_means, int n_max, int d, int dtype, const void* d_proj,
                                  const float* d_bias, int k, const int32_t* d_rows, const int32_t* d_count, void* d_fp,
                                  float* d_inv, hipStream_t st) {
  if (dtype == LLMC_F32)
    return project_rows_t<float>(d_means, n_max, d, (const float*)d_proj, d_bias, k, d_rows, d_count, (float*)d_fp, d_inv,
                                 st);
  return project_rows_t<bf16_t>(d_means, n_max, d, (const bf16_t*)d_proj, d_bias, k, d_rows, d_count, (bf16_t*)d_fp,
                                d_inv, st);
}

// token means of the sequences rows[0 .. *count) (or 0 .. n_max) of h, written to out[(dst[i] or i) * ld_out ..] fp32
template <typename T>
static llmc_status_t pool_rows_t(const T* h, int n_max, int S, int d, const int32_t* rows, const int32_t* count,
                                 const int32_t* dst, float* out, hipStream_t st, int ld_out) {
  constexpr int VEC = Vec16<T>::N;
  const int G = d / VEC;
  const int R = pool_row_groups(G);
  { ProfScope ps_("pool_direct_kernel", st);
    LLMC_KERNEL_GGL(pool_direct_kernel<T>, dim3(n_max), dim3(G * R), (size_t)R * d * sizeof(float), st, h, S, d, G, R,
                       rows, count, dst, out, ld_out > 0 ? ld_out : d); }
  LLMC_LAUNCH_CHECK("pool_direct_kernel");
  return LLMC_OK;
}

llmc_status_t launch_pool_rows(const void* d_h, int n_max, int S, int d, int dtype, const int32_t* d_rows,
                               const int32_t* d_count, const int32_t* d_dst, float* d_out, hipStream_t st, int ld_out) {
  if (dtype == LLMC_F32)
    return pool_rows_t<float>((const float*)d_h, n_max, S, d, d_rows, d_count, d_dst, d_out, st, ld_out);
  return pool_rows_t<bf16_t>((const bf16_t*)d_h, n_max, S, d, d_rows, d_count, d_dst, d_out, st, ld_out);
}

// same pooling and projection, but the key is the sign of each projection
llmc_status_t launch_fingerprint_bits(const void* d_h, int B, int S, int d, int dtype, const void* d_proj,
                                      const float* d_bias, int k, uint32_t* d_bits, void* ws, hipStream_t st,
                                      const float* pooled_in, const uint8_t* pooled_valid, bool few_uncarried) {
  if (dtype == LLMC_F32)
    return fingerprint_t<float>((const float*)d_h, B, S, d, (const float*)d_proj, d_bias, k, nullptr, nullptr, d_bits,
                                (float*)ws, pooled_in, pooled_valid, st, nullptr, nullptr, few_uncarried);
  return fingerprint_t<bf16_t>((const bf16_t*)d_h, B, S, d, (const bf16_t*)d_proj, d_bias, k, nullptr, nullptr, d_bits,
                               (float*)ws, pooled_in, pooled_valid, st, nullptr, nullptr, few_uncarried);
}

llmc_status_t launch_inv_norm(const void* d_fp, int64_t n, int k, int dtype, float* d_out, hipStream_t st) {
  const int rows_per_block = 4;
  const unsigned blocks = (unsigned)((n + rows_per_block - 1) / rows_per_block);
  if (dtype == LLMC_F32)
    { ProfScope ps_("inv_norm_kernel", st); LLMC_KERNEL_GGL(inv_norm_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)d_fp, n, k, d_out); }
  else
    { ProfScope ps_("inv_norm_kernel", st); LLMC_KERNEL_GGL(inv_norm_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, (const bf16_t*)d_fp, n, k, d_out); }
  LLMC_LAUNCH_CHECK("inv_norm_kernel");
  return LLMC_OK;
}

}  // namespace llmc
