// The miss path: one transformer block f_l (Section IV-A of the paper) applied to the
// sequences that found no match, named by a device-side row list and count.
//
// Rows are processed in a compact token space: compact token r belongs to list entry
// r / S and is token r % S of sequence rows[r / S].  Every kernel is launched for the
// worst case (all B sequences) and reads the real count on the device; workgroups
// beyond it exit at once, so the host never learns the number of misses.
//
// Kernels: linear layers on the bf16 matrix cores (fp32 accumulate) with bias, GELU,
// residual and row gather/scatter fused into the epilogue; a plain fp32 FMA GEMM for
// fp32 runs; LayerNorm with one wavefront per token (the last LayerNorm of a post-LN block
// also leaves the pooled chunk sums of the rows it writes for the next fingerprint); the
// fp32 softmax attention with one thread per query row.  The bf16 attention on the matrix
// cores is a translation unit of its own.
#include "common.h"
#include <algorithm>
#include "gemm.h"

namespace llmc {

typedef MmaCfg<128, 128, 32, 2, 2> GemmCfg;

// Launches are sized for the worst case (every sequence a miss) but capped: workgroups walk
// their tiles / rows with a grid stride and read the real count on the device, so a layer
// with few or no misses costs a small, fixed number of idle workgroups.
constexpr int kMaxGrid = 512;

// ---- fp32 GEMM, plain FMA: 64x64 tile, 16-wide k step, 4x4 outputs per thread ------------------
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs g, int tiles_n) {
  __shared__ float sA[16][64 + 4];
  __shared__ float sB[16][64 + 4];
  const int n_seq = g.count ? min(*g.count, g.max_seqs) : g.max_seqs;
  const int M = n_seq * g.S;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x % tiles_n;
  const int m0 = tile_m * 64, n0 = tile_n * 64;
  if (m0 >= M) return;
  const int tid = threadIdx.x;
  const float* A = (const float*)g.A;
  const float* W = (const float*)g.W;
  // each thread loads one float4 of A and one of W per k step: row = tid / 4, k = (tid % 4) * 4
  const int lr = tid >> 2, lk = (tid & 3) * 4;
  const float* ap = A + map_row(g.a_rows, min(m0 + lr, M - 1), g.S) * g.lda + lk;
  const float* wp = W + (size_t)min(n0 + lr, g.N - 1) * g.K + lk;
  const int tm = (tid >> 4) * 4, tn = (tid & 15) * 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < g.K; k0 += 16) {
    const float4 va = *reinterpret_cast<const float4*>(ap + k0);
    const float4 vw = *reinterpret_cast<const float4*>(wp + k0);
    sA[lk + 0][lr] = va.x; sA[lk + 1][lr] = va.y; sA[lk + 2][lr] = va.z; sA[lk + 3][lr] = va.w;
    sB[lk + 0][lr] = vw.x; sB[lk + 1][lr] = vw.y; sB[lk + 2][lr] = vw.z; sB[lk + 3][lr] = vw.w;
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = sA[kk][tm + i]; b[i] = sB[kk][tn + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  const float* bias = (const float*)g.bias;
  const float* resid = (const float*)g.resid;
  float* out = (float*)g.out;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + tm + i;
    if (m >= M) continue;
    const int64_t ro = map_row(g.o_rows, m, g.S) * g.ldo;
    const int64_t rr = resid ? map_row(g.r_rows, m, g.S) * g.ldr : 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tn + j;
      if (n >= g.N) continue;
      float v = apply_act(acc[i][j] + (bias ? bias[n] : 0.f), g.act);
      if (resid) v += resid[rr + n];
      out[ro + n] = v;
    }
  }
}

// 128 x 128 block, 8 wavefronts (2 x 4), two 64-column stages filled by direct-to-LDS loads: 68 KiB of LDS,
// so two workgroups share a compute unit and one's epilogue overlaps the other's main loop
typedef DmaCfg<128, 128, 2, 4, 2> GemmDmaCfg;
// with few rows: 64 x 128 blocks, three stages (72 KiB, still two workgroups per compute unit)
typedef DmaCfg<64, 128, 2, 4, 3> GemmDmaSmallCfg;

static llmc_status_t launch_gemm(const GemmArgs& g, int dtype, hipStream_t st) {
  if (dtype == LLMC_BF16) {
    if (g.K % 64 == 0) {
      using C = GemmDmaCfg;
      using CS = GemmDmaSmallCfg;
      static std::atomic<bool> lds_set[64];
      const auto kernel = gemm_bf16_dma_kernel<C, CS>;
      const size_t lds_bytes = gemm_dma_smem_bytes<C, CS>();
      LLMC_TRY(ensure_dynamic_lds((const void*)kernel, lds_bytes, lds_set));
      const int tiles_n = (g.N + C::BN - 1) / C::BN;
      // the grid covers the smaller tiling too, which the kernel takes when the rows it finds on the device are few
      const int tiles_m = (g.max_seqs * g.S + CS::BM - 1) / CS::BM;
      GemmArgs a = g;
      a.xcd_chunks = tiles_n <= 8 ? 1 : 2;   // every XCD walks its own eighth of the tile list; wide outputs in grouped order
      ProfScope ps_("gemm_bf16_kernel", st);
      LLMC_KERNEL_GGL(kernel, dim3(std::min((tiles_m * tiles_n + 7) & ~7, kMaxGrid)), dim3(C::THREADS), lds_bytes, st, a,
                      tiles_n);
    } else {
      const int tiles_n = (g.N + GemmCfg::BN - 1) / GemmCfg::BN;
      const int tiles_m = (g.max_seqs * g.S + GemmCfg::BM - 1) / GemmCfg::BM;
      ProfScope ps_("gemm_bf16_kernel", st);
      LLMC_KERNEL_GGL(gemm_bf16_kernel<GemmCfg>, dim3(std::min(tiles_m * tiles_n, kMaxGrid)), dim3(GemmCfg::THREADS),
                         0, st, g, tiles_n);
    }
  } else {
    const int tiles_n = (g.N + 63) / 64;
    const int tiles_m = (g.max_seqs * g.S + 63) / 64;
    ProfScope ps_("gemm_f32_kernel", st);
    LLMC_KERNEL_GGL(gemm_f32_kernel, dim3((unsigned)tiles_m * tiles_n), dim3(256), 0, st, g, tiles_n);
  }
  LLMC_LAUNCH_CHECK("gemm");
  return LLMC_OK;
}

// ---- LayerNorm: one wavefront per token, two-pass statistics in fp32 -----------------------------
template <typename T, int MAXV>
__global__ __launch_bounds__(256) void layernorm_kernel(const T* __restrict__ in, int ld_in, const int32_t* in_rows,
                                                        T* __restrict__ out, int ld_out, const int32_t* out_rows,
                                                        const T* __restrict__ gamma, const T* __restrict__ beta,
                                                        float eps, int d, int S, const int32_t* count, int max_seqs) {
  constexpr int VEC = Vec16<T>::N;
  const int n_seq = count ? min(*count, max_seqs) : max_seqs;
  const int M = n_seq * S;
  const int lane = threadIdx.x & 63;
  const int nvec = d / VEC;
  for (int r = blockIdx.x * 4 + (threadIdx.x >> 6); r < M; r += gridDim.x * 4) {
  const T* src = in + map_row(in_rows, r, S) * ld_in;
  float x[MAXV][VEC];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int v = lane + i * 64;
    if (v < nvec) {
      Vec16<T>::load(src + v * VEC, x[i]);
#pragma unroll
      for (int e = 0; e < VEC; ++e) s += x[i][e];
    }
  }
  const float mean = wave_sum(s) / (float)d;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int v = lane + i * 64;
    if (v < nvec) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float c = x[i][e] - mean;
        q += c * c;
      }
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)d + eps);
  T* dst = out + map_row(out_rows, r, S) * ld_out;
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int v = lane + i * 64;
    if (v < nvec) {
      float gv[VEC], bv[VEC], y[VEC];
      Vec16<T>::load(gamma + v * VEC, gv);
      Vec16<T>::load(beta + v * VEC, bv);
#pragma unroll
      for (int e = 0; e < VEC; ++e) y[e] = (x[i][e] - mean) * rstd * gv[e] + bv[e];
      Vec16<T>::store(dst + v * VEC, y);
    }
  }
  }
}

// ---- the block's LAST LayerNorm with the next layer's pooling folded in ---------------------------------------
// The output of a post-LayerNorm block is written by this kernel, and the next layer's fingerprint starts by
// summing exactly these rows over the tokens.  A workgroup owns one (sequence, 64-token chunk): its wavefronts
// normalise the chunk's tokens (same arithmetic as layernorm_kernel), store them, and keep the ROUNDED outputs in
// LDS; then the chunk's column sums are formed in the order of the fingerprint's pooling kernel -- token t of the
// chunk belongs to row group t % R, a group's tokens are added in ascending order starting from zero, and the
// groups are added in ascending order -- so the partial sums are the bits that kernel would produce, and the
// sequence is flagged so that the next call does not read its rows again.  grid (chunks, max_seqs).
constexpr int kLnPoolThreads = 1024;
constexpr int kLnPoolChunk = 64;             // tokens per pooling chunk: must equal the fingerprint's
constexpr int kLnPoolTokPerWave = kLnPoolChunk / (kLnPoolThreads / 64);

template <typename T, int MAXV>
__global__ __launch_bounds__(kLnPoolThreads) void layernorm_pool_kernel(
    const T* __restrict__ in, int ld_in, T* __restrict__ out, int ld_out, const int32_t* __restrict__ out_rows,
    const T* __restrict__ gamma, const T* __restrict__ beta, float eps, int d, int S, const int32_t* count, int max_seqs,
    float* __restrict__ partial, int n_chunks, int R, uint8_t* __restrict__ pooled_flags) {
  constexpr int VEC = Vec16<T>::N;
  constexpr int TPW = kLnPoolTokPerWave;
  extern __shared__ __attribute__((aligned(16))) unsigned char ln_lds[];
  T* tile = reinterpret_cast<T*>(ln_lds);                 // [kLnPoolChunk][d], the outputs as stored
  const int n_seq = count ? min(*count, max_seqs) : max_seqs;
  const int q = blockIdx.y, chunk = blockIdx.x;
  if (q >= n_seq) return;
  const int seq = out_rows ? out_rows[q] : q;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nvec = d / VEC;
  const int t0 = chunk * kLnPoolChunk, t1 = min(S, t0 + kLnPoolChunk);
  // a wavefront owns TPW consecutive tokens of the chunk; all their rows are requested before the first is reduced
  const int tw = t0 + wave * TPW;
  float x[TPW][MAXV][VEC];
#pragma unroll
  for (int u = 0; u < TPW; ++u) {
    const int t = min(tw + u, S - 1);                     // the block's temporaries are in compact token order
    const T* src = in + ((size_t)q * S + t) * ld_in;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
      const int v = lane + i * 64;
      if (v < nvec) Vec16<T>::load(src + v * VEC, x[u][i]);
    }
  }
  float gv[MAXV][VEC], bv[MAXV][VEC];
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int v = lane + i * 64;
    if (v < nvec) {
      Vec16<T>::load(gamma + v * VEC, gv[i]);
      Vec16<T>::load(beta + v * VEC, bv[i]);
    }
  }
#pragma unroll
  for (int u = 0; u < TPW; ++u) {
    const int t = tw + u;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
      const int v = lane + i * 64;
      if (v < nvec) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) s += x[u][i][e];
      }
    }
    const float mean = wave_sum(s) / (float)d;
    float qq = 0.f;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
      const int v = lane + i * 64;
      if (v < nvec) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float c = x[u][i][e] - mean;
          qq += c * c;
        }
      }
    }
    const float rstd = 1.0f / sqrtf(wave_sum(qq) / (float)d + eps);
    if (t < t1) {
      T* dst = out + ((size_t)seq * S + t) * ld_out;
      T* keep = tile + (size_t)(t - t0) * d;
#pragma unroll
      for (int i = 0; i < MAXV; ++i) {
        const int v = lane + i * 64;
        if (v < nvec) {
          float y[VEC];
#pragma unroll
          for (int e = 0; e < VEC; ++e) y[e] = (x[u][i][e] - mean) * rstd * gv[i][e] + bv[i][e];
          Vec16<T>::store(dst + v * VEC, y);
          Vec16<T>::store(keep + v * VEC, y);
        }
      }
    }
  }
  __syncthreads();
  float* po = partial + ((size_t)seq * n_chunks + chunk) * d;
  for (int c = threadIdx.x; c < d; c += kLnPoolThreads) {
    float total = 0.f;
    for (int r = 0; r < R; ++r) {
      float acc = 0.f;
      for (int t = t0 + r; t < t1; t += R) acc += Elem<T>::load(tile + (size_t)(t - t0) * d + c);
      total = r == 0 ? acc : total + acc;
    }
    po[c] = total;
  }
  if (chunk == 0 && threadIdx.x == 0) pooled_flags[seq] = 2;
}

template <typename T>
static llmc_status_t launch_ln(const void* in, const int32_t* in_rows, void* out, const int32_t* out_rows,
                               const void* gamma, const void* beta, float eps, int d, int S, const int32_t* count,
                               int max_seqs, hipStream_t st) {
  constexpr int VEC = Vec16<T>::N;
  const int nvec = d / VEC;
  const unsigned blocks = (unsigned)std::min((max_seqs * S + 3) / 4, 2 * kMaxGrid);
#define LN_CASE(MV)                                                                                     \
  {                                                                                                     \
    ProfScope ps_("layernorm_kernel", st);                                                              \
    LLMC_KERNEL_GGL((layernorm_kernel<T, MV>), dim3(blocks), dim3(256), 0, st, (const T*)in, d,      \
                       in_rows, (T*)out, d, out_rows, (const T*)gamma, (const T*)beta, eps, d, S, count, \
                       max_seqs);                                                                       \
  }
  if (nvec <= 64) LN_CASE(1)
  else if (nvec <= 128) LN_CASE(2)
  else if (nvec <= 256) LN_CASE(4)
  else if (nvec <= 512) LN_CASE(8)
  else return set_error(LLMC_ERR_SHAPE, "LayerNorm width %d too large", d);
#undef LN_CASE
  LLMC_LAUNCH_CHECK("layernorm");
  return LLMC_OK;
}

// the fused form needs the chunk's outputs in LDS; wider rows take the plain kernel and the next call pools them
template <typename T>
static bool ln_pool_fits(int d) { return (size_t)kLnPoolChunk * d * sizeof(T) <= 128 * 1024 && d / Vec16<T>::N <= 128; }

template <typename T>
static llmc_status_t launch_ln_pool(const void* in, void* out, const int32_t* out_rows, const void* gamma,
                                    const void* beta, float eps, int d, int S, const int32_t* count, int max_seqs,
                                    float* partial, uint8_t* pooled_flags, hipStream_t st) {
  constexpr int VEC = Vec16<T>::N;
  const int nvec = d / VEC;
  const int G = d / VEC;
  const int R = std::max(1, std::min(8, 1024 / G));        // the pooling kernel's row groups for this width
  const int n_chunks = (S + kLnPoolChunk - 1) / kLnPoolChunk;
  const size_t lds = (size_t)kLnPoolChunk * d * sizeof(T);
  dim3 grid(n_chunks, max_seqs);
#define LNP_CASE(MV)                                                                                            \
  {                                                                                                             \
    static std::atomic<bool> lds_set[64];                                                                       \
    LLMC_TRY(ensure_dynamic_lds((const void*)(layernorm_pool_kernel<T, MV>), lds, lds_set));                    \
    ProfScope ps_("layernorm_kernel", st);                                                                      \
    LLMC_KERNEL_GGL((layernorm_pool_kernel<T, MV>), grid, dim3(kLnPoolThreads), lds, st, (const T*)in, d, (T*)out, \
                    d, out_rows, (const T*)gamma, (const T*)beta, eps, d, S, count, max_seqs, partial, n_chunks, R,  \
                    pooled_flags);                                                                              \
  }
  if (nvec <= 64) LNP_CASE(1)
  else LNP_CASE(2)
#undef LNP_CASE
  LLMC_LAUNCH_CHECK("layernorm_pool");
  return LLMC_OK;
}

// ---- attention: one thread per query row, online softmax over 32-key tiles ------------------------
// qkv [T, 3d] compact; ctx [T, d] compact.  grid (ceil(S / 128), heads, max_seqs).
template <typename T, bool CAUSAL>
__global__ __launch_bounds__(128) void attention_kernel(const T* __restrict__ qkv, T* __restrict__ ctx, int S, int d,
                                                        float scale, const int32_t* count, int max_seqs) {
  constexpr int DH = 64, KT = 32, VEC = Vec16<T>::N;
  __shared__ __attribute__((aligned(16))) float sK[KT][DH];
  __shared__ __attribute__((aligned(16))) float sV[KT][DH];
  const int n_seq = count ? min(*count, max_seqs) : max_seqs;
  const int seq = blockIdx.z;
  if (seq >= n_seq) return;
  const int head = blockIdx.y;
  const int q0 = blockIdx.x * 128;
  const int qi = q0 + threadIdx.x;
  const int qrow = min(qi, S - 1);
  const size_t ld = 3 * (size_t)d;
  const T* base = qkv + (size_t)seq * S * ld + head * DH;
  float q[DH], o[DH];
#pragma unroll
  for (int c = 0; c < DH; c += VEC) Vec16<T>::load(base + (size_t)qrow * ld + c, &q[c]);
#pragma unroll
  for (int c = 0; c < DH; ++c) o[c] = 0.f;
  float m = -INFINITY, l = 0.f;
  const int kv_end = CAUSAL ? min(S, q0 + 128) : S;
  for (int k0 = 0; k0 < kv_end; k0 += KT) {
    __syncthreads();
    for (int v = threadIdx.x; v < KT * DH / VEC; v += 128) {
      const int j = v / (DH / VEC), c = (v % (DH / VEC)) * VEC;
      const int kr = min(k0 + j, S - 1);
      Vec16<T>::load(base + (size_t)kr * ld + d + c, &sK[j][c]);
      Vec16<T>::load(base + (size_t)kr * ld + 2 * d + c, &sV[j][c]);
    }
    __syncthreads();
    float s[KT];
    float tmax = -INFINITY;
#pragma unroll
    for (int j = 0; j < KT; ++j) {
      float a = 0.f;
#pragma unroll
      for (int c = 0; c < DH; ++c) a = fmaf(q[c], sK[j][c], a);
      a *= scale;
      const int kv = k0 + j;
      if (kv >= S || (CAUSAL && kv > qrow)) a = -INFINITY;
      s[j] = a;
      tmax = fmaxf(tmax, a);
    }
    const float m_new = fmaxf(m, tmax);
    if (m_new == -INFINITY) continue;   // nothing visible yet in this tile (cannot happen for kv 0)
    const float corr = __expf(m - m_new);
    l *= corr;
#pragma unroll
    for (int c = 0; c < DH; ++c) o[c] *= corr;
#pragma unroll
    for (int j = 0; j < KT; ++j) {
      const float p = __expf(s[j] - m_new);
      l += p;
#pragma unroll
      for (int c = 0; c < DH; ++c) o[c] = fmaf(p, sV[j][c], o[c]);
    }
    m = m_new;
  }
  if (qi < S) {
    const float inv = 1.0f / l;
    T* dst = ctx + ((size_t)seq * S + qi) * d + head * DH;
#pragma unroll
    for (int c = 0; c < DH; c += VEC) {
      float y[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) y[e] = o[c + e] * inv;
      Vec16<T>::store(dst + c, y);
    }
  }
}

template <typename T>
static llmc_status_t launch_attention(const void* qkv, void* ctx, int S, int d, int n_heads, bool causal,
                                      const int32_t* count, int max_seqs, hipStream_t st) {
  const float scale = 1.0f / sqrtf((float)(d / n_heads));
  if (sizeof(T) == 2) return launch_attention_bf16(qkv, ctx, S, d, n_heads, causal, count, max_seqs, st);
  {
    dim3 grid((S + 127) / 128, n_heads, max_seqs);
    ProfScope ps_("attention_kernel", st);
    if (causal)
      LLMC_KERNEL_GGL((attention_kernel<T, true>), grid, dim3(128), 0, st, (const T*)qkv, (T*)ctx, S, d, scale, count,
                         max_seqs);
    else
      LLMC_KERNEL_GGL((attention_kernel<T, false>), grid, dim3(128), 0, st, (const T*)qkv, (T*)ctx, S, d, scale,
                         count, max_seqs);
  }
  LLMC_LAUNCH_CHECK("attention");
  return LLMC_OK;
}

// ---- the block -----------------------------------------------------------------------------------
size_t layer_ws_bytes(const llmc_layer_desc_t* L, int B, int S) {
  const size_t T = (size_t)B * S, e = elem_size(L->dtype);
  return align_up(T * 3 * L->d * e, 256) + 3 * align_up(T * L->d * e, 256) + align_up(T * L->d_ff * e, 256);
}

template <typename T>
static llmc_status_t layer_t(const llmc_layer_desc_t* L, const void* h_in, void* h_out, int B, int S,
                             const int32_t* rows, const int32_t* count, void* ws, hipStream_t st,
                             float* pool_partial, uint8_t* pooled_flags) {
  const int d = L->d, dff = L->d_ff;
  const size_t Tn = (size_t)B * S, e = sizeof(T);
  char* p = (char*)ws;
  void* qkv = p; p += align_up(Tn * 3 * d * e, 256);
  void* ctx = p; p += align_up(Tn * d * e, 256);
  void* t0 = p;  p += align_up(Tn * d * e, 256);
  void* t1 = p;  p += align_up(Tn * d * e, 256);
  void* ff = p;
  const int act = L->gelu == 0 ? 1 : 2;
  GemmArgs g{};
  g.S = S; g.count = count; g.max_seqs = B;
  auto gemm = [&](const void* A, int lda, const int32_t* a_rows, const void* W, const void* bias, int N, int K,
                  int act_, const void* resid, const int32_t* r_rows, void* out, const int32_t* o_rows) {
    GemmArgs a = g;
    a.A = A; a.lda = lda; a.a_rows = a_rows; a.W = W; a.bias = bias; a.N = N; a.K = K; a.act = act_;
    a.resid = resid; a.ldr = N; a.r_rows = r_rows; a.out = out; a.ldo = N; a.o_rows = o_rows;
    return launch_gemm(a, L->dtype, st);
  };
  if (L->arch == 0) {
    LLMC_TRY(gemm(h_in, d, rows, L->d_wqkv, L->d_bqkv, 3 * d, d, 0, nullptr, nullptr, qkv, nullptr));
    LLMC_TRY(launch_attention<T>(qkv, ctx, S, d, L->n_heads, false, count, B, st));
    LLMC_TRY(gemm(ctx, d, nullptr, L->d_wo, L->d_bo, d, d, 0, h_in, rows, t0, nullptr));
    LLMC_TRY(launch_ln<T>(t0, nullptr, t1, nullptr, L->d_ln1_g, L->d_ln1_b, L->ln_eps, d, S, count, B, st));
    LLMC_TRY(gemm(t1, d, nullptr, L->d_w1, L->d_b1, dff, d, act, nullptr, nullptr, ff, nullptr));
    LLMC_TRY(gemm(ff, dff, nullptr, L->d_w2, L->d_b2, d, dff, 0, t1, nullptr, t0, nullptr));
    if (pool_partial && pooled_flags && ln_pool_fits<T>(d))
      LLMC_TRY(launch_ln_pool<T>(t0, h_out, rows, L->d_ln2_g, L->d_ln2_b, L->ln_eps, d, S, count, B, pool_partial,
                                 pooled_flags, st));
    else
      LLMC_TRY(launch_ln<T>(t0, nullptr, h_out, rows, L->d_ln2_g, L->d_ln2_b, L->ln_eps, d, S, count, B, st));
  } else {
    LLMC_TRY(launch_ln<T>(h_in, rows, t1, nullptr, L->d_ln1_g, L->d_ln1_b, L->ln_eps, d, S, count, B, st));
    LLMC_TRY(gemm(t1, d, nullptr, L->d_wqkv, L->d_bqkv, 3 * d, d, 0, nullptr, nullptr, qkv, nullptr));
    LLMC_TRY(launch_attention<T>(qkv, ctx, S, d, L->n_heads, true, count, B, st));
    LLMC_TRY(gemm(ctx, d, nullptr, L->d_wo, L->d_bo, d, d, 0, h_in, rows, t0, nullptr));
    LLMC_TRY(launch_ln<T>(t0, nullptr, t1, nullptr, L->d_ln2_g, L->d_ln2_b, L->ln_eps, d, S, count, B, st));
    LLMC_TRY(gemm(t1, d, nullptr, L->d_w1, L->d_b1, dff, d, act, nullptr, nullptr, ff, nullptr));
    LLMC_TRY(gemm(ff, dff, nullptr, L->d_w2, L->d_b2, d, dff, 0, t0, nullptr, h_out, rows));
  }
  return LLMC_OK;
}

// ---- prefix attention statistics (Section IV-B): MHA over the first tokens of every sequence ----------------------
// out[b][t][:] = in[b][t][:] for t < n_prefix; one workgroup per token row, 16-byte vectors
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void prefix_copy_kernel(const u32x4_t* __restrict__ in, u32x4_t* __restrict__ out,
                                                          int S, int n_prefix, int vec_per_row) {
  const int b = blockIdx.x / n_prefix, t = blockIdx.x % n_prefix;
  const u32x4_t* src = in + ((size_t)b * S + t) * vec_per_row;
  u32x4_t* dst = out + (size_t)blockIdx.x * vec_per_row;
  for (int v = threadIdx.x; v < vec_per_row; v += 256) dst[v] = src[v];
}

size_t prefix_attention_ws_bytes(const llmc_layer_desc_t* L, int B, int n_prefix) {
  const size_t T = (size_t)B * n_prefix, e = elem_size(L->dtype);
  return align_up(T * 3 * L->d * e, 256) + 3 * align_up(T * L->d * e, 256);
}

template <typename T>
static llmc_status_t prefix_attention_t(const llmc_layer_desc_t* L, const void* h, int B, int S, int n_p, void* ws,
                                        float* out, int ld_out, hipStream_t st) {
  const int d = L->d;
  const size_t Tn = (size_t)B * n_p, e = sizeof(T);
  char* p = (char*)ws;
  void* qkv = p; p += align_up(Tn * 3 * d * e, 256);
  void* x = p;   p += align_up(Tn * d * e, 256);
  void* ctx = p; p += align_up(Tn * d * e, 256);
  void* ao = p;
  { ProfScope ps_("prefix_copy_kernel", st);
    LLMC_KERNEL_GGL(prefix_copy_kernel, dim3((unsigned)Tn), dim3(256), 0, st, (const u32x4_t*)h, (u32x4_t*)x, S, n_p,
                    (int)((size_t)d * e / 16)); }
  LLMC_LAUNCH_CHECK("prefix_copy_kernel");
  const void* a_in = x;
  if (L->arch == 1) {       // the pre-LayerNorm block attends over LN1(x)
    LLMC_TRY(launch_ln<T>(x, nullptr, ctx, nullptr, L->d_ln1_g, L->d_ln1_b, L->ln_eps, d, n_p, nullptr, B, st));
    a_in = ctx;
  }
  GemmArgs g{};
  g.S = n_p; g.count = nullptr; g.max_seqs = B; g.act = 0; g.resid = nullptr; g.r_rows = nullptr; g.a_rows = nullptr;
  g.o_rows = nullptr;
  GemmArgs a = g;
  a.A = a_in; a.lda = d; a.W = L->d_wqkv; a.bias = L->d_bqkv; a.N = 3 * d; a.K = d; a.ldr = 3 * d; a.out = qkv; a.ldo = 3 * d;
  LLMC_TRY(launch_gemm(a, L->dtype, st));
  void* ctx2 = L->arch == 1 ? x : ctx;        // LN1's output has been consumed by the projection above
  LLMC_TRY(launch_attention<T>(qkv, ctx2, n_p, d, L->n_heads, L->arch == 1, nullptr, B, st));
  a = g;
  a.A = ctx2; a.lda = d; a.W = L->d_wo; a.bias = L->d_bo; a.N = d; a.K = d; a.ldr = d; a.out = ao; a.ldo = d;
  LLMC_TRY(launch_gemm(a, L->dtype, st));
  return launch_pool_rows(ao, B, n_p, d, L->dtype, nullptr, nullptr, nullptr, out, st, ld_out);
}

llmc_status_t launch_prefix_attention_mean(const llmc_layer_desc_t* L, const void* d_h, int B, int S, int n_prefix,
                                           void* ws, float* d_out, int ld_out, hipStream_t st) {
  if (L->dtype == LLMC_F32) return prefix_attention_t<float>(L, d_h, B, S, n_prefix, ws, d_out, ld_out, st);
  return prefix_attention_t<bf16_t>(L, d_h, B, S, n_prefix, ws, d_out, ld_out, st);
}

llmc_status_t launch_linear(const void* A, int lda, const int32_t* a_rows, const void* W, const void* bias, int N, int K,
                            void* out, int ldo, const int32_t* o_rows, int S, const int32_t* count, int max_seqs,
                            int dtype, hipStream_t st) {
  GemmArgs a{};
  a.A = A; a.lda = lda; a.a_rows = a_rows; a.W = W; a.bias = bias; a.N = N; a.K = K; a.act = 0;
  a.resid = nullptr; a.ldr = N; a.r_rows = nullptr; a.out = out; a.ldo = ldo; a.o_rows = o_rows;
  a.S = S; a.count = count; a.max_seqs = max_seqs;
  return launch_gemm(a, dtype, st);
}

llmc_status_t launch_layer(const llmc_layer_desc_t* L, const void* d_h_in, void* d_h_out, int B, int S,
                           const int32_t* d_rows, const int32_t* d_count, void* ws, hipStream_t st,
                           float* pool_partial, uint8_t* pooled_flags) {
  if (L->dtype == LLMC_F32)
    return layer_t<float>(L, d_h_in, d_h_out, B, S, d_rows, d_count, ws, st, pool_partial, pooled_flags);
  return layer_t<bf16_t>(L, d_h_in, d_h_out, B, S, d_rows, d_count, ws, st, pool_partial, pooled_flags);
}

}  // namespace llmc
