// Bank match (Section III-C of the paper; the "exists an entry with sim > tau" test of
// Section IV-A and Algorithm 1 is a maximum over the bank): for each query key the valid
// entry of largest cosine similarity.
//
// Stage 1 (bulk): scores^T = bank * queries^T on the bf16 matrix cores.  Bank rows are the
// M side of the instruction, so a lane holds ONE query column and 16 bank rows per 32x32
// fragment: the running maximum is a per-lane register operation with no cross-lane
// traffic, and the score matrix is never written.  A lane does not track single rows but
// "groups": the 16 bank rows of one fragment half, numbered  (row_base / 32) * 2 + half.
// It keeps its two best groups (value = max over the group of acc * inv_norm).
// Free slots carry NaN in the library's inv_norm mirror and fmaxf drops them.
//
// Stage 2 (exact): one wavefront per query merges the partial results of all bank
// splits, then evaluates the rows of the best group -- and of the runner-up group when it
// is within 1e-5 of the best -- in fp64 and picks the winner there (lowest slot on exact
// ties).  The reported similarity is that fp64 cosine.
#include "common.h"
#include "mma.h"

namespace llmc {

struct Top2 {
  float v1; int g1;
  float v2; int g2;
};

__device__ __forceinline__ bool better(float v, int g, float v0, int g0) {
  return v > v0 || (v == v0 && g >= 0 && (g0 < 0 || g < g0));
}
__device__ __forceinline__ void top2_push(Top2& t, float v, int g) {
  if (g < 0) return;
  if (better(v, g, t.v1, t.g1)) {
    t.v2 = t.v1; t.g2 = t.g1; t.v1 = v; t.g1 = g;
  } else if (better(v, g, t.v2, t.g2) && g != t.g1) {
    t.v2 = v; t.g2 = g;
  }
}
__device__ __forceinline__ Top2 top2_empty() { return Top2{-INFINITY, -1, -INFINITY, -1}; }

// rows of group g: base = (g / 2) * 32 + (g % 2) * 4;  row(r) = base + 8 * (r / 4) + (r % 4), r = 0..15
__device__ __forceinline__ int group_row(int g, int r) { return (g >> 1) * 32 + (g & 1) * 4 + 8 * (r >> 2) + (r & 3); }

typedef MmaCfg<128, 128, 32, 2, 2> MatchCfg;

// grid (n_split, query_blocks)
__global__ __launch_bounds__(MatchCfg::THREADS) void match_bf16_kernel(
    const uint16_t* __restrict__ bank, const float* __restrict__ binv_eff, int N, int K,
    const uint16_t* __restrict__ queries, int B, int tiles_per_split, Top2* __restrict__ partial) {
  using C = MatchCfg;
  __shared__ __attribute__((aligned(16))) uint16_t lds[C::LDS_BYTES / 2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int q0 = blockIdx.y * C::BN;
  const int n_tiles = (N + C::BM - 1) / C::BM;
  const int t_begin = blockIdx.x * tiles_per_split;
  const int t_end = min(n_tiles, t_begin + tiles_per_split);

  const uint16_t* b_ptr[C::NLOAD_B];
#pragma unroll
  for (int i = 0; i < C::NLOAD_B; ++i) {
    const int v = tid + i * C::THREADS;
    const int r = min(q0 + v / C::VEC_PER_ROW, B - 1);
    b_ptr[i] = queries + (size_t)r * K + (v % C::VEC_PER_ROW) * 8;
  }
  Top2 best[C::FN];
#pragma unroll
  for (int j = 0; j < C::FN; ++j) best[j] = top2_empty();

  for (int t = t_begin; t < t_end; ++t) {
    const int m0 = t * C::BM;
    const uint16_t* a_ptr[C::NLOAD_A];
#pragma unroll
    for (int i = 0; i < C::NLOAD_A; ++i) {
      const int v = tid + i * C::THREADS;
      const int r = min(m0 + v / C::VEC_PER_ROW, N - 1);
      a_ptr[i] = bank + (size_t)r * K + (v % C::VEC_PER_ROW) * 8;
    }
    f32x16_t acc[C::FM][C::FN];
#pragma unroll
    for (int i = 0; i < C::FM; ++i)
#pragma unroll
      for (int j = 0; j < C::FN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    mma_block<C>(a_ptr, b_ptr, K, lds, acc);
#pragma unroll
    for (int i = 0; i < C::FM; ++i) {
      const int rb = m0 + wm * (C::BM / C::WM) + i * 32;     // fragment's first bank row (multiple of 32)
      const int g = (rb >> 5) * 2 + (lane >> 5);
      float bi[16];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        // binv_eff is padded with NaN up to a multiple of the tile height
        const float4 v4 = *reinterpret_cast<const float4*>(binv_eff + rb + (lane >> 5) * 4 + 8 * c);
        bi[4 * c] = v4.x; bi[4 * c + 1] = v4.y; bi[4 * c + 2] = v4.z; bi[4 * c + 3] = v4.w;
      }
#pragma unroll
      for (int j = 0; j < C::FN; ++j) {
        float mx = acc[i][j][0] * bi[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, acc[i][j][r] * bi[r]);
        // tiles ascend, so a strict comparison keeps the lowest group among equals
        if (mx > best[j].v1) {
          best[j].v2 = best[j].v1; best[j].g2 = best[j].g1; best[j].v1 = mx; best[j].g1 = g;
        } else if (mx > best[j].v2) {
          best[j].v2 = mx; best[j].g2 = g;
        }
      }
    }
  }
  // merge the 2 lane halves x WM waves that saw the same query column
  __syncthreads();
  Top2* sc = reinterpret_cast<Top2*>(lds);   // [WM * 2][BN]
#pragma unroll
  for (int j = 0; j < C::FN; ++j) {
    const int col = wn * (C::BN / C::WN) + j * 32 + (lane & 31);
    sc[(wm * 2 + (lane >> 5)) * C::BN + col] = best[j];
  }
  __syncthreads();
  if (tid < C::BN && q0 + tid < B) {
    Top2 t = top2_empty();
    for (int s = 0; s < C::WM * 2; ++s) {
      const Top2 c = sc[s * C::BN + tid];
      top2_push(t, c.v1, c.g1);
      top2_push(t, c.v2, c.g2);
    }
    partial[(size_t)blockIdx.x * B + q0 + tid] = t;
  }
}

// fp32 keys: plain FMA.  grid (B); thread t scans groups t, t + 256, ...
__global__ __launch_bounds__(256) void match_f32_kernel(const float* __restrict__ bank,
                                                        const float* __restrict__ binv_eff, int N, int K,
                                                        const float* __restrict__ queries, Top2* __restrict__ partial) {
  extern __shared__ float sq[];    // [K] query, then Top2[256]
  const int b = blockIdx.x;
  for (int i = threadIdx.x; i < K; i += 256) sq[i] = queries[(size_t)b * K + i];
  __syncthreads();
  const int n_groups = ((N + 31) / 32) * 2;
  Top2 t = top2_empty();
  for (int g = threadIdx.x; g < n_groups; g += 256) {
    float mx = NAN;
    for (int r = 0; r < 16; ++r) {
      const int row = group_row(g, r);
      if (row >= N) continue;
      const float* kp = bank + (size_t)row * K;
      float a = 0.f;
      for (int i = 0; i < K; ++i) a = fmaf(sq[i], kp[i], a);
      mx = fmaxf(mx, a * binv_eff[row]);
    }
    top2_push(t, mx, g);
  }
  Top2* sc = reinterpret_cast<Top2*>(sq + K);
  sc[threadIdx.x] = t;
  __syncthreads();
  if (threadIdx.x == 0) {
    Top2 m = top2_empty();
    for (int i = 0; i < 256; ++i) {
      top2_push(m, sc[i].v1, sc[i].g1);
      top2_push(m, sc[i].v2, sc[i].g2);
    }
    partial[b] = m;
  }
}

// one wavefront per query
template <typename T>
__global__ __launch_bounds__(256) void match_finalize_kernel(
    const Top2* __restrict__ partial, int n_split, const T* __restrict__ bank, const float* __restrict__ binv,
    const uint8_t* __restrict__ valid, int N, int K, const T* __restrict__ queries, const float* __restrict__ qinv,
    int B, float tau, int32_t* __restrict__ idx_out, float* __restrict__ sim_out, uint8_t* __restrict__ hit_out,
    uint8_t* __restrict__ tie_out) {
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (b >= B) return;
  const int lane = threadIdx.x & 63;
  Top2 t = top2_empty();
  for (int s = lane; s < n_split; s += 64) {
    const Top2 c = partial[(size_t)s * B + b];
    top2_push(t, c.v1, c.g1);
    top2_push(t, c.v2, c.g2);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    Top2 c;
    c.v1 = __shfl_xor(t.v1, o, 64); c.g1 = __shfl_xor(t.g1, o, 64);
    c.v2 = __shfl_xor(t.v2, o, 64); c.g2 = __shfl_xor(t.g2, o, 64);
    top2_push(t, c.v1, c.g1);
    top2_push(t, c.v2, c.g2);
  }
  const float qi = qinv[b];
  const double qi64 = (double)qi;
  // scores so far are |q| * cos; the runner-up counts as tied within 1e-5 in cosine
  const float gap = qi > 0.f ? 1e-5f / qi : 0.f;
  const bool two = t.g2 >= 0 && t.v2 >= t.v1 - gap;
  double best = -INFINITY;
  int best_j = -1;
  const int n_groups = (t.g1 < 0) ? 0 : (two ? 2 : 1);
  for (int c = 0; c < n_groups; ++c) {
    const int g = c == 0 ? t.g1 : t.g2;
    for (int r = 0; r < 16; ++r) {
      const int j = group_row(g, r);
      if (j >= N || !valid[j]) continue;   // uniform across the wavefront
      double a = 0.0;
      for (int i = lane; i < K; i += 64)
        a += (double)Elem<T>::load(queries + (size_t)b * K + i) * (double)Elem<T>::load(bank + (size_t)j * K + i);
      a = wave_sum(a);
      const double s = a * qi64 * (double)binv[j];
      if (s > best || (s == best && j < best_j)) { best = s; best_j = j; }
    }
  }
  if (lane == 0) {
    idx_out[b] = best_j;
    if (sim_out) sim_out[b] = (float)best;
    if (hit_out) hit_out[b] = (best_j >= 0 && best > (double)tau) ? 1 : 0;
    if (tie_out) tie_out[b] = two ? 1 : 0;
  }
}

static void split_plan(int N, int B, int* n_split, int* tiles_per_split) {
  const int tiles = (N + MatchCfg::BM - 1) / MatchCfg::BM;
  const int qb = (B + MatchCfg::BN - 1) / MatchCfg::BN;
  int want = (1024 + qb - 1) / qb;
  if (want > tiles) want = tiles;
  if (want < 1) want = 1;
  const int per = (tiles + want - 1) / want;
  *tiles_per_split = per;
  *n_split = (tiles + per - 1) / per;
}

size_t match_ws_bytes(int n_slots, int k, int dtype, int B) {
  (void)k;
  int ns = 1, per = 1;
  if (dtype == LLMC_BF16) split_plan(n_slots, B, &ns, &per);
  return align_up((size_t)ns * B * sizeof(Top2), 256);
}

llmc_status_t launch_match(const llmc_bank* bank, const void* d_fp, const float* d_inv, int B, float tau,
                           int32_t* d_idx, float* d_sim, uint8_t* d_hit, uint8_t* d_near_tie, void* ws,
                           hipStream_t st) {
  const llmc_bank_desc_t& D = bank->desc;
  const int N = D.n_slots, K = D.k;
  Top2* partial = (Top2*)ws;
  int ns = 1, per = 1;
  if (D.dtype == LLMC_BF16) {
    split_plan(N, B, &ns, &per);
    dim3 grid(ns, (B + MatchCfg::BN - 1) / MatchCfg::BN);
    { ProfScope ps_("match_bf16_kernel", st); hipLaunchKernelGGL(match_bf16_kernel, grid, dim3(MatchCfg::THREADS), 0, st, (const uint16_t*)D.d_fp,
                       bank->d_binv_eff, N, K, (const uint16_t*)d_fp, B, per, partial); }
    LLMC_LAUNCH_CHECK("match_bf16_kernel");
    { ProfScope ps_("match_finalize_kernel", st); hipLaunchKernelGGL((match_finalize_kernel<bf16_t>), dim3((B + 3) / 4), dim3(256), 0, st, partial, ns,
                       (const bf16_t*)D.d_fp, D.d_inv_norm, D.d_valid, N, K, (const bf16_t*)d_fp, d_inv, B, tau, d_idx,
                       d_sim, d_hit, d_near_tie); }
  } else {
    { ProfScope ps_("match_f32_kernel", st); hipLaunchKernelGGL(match_f32_kernel, dim3(B), dim3(256), (size_t)K * sizeof(float) + 256 * sizeof(Top2), st,
                       (const float*)D.d_fp, bank->d_binv_eff, N, K, (const float*)d_fp, partial); }
    LLMC_LAUNCH_CHECK("match_f32_kernel");
    { ProfScope ps_("match_finalize_kernel", st); hipLaunchKernelGGL((match_finalize_kernel<float>), dim3((B + 3) / 4), dim3(256), 0, st, partial, 1,
                       (const float*)D.d_fp, D.d_inv_norm, D.d_valid, N, K, (const float*)d_fp, d_inv, B, tau, d_idx,
                       d_sim, d_hit, d_near_tie); }
  }
  LLMC_LAUNCH_CHECK("match_finalize_kernel");
  return LLMC_OK;
}

}  // namespace llmc
