// Bank match (Section III-C of the paper; the "exists an entry with sim > tau" test of
// Section IV-A and Algorithm 1 is a maximum over the bank): for each query key the valid
// entry of largest cosine similarity.
//
// Stage 1 (bulk): scores^T = bank * queries^T on the bf16 matrix cores.  Bank rows are the
// M side of the instruction, so a lane holds ONE query column and 16 bank rows per 32x32
// fragment: the running maximum is a per-lane register operation with no cross-lane
// traffic, and the score matrix is never written.  A lane does not track single rows but
// "groups": the 16 bank rows of one fragment half, numbered  (row_base / 32) * 2 + half.
// It keeps its two best groups (value = max over the group of acc * inv_norm) and the VALUE of
// the third best.  Free slots carry NaN in the library's inv_norm mirror and fmaxf drops them.
//
// Stage 2 (exact): one wavefront per query merges the partial results of all bank
// splits, then evaluates the rows of the best group -- and of the runner-up group when it
// is within 1e-5 of the best -- in fp64 and picks the winner there (lowest slot on exact
// ties).  The reported similarity is that fp64 cosine.  If the third best value is within
// 1e-5 of the best as well (three or more groups that fp32 cannot tell apart: several
// near-identical keys spread over the bank), the two kept groups may not hold the exact
// arg-max; the slot returned is then the best of those two groups, within that margin of the
// true maximum, and the row is flagged (near-tie flag 2, counted separately) so that it is
// reported rather than silently wrong.
#include "common.h"
#include "mma.h"

namespace llmc {

struct Top2 {
  float v1; int g1;
  float v2; int g2;
  float v3;            // third best value (its group is not kept)
};

__device__ __forceinline__ bool better(float v, int g, float v0, int g0) {
  return v > v0 || (v == v0 && g >= 0 && (g0 < 0 || g < g0));
}
__device__ __forceinline__ void top2_push(Top2& t, float v, int g) {
  if (g < 0) return;
  if (better(v, g, t.v1, t.g1)) {
    t.v3 = t.v2; t.v2 = t.v1; t.g2 = t.g1; t.v1 = v; t.g1 = g;
  } else if (g != t.g1) {
    if (better(v, g, t.v2, t.g2)) {
      t.v3 = t.v2; t.v2 = v; t.g2 = g;
    } else if (g != t.g2) {
      t.v3 = fmaxf(t.v3, v);
    }
  }
}
// merge another list's entries (its two groups, then its third value) into t
__device__ __forceinline__ void top2_merge(Top2& t, const Top2& c) {
  top2_push(t, c.v1, c.g1);
  top2_push(t, c.v2, c.g2);
  t.v3 = fmaxf(t.v3, c.v3);
}
__device__ __forceinline__ Top2 top2_empty() { return Top2{-INFINITY, -1, -INFINITY, -1, -INFINITY}; }
// one more group maximum in a stream of ascending groups (strict comparisons keep the lowest group among equals)
__device__ __forceinline__ void top2_next(Top2& t, float mx, int g) {
  const bool b1 = mx > t.v1, b2 = mx > t.v2;                        // NaN compares false
  const float v3n = b2 ? t.v2 : fmaxf(t.v3, mx);                    // fmaxf drops a NaN maximum
  const float v2n = b1 ? t.v1 : (b2 ? mx : t.v2);
  const int g2n = b1 ? t.g1 : (b2 ? g : t.g2);
  t.v1 = b1 ? mx : t.v1;
  t.g1 = b1 ? g : t.g1;
  t.v2 = v2n;
  t.g2 = g2n;
  t.v3 = v3n;
}

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
        top2_next(best[j], mx, g);
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
    for (int s = 0; s < C::WM * 2; ++s) top2_merge(t, sc[s * C::BN + tid]);
    partial[(size_t)blockIdx.x * B + q0 + tid] = t;
  }
}

// ---- streaming variant: queries stay in registers, the bank streams through LDS ------------------
// A workgroup of 8 wavefronts owns 512 query columns (64 per wavefront, held as B-operand
// fragments in registers for the whole kernel) and walks a range of 64-row bank tiles.  Tiles
// arrive by direct global -> LDS loads into a ring of stages; all wavefronts read the same
// bank fragments from LDS, so LDS traffic is one tile read per wavefront and no query is ever
// re-fetched.  Rows of a tile are 2*K bytes; their 16-byte chunks are XOR-swizzled by the row
// number so that the 16-byte fragment reads of 16 consecutive rows fall on distinct banks.
template <int K_, int NW_>
struct StreamCfg {
  static constexpr int K = K_, KS = K / 16, CHUNKS = K / 8, ROWB = K * 2;
  static constexpr int NW = NW_, THREADS = NW * 64, FM = 2, FN = 2;
  static constexpr int RB = FM * 32;                 // bank rows per tile
  static constexpr int QW = FN * 32, QB = NW * QW;   // queries per wavefront / workgroup
  static constexpr int ROWS_PER_INSTR = 1024 / ROWB; // tile rows filled by one wavefront load
  static constexpr int L = RB / ROWS_PER_INSTR / NW + 1;   // loads per lane per stage: tile blocks + the norms
  static constexpr int TILE_ELEMS = RB * K;
  static constexpr int STAGE_ELEMS = TILE_ELEMS + NW * RB * 2;   // + one fp32 copy of the tile's inverse norms per wavefront
  // 8 wavefronts: one workgroup per compute unit with a deep ring; 4 wavefronts: two independent
  // workgroups per compute unit (their epilogues and main loops interleave), two stages each
  static constexpr int STAGES = NW == 8 ? ((K >= 256) ? 4 : 3) : 2;
  static constexpr size_t LDS_BYTES = (size_t)STAGES * STAGE_ELEMS * 2;
  static_assert(K == 64 || K == 128 || K == 256, "supported key lengths");
  static_assert(L >= 2 && (RB / ROWS_PER_INSTR) % NW == 0 && RB == 64, "load tiling");
  __device__ static __forceinline__ int swz(int row) { return ROWB >= 256 ? (row & 15) : ((row >> 1) & 7); }
};

// grid: 1-D, see launch_match for the workgroup -> (split, query block) map
template <int K_, int NW_>
__global__ __launch_bounds__(NW_ * 64) void match_stream_kernel(
    const uint16_t* __restrict__ bank, const float* __restrict__ binv_eff, int N, const uint16_t* __restrict__ queries,
    int B, int n_qb, int n_split, int tiles_per_split, Top2* __restrict__ partial) {
  using C = StreamCfg<K_, NW_>;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_dyn[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // workgroups are dealt round-robin to the 8 XCDs: keep the query blocks of one bank split on
  // one XCD and adjacent in time, so that its L2 serves the bank tiles to all of them
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int split = (local / n_qb) * 8 + xcd, qb = local % n_qb;
  if (split >= n_split) return;
  const int n_tiles = (N + C::RB - 1) / C::RB;
  const int t_begin = split * tiles_per_split;
  const int t_end = min(n_tiles, t_begin + tiles_per_split);
  const int q_base = qb * C::QB + wave * C::QW;

  // this lane's part of every load of a stage: tile row and (swizzled) chunk
  int ld_row[C::L - 1], ld_off[C::L - 1];
#pragma unroll
  for (int j = 0; j < C::L - 1; ++j) {
    const int blk = j * C::NW + wave;                       // 1 KiB block of the stage
    const int row = blk * C::ROWS_PER_INSTR + lane / C::CHUNKS;
    ld_row[j] = row;
    ld_off[j] = ((lane % C::CHUNKS) ^ C::swz(row)) * 8;
  }
  auto issue = [&](int t) {
    uint16_t* st = lds_dyn + ((t - t_begin) % C::STAGES) * C::STAGE_ELEMS;
#pragma unroll
    for (int j = 0; j < C::L - 1; ++j) {
      const int r = min(t * C::RB + ld_row[j], N - 1);
      __builtin_amdgcn_global_load_lds(LLMC_GPTR(bank + (size_t)r * C::K + ld_off[j]),
                                       LLMC_LPTR(st + (j * C::NW + wave) * 512), 16, 0, 0);
    }
    // the tile's 64 inverse norms (the mirror is padded with NaN past N), one private copy per wavefront
    __builtin_amdgcn_global_load_lds(LLMC_GPTR(binv_eff + (size_t)t * C::RB + lane),
                                     LLMC_LPTR(st + C::TILE_ELEMS + wave * C::RB * 2), 4, 0, 0);
  };
#pragma unroll
  for (int s = 0; s < C::STAGES - 1; ++s)
    if (t_begin + s < t_end) issue(t_begin + s);

  // query fragments: column (lane % 32) of fragment j, k = ks * 16 + (lane / 32) * 8 .. + 8
  bf16x8_t bq[C::FN][C::KS];
#pragma unroll
  for (int j = 0; j < C::FN; ++j) {
    const int q = min(q_base + j * 32 + (lane & 31), B - 1);
    const uint16_t* qp = queries + (size_t)q * C::K + (lane >> 5) * 8;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) bq[j][ks] = *reinterpret_cast<const bf16x8_t*>(qp + ks * 16);
  }
  Top2 best[C::FN];
#pragma unroll
  for (int j = 0; j < C::FN; ++j) best[j] = top2_empty();
  const int frag_off = (lane & 31) * C::K;
  const int fsw = C::swz(lane & 31), half = lane >> 5;

  for (int t = t_begin; t < t_end; ++t) {
    const int ahead = min(C::STAGES - 2, t_end - 1 - t);
    if (ahead <= 0) LLMC_WAIT_VM(0);
    else if (ahead == 1) LLMC_WAIT_VM(C::L);
    else LLMC_WAIT_VM(2 * C::L);
    dma::barrier();
    if (t + C::STAGES - 1 < t_end) issue(t + C::STAGES - 1);
    const uint16_t* stage = lds_dyn + ((t - t_begin) % C::STAGES) * C::STAGE_ELEMS;
    const uint16_t* st = stage + frag_off;
    const float* sbinv = reinterpret_cast<const float*>(stage + C::TILE_ELEMS + wave * C::RB * 2);
    f32x16_t acc[C::FM][C::FN];
#pragma unroll
    for (int i = 0; i < C::FM; ++i)
#pragma unroll
      for (int j = 0; j < C::FN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    // bank fragments of step ks + 1 are fetched while step ks multiplies
    bf16x8_t fa[2][C::FM];
#pragma unroll
    for (int i = 0; i < C::FM; ++i)
      fa[0][i] = *reinterpret_cast<const bf16x8_t*>(st + i * 32 * C::K + ((half ^ fsw) * 8));
    __builtin_amdgcn_sched_group_barrier(0x100, C::FM, 0);
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
      const int c = ks & 1, n = c ^ 1;
      if (ks + 1 < C::KS) {
#pragma unroll
        for (int i = 0; i < C::FM; ++i)
          fa[n][i] = *reinterpret_cast<const bf16x8_t*>(st + i * 32 * C::K + ((((ks + 1) * 2 + half) ^ fsw) * 8));
      }
#pragma unroll
      for (int i = 0; i < C::FM; ++i)
#pragma unroll
        for (int j = 0; j < C::FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c][i], bq[j][ks], acc[i][j], 0, 0, 0);
      // keep the order written above: the next step's LDS reads first, then this step's MFMAs
      __builtin_amdgcn_sched_group_barrier(0x100, C::FM, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, C::FM * C::FN, 0);
    }
#pragma unroll
    for (int i = 0; i < C::FM; ++i) {
      const int rb = t * C::RB + i * 32;
      const int g = (rb >> 5) * 2 + half;
      float bi[16];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float4 v4 = *reinterpret_cast<const float4*>(sbinv + i * 32 + half * 4 + 8 * c);
        bi[4 * c] = v4.x; bi[4 * c + 1] = v4.y; bi[4 * c + 2] = v4.z; bi[4 * c + 3] = v4.w;
      }
#pragma unroll
      for (int j = 0; j < C::FN; ++j) {
        float mx = acc[i][j][0] * bi[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, acc[i][j][r] * bi[r]);
        top2_next(best[j], mx, g);
      }
    }
  }
  // the two lane halves saw different rows of the same query column
#pragma unroll
  for (int j = 0; j < C::FN; ++j) {
    Top2 o;
    o.v1 = __shfl_xor(best[j].v1, 32, 64); o.g1 = __shfl_xor(best[j].g1, 32, 64);
    o.v2 = __shfl_xor(best[j].v2, 32, 64); o.g2 = __shfl_xor(best[j].g2, 32, 64);
    o.v3 = __shfl_xor(best[j].v3, 32, 64);
    Top2 m = best[j];
    top2_merge(m, o);
    const int q = q_base + j * 32 + (lane & 31);
    if (half == 0 && q < B) partial[(size_t)split * B + q] = m;
  }
}

// ---- skewed streaming variant for many queries ----------------------------------------------------
// Same data flow as match_stream_kernel with 8 wavefronts (two per SIMD), but the two
// wavefronts of a SIMD run the tile loop one half step apart: after the barrier of tile t the
// "early" wavefront multiplies tile t and then reduces it, while the "late" wavefront first
// reduces tile t - 1 (held in its accumulators across the barrier) and then multiplies tile t.
// The vector-ALU reduction of one wavefront therefore runs while the other one owns the matrix
// pipe, instead of both alternating between the two in step.  A late wavefront still reads the
// inverse norms of tile t - 1 during tile t, so a ring stage is refilled two barriers after its
// tile.  Accumulators start as NaN, which the first reduction of a late wavefront drops.
template <int K_>
struct SkewCfg : StreamCfg<K_, 8> {
  using S = StreamCfg<K_, 8>;
  static constexpr int STAGES = 4;
  static constexpr size_t LDS_BYTES = (size_t)STAGES * S::STAGE_ELEMS * 2;
};

template <int K_>
__global__ __launch_bounds__(512) void match_skew_kernel(
    const uint16_t* __restrict__ bank, const float* __restrict__ binv_eff, int N, const uint16_t* __restrict__ queries,
    int B, int n_qb, int n_split, int tiles_per_split, Top2* __restrict__ partial) {
  using C = SkewCfg<K_>;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_dyn[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const bool late = wave >= C::NW / 2;      // wavefronts w and w + 4 share a SIMD
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int split = (local / n_qb) * 8 + xcd, qb = local % n_qb;
  if (split >= n_split) return;
  const int n_tiles = (N + C::RB - 1) / C::RB;
  const int t_begin = split * tiles_per_split;
  const int t_end = min(n_tiles, t_begin + tiles_per_split);
  const int q_base = qb * C::QB + wave * C::QW;

  // load j of a stage fills tile rows ld_row + j * JSTEP; JSTEP is a multiple of the swizzle period,
  // so the (swizzled) chunk of this lane is the same for every j
  constexpr int JSTEP = C::NW * C::ROWS_PER_INSTR;
  static_assert(JSTEP % 16 == 0, "one swizzled chunk per lane");
  const int ld_row = wave * C::ROWS_PER_INSTR + lane / C::CHUNKS;
  const int ld_off = ((lane % C::CHUNKS) ^ C::swz(ld_row)) * 8;
  auto issue = [&](int t) {
    uint16_t* st = lds_dyn + ((t - t_begin) % C::STAGES) * C::STAGE_ELEMS;
#pragma unroll
    for (int j = 0; j < C::L - 1; ++j) {
      const int r = min(t * C::RB + ld_row + j * JSTEP, N - 1);
      __builtin_amdgcn_global_load_lds(LLMC_GPTR(bank + (size_t)r * C::K + ld_off),
                                       LLMC_LPTR(st + (j * C::NW + wave) * 512), 16, 0, 0);
    }
    __builtin_amdgcn_global_load_lds(LLMC_GPTR(binv_eff + (size_t)t * C::RB + lane),
                                     LLMC_LPTR(st + C::TILE_ELEMS + wave * C::RB * 2), 4, 0, 0);
  };
#pragma unroll
  for (int s = 0; s < C::STAGES - 2; ++s)
    if (t_begin + s < t_end) issue(t_begin + s);

  bf16x8_t bq[C::FN][C::KS];
#pragma unroll
  for (int j = 0; j < C::FN; ++j) {
    const int q = min(q_base + j * 32 + (lane & 31), B - 1);
    const uint16_t* qp = queries + (size_t)q * C::K + (lane >> 5) * 8;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) bq[j][ks] = *reinterpret_cast<const bf16x8_t*>(qp + ks * 16);
  }
  Top2 best[C::FN];
#pragma unroll
  for (int j = 0; j < C::FN; ++j) best[j] = top2_empty();
  const int frag_off = (lane & 31) * C::K;
  const int fsw = C::swz(lane & 31), half = lane >> 5;

  f32x16_t acc[C::FM][C::FN];
#pragma unroll
  for (int i = 0; i < C::FM; ++i)
#pragma unroll
    for (int j = 0; j < C::FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = NAN;

  // running maximum over the accumulators of tile t, scaled by the inverse norms at sb; the maximum of a
  // fragment's 16 scores is a chain (the fourth product of each group of four is carried into the next link),
  // so that every link is one three-operand maximum
  auto reduce = [&](const float* sb, int t) {
#pragma unroll
    for (int i = 0; i < C::FM; ++i) {
      const int g = t * 4 + i * 2 + half;
      float m[C::FN], carry[C::FN];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float4 v4 = *reinterpret_cast<const float4*>(sb + i * 32 + half * 4 + 8 * c);
#pragma unroll
        for (int j = 0; j < C::FN; ++j) {
          const float p0 = acc[i][j][4 * c] * v4.x, p1 = acc[i][j][4 * c + 1] * v4.y;
          const float p2 = acc[i][j][4 * c + 2] * v4.z, p3 = acc[i][j][4 * c + 3] * v4.w;
          if (c == 0) {
            m[j] = fmaxf(fmaxf(p0, p1), p2);
          } else {
            m[j] = fmaxf(fmaxf(m[j], carry[j]), p0);
            m[j] = fmaxf(fmaxf(m[j], p1), p2);
          }
          carry[j] = p3;
        }
      }
#pragma unroll
      for (int j = 0; j < C::FN; ++j) {
        top2_next(best[j], fmaxf(m[j], carry[j]), g);
      }
    }
  };

  for (int t = t_begin; t < t_end; ++t) {
    if (t + 1 < t_end) LLMC_WAIT_VM(C::L);
    else LLMC_WAIT_VM(0);
    dma::barrier();
    if (t + C::STAGES - 2 < t_end) issue(t + C::STAGES - 2);
    const uint16_t* stage = lds_dyn + ((t - t_begin) % C::STAGES) * C::STAGE_ELEMS;
    if (late) {
      const uint16_t* prev = lds_dyn + ((t - t_begin + C::STAGES - 1) % C::STAGES) * C::STAGE_ELEMS;
      reduce(reinterpret_cast<const float*>(prev + C::TILE_ELEMS + wave * C::RB * 2), t - 1);
    }
    const uint16_t* st = stage + frag_off;
    bf16x8_t fa[2][C::FM];
#pragma unroll
    for (int i = 0; i < C::FM; ++i)
      fa[0][i] = *reinterpret_cast<const bf16x8_t*>(st + i * 32 * C::K + ((half ^ fsw) * 8));
    __builtin_amdgcn_sched_group_barrier(0x100, C::FM, 0);
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
      const int c = ks & 1, n = c ^ 1;
      // the fragments of this step were requested one step ago; waiting for them BEFORE requesting the
      // next ones keeps the wait from covering a request that has only just been issued
      __builtin_amdgcn_sched_barrier(0);
      LLMC_WAIT_LGKM(0);
      __builtin_amdgcn_sched_barrier(0);
      if (ks + 1 < C::KS) {
#pragma unroll
        for (int i = 0; i < C::FM; ++i)
          fa[n][i] = *reinterpret_cast<const bf16x8_t*>(st + i * 32 * C::K + ((((ks + 1) * 2 + half) ^ fsw) * 8));
      }
#pragma unroll
      for (int i = 0; i < C::FM; ++i)
#pragma unroll
        for (int j = 0; j < C::FN; ++j) {
          if (ks == 0) {
            f32x16_t z;
#pragma unroll
            for (int r = 0; r < 16; ++r) z[r] = 0.f;
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c][i], bq[j][ks], z, 0, 0, 0);
          } else {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c][i], bq[j][ks], acc[i][j], 0, 0, 0);
          }
        }
      __builtin_amdgcn_sched_group_barrier(0x100, C::FM, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, C::FM * C::FN, 0);
    }
    if (!late) reduce(reinterpret_cast<const float*>(stage + C::TILE_ELEMS + wave * C::RB * 2), t);
  }
  if (late) {
    const uint16_t* stage = lds_dyn + ((t_end - 1 - t_begin) % C::STAGES) * C::STAGE_ELEMS;
    reduce(reinterpret_cast<const float*>(stage + C::TILE_ELEMS + wave * C::RB * 2), t_end - 1);
  }
#pragma unroll
  for (int j = 0; j < C::FN; ++j) {
    Top2 o;
    o.v1 = __shfl_xor(best[j].v1, 32, 64); o.g1 = __shfl_xor(best[j].g1, 32, 64);
    o.v2 = __shfl_xor(best[j].v2, 32, 64); o.g2 = __shfl_xor(best[j].g2, 32, 64);
    o.v3 = __shfl_xor(best[j].v3, 32, 64);
    Top2 m = best[j];
    top2_merge(m, o);
    const int q = q_base + j * 32 + (lane & 31);
    if (half == 0 && q < B) partial[(size_t)split * B + q] = m;
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
    for (int i = 0; i < 256; ++i) top2_merge(m, sc[i]);
    partial[b] = m;
  }
}

// One wavefront per query: merge the partial results of all bank splits, then decide the
// winner exactly.  The 64 lanes evaluate the 16 rows of a candidate group at once, 4 lanes
// per row, each over a quarter of the key in fp64; the four partial sums are added in a
// fixed order, and a butterfly picks the largest cosine (lowest slot among equals).
template <typename T>
__global__ __launch_bounds__(256) void match_finalize_kernel(
    const Top2* __restrict__ partial, int n_split, const T* __restrict__ bank, const float* __restrict__ binv,
    const uint8_t* __restrict__ valid, int N, int K, const T* __restrict__ queries, const float* __restrict__ qinv,
    int B, float tau, int32_t* __restrict__ idx_out, float* __restrict__ sim_out, uint8_t* __restrict__ hit_out,
    uint8_t* __restrict__ tie_out) {
  constexpr int VEC = Vec16<T>::N;
  const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (b >= B) return;
  const int lane = threadIdx.x & 63;
  Top2 t = top2_empty();
  // four partial results in flight per lane, merged in ascending split order
  for (int s0 = lane; s0 < n_split; s0 += 4 * 64) {
    Top2 c[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int s = s0 + u * 64;
      c[u] = s < n_split ? partial[(size_t)s * B + b] : top2_empty();
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) top2_merge(t, c[u]);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    Top2 c;
    c.v1 = __shfl_xor(t.v1, o, 64); c.g1 = __shfl_xor(t.g1, o, 64);
    c.v2 = __shfl_xor(t.v2, o, 64); c.g2 = __shfl_xor(t.g2, o, 64);
    c.v3 = __shfl_xor(t.v3, o, 64);
    top2_merge(t, c);
  }
  const float qi = qinv[b];
  const double qi64 = (double)qi;
  // scores so far are |q| * cos; the runner-up counts as tied within 1e-5 in cosine
  const float gap = qi > 0.f ? 1e-5f / qi : 0.f;
  const bool two = t.g2 >= 0 && t.v2 >= t.v1 - gap;
  // three or more groups that close: the two kept ones may not hold the arg-max; flagged and counted
  const bool many = two && t.v3 >= t.v1 - gap;
  const int n_groups = (t.g1 < 0) ? 0 : (two ? 2 : 1);
  const int r = lane >> 2, part = lane & 3;
  const int per = K / 4;                       // K is a multiple of 32, so per is a multiple of 8
  const T* qp = queries + (size_t)b * K + part * per;
  double best = -INFINITY;
  int best_j = -1;
  for (int c = 0; c < n_groups; ++c) {
    const int g = c == 0 ? t.g1 : t.g2;
    const int j = group_row(g, r);
    const int jc = min(j, N - 1);            // loads are issued for every lane, validity is applied afterwards
    const bool ok = j < N && valid[jc] != 0;
    const double bj = (double)binv[jc];
    const T* kp = bank + (size_t)jc * K + part * per;
    double a = 0.0;
    // eight 16-byte vectors of the query and of the key in flight; products added in ascending order
    int i = 0;
    for (; i + 8 * VEC <= per; i += 8 * VEC) {
      float x[8][VEC], y[8][VEC];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        Vec16<T>::load(qp + i + u * VEC, x[u]);
        Vec16<T>::load(kp + i + u * VEC, y[u]);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int e = 0; e < VEC; ++e) a += (double)x[u][e] * (double)y[u][e];
    }
    for (; i < per; i += VEC) {
      float x[VEC], y[VEC];
      Vec16<T>::load(qp + i, x);
      Vec16<T>::load(kp + i, y);
#pragma unroll
      for (int e = 0; e < VEC; ++e) a += (double)x[e] * (double)y[e];
    }
    a += __shfl_xor(a, 1, 64);
    a += __shfl_xor(a, 2, 64);
    if (ok) {
      const double s = a * qi64 * bj;
      if (s > best || (s == best && (best_j < 0 || j < best_j))) { best = s; best_j = j; }
    }
  }
#pragma unroll
  for (int o = 4; o < 64; o <<= 1) {
    const double os = __shfl_xor(best, o, 64);
    const int oj = __shfl_xor(best_j, o, 64);
    if (oj >= 0 && (best_j < 0 || os > best || (os == best && oj < best_j))) { best = os; best_j = oj; }
  }
  if (lane == 0) {
    idx_out[b] = best_j;
    if (sim_out) sim_out[b] = (float)best;
    if (hit_out) hit_out[b] = (best_j >= 0 && best > (double)tau) ? 1 : 0;
    if (tie_out) tie_out[b] = many ? 2 : (two ? 1 : 0);
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

// streaming kernel: about four workgroups per compute unit, at most 1024 splits
static void stream_plan(int N, int B, int RB, int QB, int* n_qb, int* n_split, int* tiles_per_split) {
  const int tiles = (N + RB - 1) / RB;
  const int qb = (B + QB - 1) / QB;
  int want = (1024 + qb - 1) / qb;
  if (want > tiles) want = tiles;
  if (want > 1024) want = 1024;
  if (want < 1) want = 1;
  const int per = (tiles + want - 1) / want;
  *n_qb = qb;
  *tiles_per_split = per;
  *n_split = (tiles + per - 1) / per;
}

// Few queries: workgroups of 4 wavefronts (256 query columns), two per compute unit.
// Many queries: workgroups of 8 wavefronts (512 query columns) with the deep ring.
static int stream_waves(int B) { return B <= 256 ? 4 : 8; }
static bool use_stream(int k) { return k == 64 || k == 128 || k == 256; }

// upper bound of match_ws_bytes over all banks: at most 1024 splits
size_t match_ws_max_bytes(int B) { return align_up((size_t)1024 * B * sizeof(Top2), 256); }

size_t match_ws_bytes(int n_slots, int k, int dtype, int B) {
  int ns = 1, per = 1, nqb = 1;
  if (dtype == LLMC_BF16) {
    if (use_stream(k)) stream_plan(n_slots, B, 64, stream_waves(B) * 64, &nqb, &ns, &per);
    else split_plan(n_slots, B, &ns, &per);
  }
  return align_up((size_t)ns * B * sizeof(Top2), 256);
}

template <int K_, int NW_>
static llmc_status_t launch_stream_nw(const llmc_bank* bank, const void* d_fp, int B, Top2* partial, int* ns_out,
                                      hipStream_t st) {
  using C = StreamCfg<K_, NW_>;
  const llmc_bank_desc_t& D = bank->desc;
  static std::atomic<bool> lds_set[64];
  LLMC_TRY(ensure_dynamic_lds((const void*)(match_stream_kernel<K_, NW_>), C::LDS_BYTES, lds_set));
  int nqb, ns, per;
  stream_plan(D.n_slots, B, C::RB, C::QB, &nqb, &ns, &per);
  const int groups = (ns + 7) / 8;                 // splits are dealt to the 8 XCDs
  const unsigned grid = (unsigned)groups * nqb * 8;
  ProfScope ps_("match_stream_kernel", st);
  LLMC_KERNEL_GGL((match_stream_kernel<K_, NW_>), dim3(grid), dim3(C::THREADS), C::LDS_BYTES, st,
                     (const uint16_t*)D.d_fp, bank->d_binv_eff, D.n_slots, (const uint16_t*)d_fp, B, nqb, ns, per,
                     partial);
  *ns_out = ns;
  return LLMC_OK;
}

template <int K_>
static llmc_status_t launch_stream(const llmc_bank* bank, const void* d_fp, int B, Top2* partial, int* ns_out,
                                   hipStream_t st) {
  if (stream_waves(B) == 4) return launch_stream_nw<K_, 4>(bank, d_fp, B, partial, ns_out, st);
  using C = SkewCfg<K_>;
  const llmc_bank_desc_t& D = bank->desc;
  static std::atomic<bool> lds_set[64];
  LLMC_TRY(ensure_dynamic_lds((const void*)(match_skew_kernel<K_>), C::LDS_BYTES, lds_set));
  int nqb, ns, per;
  stream_plan(D.n_slots, B, C::RB, C::QB, &nqb, &ns, &per);
  const unsigned grid = (unsigned)((ns + 7) / 8) * nqb * 8;    // splits are dealt to the 8 XCDs
  ProfScope ps_("match_stream_kernel", st);
  LLMC_KERNEL_GGL((match_skew_kernel<K_>), dim3(grid), dim3(512), C::LDS_BYTES, st, (const uint16_t*)D.d_fp,
                     bank->d_binv_eff, D.n_slots, (const uint16_t*)d_fp, B, nqb, ns, per, partial);
  *ns_out = ns;
  return LLMC_OK;
}

// ---- library-owned scratch for callers that cannot allocate ---------------------------------------------------
// The per-(split, query) candidates of the bulk pass normally live in a workspace the caller brings.  For callers
// that can neither allocate nor carry one around, the same kernels can write them into this file-scope device
// array instead: one copy per GPU, alive until the process ends, shared by every such call on that GPU.
static __device__ __align__(256) unsigned char scratch[LLMC_MATCH_STATIC_SCRATCH_BYTES];

// Device address of `scratch` on the current device.  In host code the array's name is only a handle for the
// symbol, never an address a kernel could use; the address is asked for once per device and kept.
llmc_status_t match_static_scratch(void** out, size_t* bytes) {
  static std::atomic<void*> ptr[64];
  int dev = 0;
  LLMC_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return set_error(LLMC_ERR_HIP, "device ordinal %d out of range", dev);
  void* p = ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    LLMC_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return set_error(LLMC_ERR_HIP, "hipGetSymbolAddress returned a null address");
    ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  *bytes = sizeof(scratch);
  return LLMC_OK;
}

llmc_status_t launch_match(const llmc_bank* bank, const void* d_fp, const float* d_inv, int B, float tau,
                           int32_t* d_idx, float* d_sim, uint8_t* d_hit, uint8_t* d_near_tie, void* ws,
                           hipStream_t st) {
  const llmc_bank_desc_t& D = bank->desc;
  const int N = D.n_slots, K = D.k;
  Top2* partial = (Top2*)ws;
  int ns = 1, per = 1;
  if (D.dtype == LLMC_BF16) {
    if (use_stream(K)) {
      if (K == 256) LLMC_TRY(launch_stream<256>(bank, d_fp, B, partial, &ns, st));
      else if (K == 128) LLMC_TRY(launch_stream<128>(bank, d_fp, B, partial, &ns, st));
      else LLMC_TRY(launch_stream<64>(bank, d_fp, B, partial, &ns, st));
      LLMC_LAUNCH_CHECK("match_stream_kernel");
    } else {
      split_plan(N, B, &ns, &per);
      dim3 grid(ns, (B + MatchCfg::BN - 1) / MatchCfg::BN);
      { ProfScope ps_("match_bf16_kernel", st); LLMC_KERNEL_GGL(match_bf16_kernel, grid, dim3(MatchCfg::THREADS), 0, st, (const uint16_t*)D.d_fp,
                         bank->d_binv_eff, N, K, (const uint16_t*)d_fp, B, per, partial); }
      LLMC_LAUNCH_CHECK("match_bf16_kernel");
    }
    { ProfScope ps_("match_finalize_kernel", st); LLMC_KERNEL_GGL((match_finalize_kernel<bf16_t>), dim3((B + 3) / 4), dim3(256), 0, st, partial, ns,
                       (const bf16_t*)D.d_fp, D.d_inv_norm, D.d_valid, N, K, (const bf16_t*)d_fp, d_inv, B, tau, d_idx,
                       d_sim, d_hit, d_near_tie); }
  } else {
    { ProfScope ps_("match_f32_kernel", st); LLMC_KERNEL_GGL(match_f32_kernel, dim3(B), dim3(256), (size_t)K * sizeof(float) + 256 * sizeof(Top2), st,
                       (const float*)D.d_fp, bank->d_binv_eff, N, K, (const float*)d_fp, partial); }
    LLMC_LAUNCH_CHECK("match_f32_kernel");
    { ProfScope ps_("match_finalize_kernel", st); LLMC_KERNEL_GGL((match_finalize_kernel<float>), dim3((B + 3) / 4), dim3(256), 0, st, partial, 1,
                       (const float*)D.d_fp, D.d_inv_norm, D.d_valid, N, K, (const float*)d_fp, d_inv, B, tau, d_idx,
                       d_sim, d_hit, d_near_tie); }
  }
  LLMC_LAUNCH_CHECK("match_finalize_kernel");
  return LLMC_OK;
}

}  // namespace llmc
