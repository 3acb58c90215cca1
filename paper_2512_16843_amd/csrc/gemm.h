// Linear layer  out = act(A * W^T + bias) (+ residual)  on the bf16 matrix cores, with the
// row gather / scatter of the miss path fused into operand loads and the epilogue.
#pragma once
#include "common.h"
#include "mma.h"

namespace llmc {

// compact token -> row of a [B*S, *] array through an optional sequence list
__device__ __forceinline__ int64_t map_row(const int32_t* rows, int r, int S) {
  if (!rows) return r;
  const int q = r / S;
  return (int64_t)rows[q] * S + (r - q * S);
}

// erf by the five-term rational approximation of Abramowitz & Stegun 7.1.26
// (absolute error below 1.5e-7), with the hardware reciprocal and exponential
__device__ __forceinline__ float erf_as(float x) {
  const float ax = fabsf(x);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  const float e = __expf(-ax * ax);
  const float r = fmaf(-p * t, e, 1.0f);
  return copysignf(r, x);
}
__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erf_as(x * 0.70710678118654752440f)); }
__device__ __forceinline__ float gelu_tanh(float x) {
  const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
  // tanh(u) = 1 - 2 / (1 + e^{2u}); e^{2u} = inf gives 1, 0 gives -1
  const float th = 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __expf(2.0f * u));
  return 0.5f * x * (1.0f + th);
}

struct GemmArgs {
  const void* A; int lda;          // [rows, K]
  const void* W;                   // [N, K]
  const void* bias;                // [N] or null
  const void* resid; int ldr;      // [rows, N] or null
  void* out; int ldo;              // [rows, N]
  int N, K, S;
  const int32_t* count;            // device: number of sequences; null = max_seqs
  int max_seqs;
  const int32_t* a_rows;           // sequence list applied to A rows, or null
  const int32_t* r_rows;           // ... to residual rows
  const int32_t* o_rows;           // ... to output rows
  int act;                         // 0 none, 1 GELU erf, 2 GELU tanh
  int xcd_chunks;                  // tile -> workgroup map of the direct-to-LDS kernel, see there
};

__device__ __forceinline__ float apply_act(float v, int act) {
  if (act == 1) return gelu_erf(v);
  if (act == 2) return gelu_tanh(v);
  return v;
}

// ---- bf16 GEMM on the matrix cores -------------------------------------------------------
// bias, activation, residual and (scattered) store of one block's accumulators
template <class C>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& g, f32x16_t (&acc)[C::FM][C::FN], int m0, int n0, int M) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  const uint16_t* bias = (const uint16_t*)g.bias;
  const uint16_t* resid = (const uint16_t*)g.resid;
  uint16_t* out = (uint16_t*)g.out;
#pragma unroll
  for (int j = 0; j < C::FN; ++j) {
    const int n = n0 + wn * (C::BN / C::WN) + j * 32 + (lane & 31);
    if (n >= g.N) continue;
    const float bv = bias ? bf16_to_f32(bias[n]) : 0.f;
#pragma unroll
    for (int i = 0; i < C::FM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * (C::BM / C::WM) + i * 32 + frag_row(lane, r);
        if (m >= M) continue;
        float v = apply_act(acc[i][j][r] + bv, g.act);
        if (resid) v += bf16_to_f32(resid[map_row(g.r_rows, m, g.S) * g.ldr + n]);
        out[map_row(g.o_rows, m, g.S) * g.ldo + n] = f32_to_bf16(v);
      }
    }
  }
}

template <class C>
__global__ __launch_bounds__(C::THREADS) void gemm_bf16_kernel(GemmArgs g, int tiles_n) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[C::LDS_BYTES / 2];
  const int n_seq = g.count ? min(*g.count, g.max_seqs) : g.max_seqs;
  const int M = n_seq * g.S;
  const int total = ((M + C::BM - 1) / C::BM) * tiles_n;
  const int tid = threadIdx.x;
  // the grid is capped: a workgroup walks tiles blockIdx.x, blockIdx.x + gridDim.x, ...
  for (int tile = blockIdx.x; tile < total; tile += gridDim.x) {
  const int tile_m = tile / tiles_n, tile_n = tile % tiles_n;
  const int m0 = tile_m * C::BM, n0 = tile_n * C::BN;
  const uint16_t* A = (const uint16_t*)g.A;
  const uint16_t* W = (const uint16_t*)g.W;
  const uint16_t* a_ptr[C::NLOAD_A];
  const uint16_t* b_ptr[C::NLOAD_B];
#pragma unroll
  for (int i = 0; i < C::NLOAD_A; ++i) {
    const int v = tid + i * C::THREADS;
    const int r = min(m0 + v / C::VEC_PER_ROW, M - 1);
    a_ptr[i] = A + map_row(g.a_rows, r, g.S) * g.lda + (v % C::VEC_PER_ROW) * 8;
  }
#pragma unroll
  for (int i = 0; i < C::NLOAD_B; ++i) {
    const int v = tid + i * C::THREADS;
    const int r = min(n0 + v / C::VEC_PER_ROW, g.N - 1);
    b_ptr[i] = W + (size_t)r * g.K + (v % C::VEC_PER_ROW) * 8;
  }
  f32x16_t acc[C::FM][C::FN];
#pragma unroll
  for (int i = 0; i < C::FM; ++i)
#pragma unroll
    for (int j = 0; j < C::FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  mma_block<C>(a_ptr, b_ptr, g.K, lds, acc);
  gemm_epilogue<C>(g, acc, m0, n0, M);
  }
}

// Epilogue through LDS, one wavefront at a time: a wavefront lays 16 rows of its accumulators (half a fragment:
// registers 8 h .. 8 h + 7 hold rows 16 h .. 16 h + 15 of it) out as fp32 [16][FN * 32 + 4] in a region of its own,
// then its lanes take 8 consecutive columns of a row each, so that bias, residual and output move as 16-byte
// vectors along rows.  No other wavefront touches the region, and LDS operations of one wavefront complete in
// order, so no barrier is needed between the two halves.  Blocks of 16 rows keep the staging of all wavefronts
// inside ONE ring stage, so the other stage can already receive the next tile's first loads.  `stage` is that
// ring stage; no barrier inside or after: the next tile's first barrier comes before anything is loaded into this
// stage again.
template <class C>
struct WaveEpilogue16 {
  static constexpr int COLS = C::FN * 32, STRIDE = COLS + 4, REGION = 16 * STRIDE;   // floats
  static constexpr int LANES_PER_ROW = COLS / 8, ROWS_PER_PASS = 64 / LANES_PER_ROW;
  static_assert(64 % LANES_PER_ROW == 0 && 16 % ROWS_PER_PASS == 0, "row vectors tile the block");
  static_assert((size_t)C::NW * REGION * 4 <= (size_t)C::STAGE_ELEMS * 2, "the staging fits one ring stage");
};

template <class C>
__device__ __forceinline__ void gemm_epilogue_wave16(const GemmArgs& g, f32x16_t (&acc)[C::FM][C::FN], int m0, int n0,
                                                     int M, float* stage, bool wait_before_last) {
  using E = WaveEpilogue16<C>;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / C::WN, wn = wave % C::WN;
  float* region = stage + wave * E::REGION;
  const uint16_t* bias = (const uint16_t*)g.bias;
  const uint16_t* resid = (const uint16_t*)g.resid;
  uint16_t* out = (uint16_t*)g.out;
  const int prow = lane / E::LANES_PER_ROW, c8 = (lane % E::LANES_PER_ROW) * 8;
  const int n = n0 + wn * E::COLS + c8;
  float bv[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) bv[e] = 0.f;
  if (bias && n < g.N) Vec16<bf16_t>::load(reinterpret_cast<const bf16_t*>(bias + n), bv);
#pragma unroll
  for (int i = 0; i < C::FM; ++i) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int j = 0; j < C::FN; ++j) {
        float* p = region + j * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 8; ++r) p[(frag_row(lane, 8 * h + r) - 16 * h) * E::STRIDE] = acc[i][j][8 * h + r];
      }
      const int mb = m0 + wm * (C::BM / C::WM) + i * 32 + h * 16;
#pragma unroll
      for (int pass = 0; pass < 16 / E::ROWS_PER_PASS; ++pass) {
        const int row = pass * E::ROWS_PER_PASS + prow;
        const int m = mb + row;
        const float4 lo = *reinterpret_cast<const float4*>(region + row * E::STRIDE + c8);
        const float4 hi = *reinterpret_cast<const float4*>(region + row * E::STRIDE + c8 + 4);
        const bool live = m < M && n < g.N;
        float v[8] = {lo.x + bv[0], lo.y + bv[1], lo.z + bv[2], lo.w + bv[3],
                      hi.x + bv[4], hi.y + bv[5], hi.z + bv[6], hi.w + bv[7]};
        if (g.act) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = apply_act(v[e], g.act);
        }
        if (resid && live) {
          float rr[8];
          Vec16<bf16_t>::load(reinterpret_cast<const bf16_t*>(resid + map_row(g.r_rows, m, g.S) * g.ldr + n), rr);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += rr[e];
        }
        // before the LAST stores of the tile: everything this wavefront has in flight has landed, in particular its
        // loads of the next tile's first step (issued before this epilogue began); the stores below are then the
        // only traffic outstanding when the next tile's main loop starts, and its first step does not wait for them
        if (wait_before_last && i == C::FM - 1 && h == 1 && pass == 16 / E::ROWS_PER_PASS - 1) LLMC_WAIT_VM(0);
        if (live) Vec16<bf16_t>::store(reinterpret_cast<bf16_t*>(out + map_row(g.o_rows, m, g.S) * g.ldo + n), v);
      }
    }
  }
}

template <class C, class CS>
constexpr size_t gemm_dma_smem_bytes() {
  return C::LDS_BYTES > CS::LDS_BYTES ? C::LDS_BYTES : CS::LDS_BYTES;
}

// at most this many C tiles in a launch: the launch takes CS tiles instead (see the kernel)
constexpr int kGemmSmallTiles = 256;

// Same contract, main loop with direct global -> LDS loads (C is a DmaCfg with two stages); K % 64 == 0.
// A workgroup walks its tiles with ONE ring of two stages that runs on across tiles: when the main loop of a tile
// ends, the first loads of the workgroup's next tile go into the stage that is free, and only then does the epilogue
// start (its staging lives in the stage the last step has just been read from), so the memory latency of a tile's
// first step hides behind the previous tile's epilogue instead of standing in front of every tile.
// Few rows (the count is read on the device): when the C tiles of a launch would not even give every compute unit
// one, the launch is cut into the smaller CS tiles instead (same columns, half the rows, so twice as many
// workgroups have work) and each tile runs its main loop with a deeper ring of its own, because a workgroup that has
// its compute unit to itself spends a step waiting for that step's loads.  An output element is accumulated over k
// in the same order by either tiling, so the bits of a row do not depend on how many rows are computed with it.
template <class C, class CS>
__global__ __launch_bounds__(C::THREADS) void gemm_bf16_dma_kernel(GemmArgs g, int tiles_n) {
  static_assert(C::THREADS == CS::THREADS && C::BN == CS::BN, "the two tilings share the launch shape and the column tiles");
  extern __shared__ __attribute__((aligned(16))) uint16_t lds_dyn[];
  const int n_seq = g.count ? min(*g.count, g.max_seqs) : g.max_seqs;
  const int M = n_seq * g.S;
  const int tiles_m = (M + C::BM - 1) / C::BM;
  const int total = tiles_m * tiles_n;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (total <= kGemmSmallTiles) {
    const int total_s = ((M + CS::BM - 1) / CS::BM) * tiles_n;
    const uint16_t* A = (const uint16_t*)g.A;
    const uint16_t* W = (const uint16_t*)g.W;
    for (int tile = blockIdx.x; tile < total_s; tile += gridDim.x) {
      const int m0 = (tile / tiles_n) * CS::BM, n0 = (tile % tiles_n) * CS::BN;
      const uint16_t* a_ptr[CS::A_INSTR];
      const uint16_t* b_ptr[CS::B_INSTR];
#pragma unroll
      for (int j = 0; j < CS::A_INSTR; ++j) {
        const int tr = CS::load_row(j, wave, lane);
        const int r = min(m0 + tr, M - 1);
        a_ptr[j] = A + map_row(g.a_rows, r, g.S) * g.lda + CS::load_chunk(tr, lane) * 8;
      }
#pragma unroll
      for (int j = 0; j < CS::B_INSTR; ++j) {
        const int tr = CS::load_row(j, wave, lane);
        const int r = min(n0 + tr, g.N - 1);
        b_ptr[j] = W + (size_t)r * g.K + CS::load_chunk(tr, lane) * 8;
      }
      f32x16_t acc[CS::FM][CS::FN];
#pragma unroll
      for (int i = 0; i < CS::FM; ++i)
#pragma unroll
        for (int j = 0; j < CS::FN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
      mma_block_dma<CS>(a_ptr, b_ptr, g.K, lds_dyn, acc);
      // every stage is free after the main loop: the staging of the epilogue takes the first one
      gemm_epilogue_wave16<CS>(g, acc, m0, n0, M, reinterpret_cast<float*>(lds_dyn), false);
      dma::barrier();             // ... and is read out before the next tile's first loads land there
    }
    return;
  }
  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  With xcd_chunks set, XCD x
  // walks the x-th eighth of the tile list, so the operand panels of neighbouring tiles are fetched into one L2
  // only and shared there; otherwise workgroups stride over the tile list.  gridDim.x % 8 == 0 when xcd_chunks.
  // xcd_chunks == 1: the list is row-major (the column tiles of a row block are adjacent: narrow outputs);
  // xcd_chunks == 2: grouped order, the list runs down 8 row blocks before it moves one column tile on, so the 64
  // tiles that an XCD's workgroups hold at one time are 8 row blocks x 8 column tiles: 16 operand panels (3 MB).
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, slots = gridDim.x >> 3;
  const int per_xcd = (total + 7) >> 3;
  const int n_it = g.xcd_chunks ? per_xcd : total;
  const int it_step = g.xcd_chunks ? slots : (int)gridDim.x;
  const uint16_t* A = (const uint16_t*)g.A;
  const uint16_t* W = (const uint16_t*)g.W;
  const uint16_t* a_ptr[C::A_INSTR];
  const uint16_t* b_ptr[C::B_INSTR];
  int m0 = 0, n0 = 0;
  // tile of list position `it` (negative: none), and this lane's load addresses for it
  auto locate = [&](int it) -> bool {
    if (it >= n_it) return false;
    const int tile = g.xcd_chunks ? xcd * per_xcd + it : it;
    if (tile >= total) return false;
    int tile_m = tile / tiles_n, tile_n = tile % tiles_n;
    if (g.xcd_chunks == 2) {
      const int group = tile / (8 * tiles_n), in_group = tile % (8 * tiles_n);
      const int rows_in_group = min(8, tiles_m - group * 8);
      tile_m = group * 8 + in_group % rows_in_group;
      tile_n = in_group / rows_in_group;
    }
    m0 = tile_m * C::BM;
    n0 = tile_n * C::BN;
#pragma unroll
    for (int j = 0; j < C::A_INSTR; ++j) {
      const int tr = C::load_row(j, wave, lane);
      const int r = min(m0 + tr, M - 1);
      a_ptr[j] = A + map_row(g.a_rows, r, g.S) * g.lda + C::load_chunk(tr, lane) * 8;
    }
#pragma unroll
    for (int j = 0; j < C::B_INSTR; ++j) {
      const int tr = C::load_row(j, wave, lane);
      const int r = min(n0 + tr, g.N - 1);
      b_ptr[j] = W + (size_t)r * g.K + C::load_chunk(tr, lane) * 8;
    }
    return true;
  };
  int it = g.xcd_chunks ? slot : (int)blockIdx.x;
  if (!locate(it)) return;
  const int nk = g.K / C::BK;
  int ring = 0;
  dma_issue<C>(a_ptr, b_ptr, 0, 0, lds_dyn);
  LLMC_WAIT_VM(0);
  while (true) {
    f32x16_t acc[C::FM][C::FN];
#pragma unroll
    for (int i = 0; i < C::FM; ++i)
#pragma unroll
      for (int j = 0; j < C::FN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    mma_block_dma_ring<C>(a_ptr, b_ptr, g.K, lds_dyn, acc, ring);
    const int cur_m0 = m0, cur_n0 = n0;
    const int last_stage = (ring + nk - 1) & 1;
    ring += nk;
    it += it_step;
    const bool more = locate(it);                       // uniform over the workgroup
    if (more) dma_issue<C>(a_ptr, b_ptr, 0, ring & 1, lds_dyn);
    gemm_epilogue_wave16<C>(g, acc, cur_m0, cur_n0, M, reinterpret_cast<float*>(lds_dyn + last_stage * C::STAGE_ELEMS), more);
    if (!more) break;
  }
}

}  // namespace llmc
