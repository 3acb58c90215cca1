// bf16 matrix-core main loop shared by the dense layer GEMMs and the bank match.
//
// Computes a BM x BN block of  C = A * B^T  with A [*, K] and B [*, K] both
// K-contiguous in global memory, fp32 accumulation on v_mfma_f32_32x32x16_bf16.
// A and B tiles of BK columns are staged through LDS (double buffered, one barrier
// per step); each of the WM x WN wavefronts owns a (BM/WM) x (BN/WN) sub-block as
// 32x32 fragments.
//
// Fragment layout of the 32x32x16 instruction, per lane l of 64:
//   A operand: row  (l % 32) of the fragment, 8 consecutive k starting at (l / 32) * 8
//   B operand: col  (l % 32),                 the same 8 k
//   C/D:       col  (l % 32); register r (0..15) is row (l / 32) * 4 + 8 * (r / 4) + (r % 4)
#pragma once
#include "common.h"

namespace llmc {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

// row of register r of a 32x32 accumulator fragment held by `lane`
__device__ __forceinline__ int frag_row(int lane, int r) { return (lane >> 5) * 4 + 8 * (r >> 2) + (r & 3); }

template <int BM_, int BN_, int BK_, int WM_, int WN_>
struct MmaCfg {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
  static constexpr int THREADS = WM * WN * 64;
  static constexpr int LDS_STRIDE = BK + 8;             // bf16 elements; +16 B keeps 8- and 16-lane groups on distinct banks
  static constexpr int FM = BM / WM / 32, FN = BN / WN / 32;
  static constexpr int VEC_PER_ROW = BK / 8;
  static constexpr int NLOAD_A = BM * VEC_PER_ROW / THREADS;
  static constexpr int NLOAD_B = BN * VEC_PER_ROW / THREADS;
  static constexpr int A_TILE = BM * LDS_STRIDE, B_TILE = BN * LDS_STRIDE;   // elements
  static constexpr size_t LDS_BYTES = 2ull * (A_TILE + B_TILE) * 2;
  static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "wave tiling");
  static_assert((BM * VEC_PER_ROW) % THREADS == 0 && (BN * VEC_PER_ROW) % THREADS == 0, "load tiling");
  static_assert(BK % 16 == 0, "k step");
};

// a_ptr[i] / b_ptr[i]: global address of this thread's i-th 16-byte vector at k = 0
// (row already resolved and clamped by the caller).  K must be a multiple of BK.
// On return every wavefront has passed a barrier after its last LDS read.
template <class C>
__device__ __forceinline__ void mma_block(const uint16_t* const (&a_ptr)[C::NLOAD_A],
                                          const uint16_t* const (&b_ptr)[C::NLOAD_B], int K, uint16_t* lds,
                                          f32x16_t (&acc)[C::FM][C::FN]) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  uint16_t* sA[2] = {lds, lds + C::A_TILE + C::B_TILE};
  uint16_t* sB[2] = {lds + C::A_TILE, lds + 2 * C::A_TILE + C::B_TILE};

  int a_off[C::NLOAD_A], b_off[C::NLOAD_B];
#pragma unroll
  for (int i = 0; i < C::NLOAD_A; ++i) {
    const int v = tid + i * C::THREADS;
    a_off[i] = (v / C::VEC_PER_ROW) * C::LDS_STRIDE + (v % C::VEC_PER_ROW) * 8;
  }
#pragma unroll
  for (int i = 0; i < C::NLOAD_B; ++i) {
    const int v = tid + i * C::THREADS;
    b_off[i] = (v / C::VEC_PER_ROW) * C::LDS_STRIDE + (v % C::VEC_PER_ROW) * 8;
  }
  uint4 ra[C::NLOAD_A], rb[C::NLOAD_B];
#pragma unroll
  for (int i = 0; i < C::NLOAD_A; ++i) ra[i] = *reinterpret_cast<const uint4*>(a_ptr[i]);
#pragma unroll
  for (int i = 0; i < C::NLOAD_B; ++i) rb[i] = *reinterpret_cast<const uint4*>(b_ptr[i]);
#pragma unroll
  for (int i = 0; i < C::NLOAD_A; ++i) *reinterpret_cast<uint4*>(sA[0] + a_off[i]) = ra[i];
#pragma unroll
  for (int i = 0; i < C::NLOAD_B; ++i) *reinterpret_cast<uint4*>(sB[0] + b_off[i]) = rb[i];
  __syncthreads();

  const int a_read = (wm * (C::BM / C::WM) + (lane & 31)) * C::LDS_STRIDE + (lane >> 5) * 8;
  const int b_read = (wn * (C::BN / C::WN) + (lane & 31)) * C::LDS_STRIDE + (lane >> 5) * 8;
  constexpr int KS = C::BK / 16;
  const int nk = K / C::BK;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < nk;
    if (more) {
      const int ko = (kt + 1) * C::BK;
#pragma unroll
      for (int i = 0; i < C::NLOAD_A; ++i) ra[i] = *reinterpret_cast<const uint4*>(a_ptr[i] + ko);
#pragma unroll
      for (int i = 0; i < C::NLOAD_B; ++i) rb[i] = *reinterpret_cast<const uint4*>(b_ptr[i] + ko);
    }
    const uint16_t* pa = sA[cur] + a_read;
    const uint16_t* pb = sB[cur] + b_read;
    bf16x8_t fa[2][C::FM], fb[2][C::FN];
#pragma unroll
    for (int i = 0; i < C::FM; ++i) fa[0][i] = *reinterpret_cast<const bf16x8_t*>(pa + i * 32 * C::LDS_STRIDE);
#pragma unroll
    for (int j = 0; j < C::FN; ++j) fb[0][j] = *reinterpret_cast<const bf16x8_t*>(pb + j * 32 * C::LDS_STRIDE);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int c = ks & 1, n = c ^ 1;
      if (ks + 1 < KS) {
#pragma unroll
        for (int i = 0; i < C::FM; ++i)
          fa[n][i] = *reinterpret_cast<const bf16x8_t*>(pa + i * 32 * C::LDS_STRIDE + (ks + 1) * 16);
#pragma unroll
        for (int j = 0; j < C::FN; ++j)
          fb[n][j] = *reinterpret_cast<const bf16x8_t*>(pb + j * 32 * C::LDS_STRIDE + (ks + 1) * 16);
      }
#pragma unroll
      for (int i = 0; i < C::FM; ++i)
#pragma unroll
        for (int j = 0; j < C::FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c][i], fb[c][j], acc[i][j], 0, 0, 0);
    }
    if (more) {
#pragma unroll
      for (int i = 0; i < C::NLOAD_A; ++i) *reinterpret_cast<uint4*>(sA[cur ^ 1] + a_off[i]) = ra[i];
#pragma unroll
      for (int i = 0; i < C::NLOAD_B; ++i) *reinterpret_cast<uint4*>(sB[cur ^ 1] + b_off[i]) = rb[i];
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------
// Main loop with direct global -> LDS loads (global_load_lds_dwordx4) and a ring of
// STAGES tile buffers, so that STAGES - 1 tiles of 64 k-columns are in flight while one is
// being multiplied.  No registers are spent on staging.
//
// One load instruction of a wavefront fills 8 tile rows of 128 bytes: lane i writes the
// 16-byte slot i of that 1 KiB block.  A 16-byte fragment read is served 16 lanes at a time
// (16 x 16 bytes = one pass over the 64 banks), and those 16 lanes read one logical chunk
// of 16 consecutive tile rows; two 128-byte rows span the banks once, so rows of equal
// parity must spread over the 8 slots of a row.  The chunks of a row are therefore stored
// XOR-swizzled by half the row number: chunk c of tile row r lives in slot c ^ ((r / 2) % 8)
// of its row.  The permutation is applied on the global side (each lane chooses which
// chunk it fetches).
//
// The compiler does not order these loads against LDS reads, so ordering is explicit:
// s_waitcnt vmcnt(n) for the wave's own loads, then a workgroup barrier.
namespace dma {
#define LLMC_GPTR(p) ((const void __attribute__((address_space(1)))*)(p))
#define LLMC_LPTR(p) ((void __attribute__((address_space(3)))*)(p))
#define LLMC_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))
// wait until at most n LDS / scalar-memory operations of this wavefront are outstanding (n <= 15)
#define LLMC_WAIT_LGKM(n) __builtin_amdgcn_s_waitcnt(0xC07F | ((n) << 8))

__device__ __forceinline__ void barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}
}  // namespace dma

template <int BM_, int BN_, int WM_, int WN_, int STAGES_>
struct DmaCfg {
  static constexpr int BM = BM_, BN = BN_, BK = 64, WM = WM_, WN = WN_, STAGES = STAGES_;
  static constexpr int NW = WM * WN, THREADS = NW * 64;
  static constexpr int FM = BM / WM / 32, FN = BN / WN / 32;
  static constexpr int A_INSTR = BM / 8 / NW, B_INSTR = BN / 8 / NW;     // loads per lane per stage
  static constexpr int L = A_INSTR + B_INSTR;
  static constexpr int STAGE_ELEMS = (BM + BN) * BK;
  static constexpr size_t LDS_BYTES = (size_t)STAGES * STAGE_ELEMS * 2;
  static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "wave tiling");
  static_assert((BM / 8) % NW == 0 && (BN / 8) % NW == 0, "load tiling");
  static_assert(STAGES >= 2 && STAGES <= 4 && 3 * L <= 63, "pipeline depth");
  // tile row and k-chunk fetched by `lane` of `wave` in its j-th load of a stage
  __device__ static __forceinline__ int load_row(int j, int wave, int lane) { return (j * NW + wave) * 8 + (lane >> 3); }
  __device__ static __forceinline__ int load_chunk(int row, int lane) { return (lane & 7) ^ ((row >> 1) & 7); }
};

// a_ptr[j] / b_ptr[j]: global address (k = 0) of the 16-byte chunk that this lane fetches in
// its j-th A / B load: row load_row(j, wave, lane) of the tile (resolved and clamped by the
// caller), element offset load_chunk(row, lane) * 8.  K must be a multiple of 64.
// The main loop is a ring of two stages that runs on across the tiles of a workgroup.
// dma_issue: the loads of k-tile kt of the tile that a_ptr / b_ptr describe, into ring stage `stage`.
template <class C>
__device__ __forceinline__ void dma_issue(const uint16_t* const (&a_ptr)[C::A_INSTR],
                                          const uint16_t* const (&b_ptr)[C::B_INSTR], int kt, int stage, uint16_t* lds) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint16_t* st = lds + stage * C::STAGE_ELEMS;
  const int ko = kt * C::BK;
#pragma unroll
  for (int j = 0; j < C::A_INSTR; ++j)
    __builtin_amdgcn_global_load_lds(LLMC_GPTR(a_ptr[j] + ko), LLMC_LPTR(st + (j * C::NW + wave) * 8 * C::BK), 16, 0, 0);
#pragma unroll
  for (int j = 0; j < C::B_INSTR; ++j)
    __builtin_amdgcn_global_load_lds(LLMC_GPTR(b_ptr[j] + ko),
                                     LLMC_LPTR(st + C::BM * C::BK + (j * C::NW + wave) * 8 * C::BK), 16, 0, 0);
}

// The main loop with the ring position carried by the caller: k-tile 0 of this tile has ALREADY been issued into
// stage ring % 2 (by the previous tile, before its epilogue, or by the kernel's prologue) AND waited for by the
// issuing wavefront; k-tile kt lives in stage (ring + kt) % 2.  Ends with a barrier: every wavefront is done reading both stages.
template <class C>
__device__ __forceinline__ void mma_block_dma_ring(const uint16_t* const (&a_ptr)[C::A_INSTR],
                                                   const uint16_t* const (&b_ptr)[C::B_INSTR], int K, uint16_t* lds,
                                                   f32x16_t (&acc)[C::FM][C::FN], int ring) {
  static_assert(C::STAGES == 2, "the cross-tile ring has two stages");
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int nk = K / C::BK;
  const int a_row = (wm * (C::BM / C::WM) + (lane & 31)) * C::BK;
  const int b_row = C::BM * C::BK + (wn * (C::BN / C::WN) + (lane & 31)) * C::BK;
  int sw[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) sw[ks] = (((ks * 2 + (lane >> 5)) ^ ((lane >> 1) & 7)) * 8);

  for (int kt = 0; kt < nk; ++kt) {
    // k-tile 0: the caller has already waited for this wavefront's loads of it (in the kernel's prologue, or late
    // in the previous tile's epilogue, so that the epilogue's last stores need not drain before the tile starts)
    if (kt > 0) LLMC_WAIT_VM(0);
    dma::barrier();
    if (kt + 1 < nk) dma_issue<C>(a_ptr, b_ptr, kt + 1, (ring + kt + 1) & 1, lds);
    const uint16_t* st = lds + ((ring + kt) & 1) * C::STAGE_ELEMS;
    bf16x8_t fa[2][C::FM], fb[2][C::FN];
#pragma unroll
    for (int i = 0; i < C::FM; ++i) fa[0][i] = *reinterpret_cast<const bf16x8_t*>(st + a_row + i * 32 * C::BK + sw[0]);
#pragma unroll
    for (int j = 0; j < C::FN; ++j) fb[0][j] = *reinterpret_cast<const bf16x8_t*>(st + b_row + j * 32 * C::BK + sw[0]);
    __builtin_amdgcn_sched_group_barrier(0x100, C::FM + C::FN, 0);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int c = ks & 1, n = c ^ 1;
      __builtin_amdgcn_sched_barrier(0);
      LLMC_WAIT_LGKM(0);
      __builtin_amdgcn_sched_barrier(0);
      if (ks + 1 < 4) {
#pragma unroll
        for (int i = 0; i < C::FM; ++i)
          fa[n][i] = *reinterpret_cast<const bf16x8_t*>(st + a_row + i * 32 * C::BK + sw[ks + 1]);
#pragma unroll
        for (int j = 0; j < C::FN; ++j)
          fb[n][j] = *reinterpret_cast<const bf16x8_t*>(st + b_row + j * 32 * C::BK + sw[ks + 1]);
      }
#pragma unroll
      for (int i = 0; i < C::FM; ++i)
#pragma unroll
        for (int j = 0; j < C::FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c][i], fb[c][j], acc[i][j], 0, 0, 0);
      if (ks + 1 < 4) __builtin_amdgcn_sched_group_barrier(0x100, C::FM + C::FN, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, C::FM * C::FN, 0);
    }
  }
  dma::barrier();
}

// The main loop of ONE tile with a ring of C::STAGES stages of its own (STAGES - 1 steps in flight): for launches
// with fewer tiles than compute units, where a workgroup has its compute unit to itself and a step's time is the
// latency of its loads.  Starts and ends with every stage free; ends with a barrier.
template <class C>
__device__ __forceinline__ void mma_block_dma(const uint16_t* const (&a_ptr)[C::A_INSTR],
                                              const uint16_t* const (&b_ptr)[C::B_INSTR], int K, uint16_t* lds,
                                              f32x16_t (&acc)[C::FM][C::FN]) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / C::WN, wn = wave % C::WN;
  const int nk = K / C::BK;

  auto issue = [&](int kt) { dma_issue<C>(a_ptr, b_ptr, kt, kt % C::STAGES, lds); };
#pragma unroll
  for (int s = 0; s < C::STAGES - 1; ++s)
    if (s < nk) issue(s);

  // fragment read offsets (elements): row * 64 + ((chunk ^ ((row / 2) & 7)) * 8), (row / 2) & 7 == (lane / 2) & 7
  const int a_row = (wm * (C::BM / C::WM) + (lane & 31)) * C::BK;
  const int b_row = C::BM * C::BK + (wn * (C::BN / C::WN) + (lane & 31)) * C::BK;
  int sw[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) sw[ks] = (((ks * 2 + (lane >> 5)) ^ ((lane >> 1) & 7)) * 8);

  for (int kt = 0; kt < nk; ++kt) {
    const int ahead = min(C::STAGES - 2, nk - 1 - kt);
    if (ahead <= 0) LLMC_WAIT_VM(0);
    else if (ahead == 1) LLMC_WAIT_VM(C::L);
    else LLMC_WAIT_VM(2 * C::L);
    dma::barrier();
    if (kt + C::STAGES - 1 < nk) issue(kt + C::STAGES - 1);
    const uint16_t* st = lds + (kt % C::STAGES) * C::STAGE_ELEMS;
    // fragments of the next 16-column step are fetched while the current step multiplies
    bf16x8_t fa[2][C::FM], fb[2][C::FN];
#pragma unroll
    for (int i = 0; i < C::FM; ++i) fa[0][i] = *reinterpret_cast<const bf16x8_t*>(st + a_row + i * 32 * C::BK + sw[0]);
#pragma unroll
    for (int j = 0; j < C::FN; ++j) fb[0][j] = *reinterpret_cast<const bf16x8_t*>(st + b_row + j * 32 * C::BK + sw[0]);
    __builtin_amdgcn_sched_group_barrier(0x100, C::FM + C::FN, 0);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int c = ks & 1, n = c ^ 1;
      // this step's fragments were requested one step ago: wait for them BEFORE requesting the next
      // ones, so that the wait never covers a request that has only just been issued
      __builtin_amdgcn_sched_barrier(0);
      LLMC_WAIT_LGKM(0);
      __builtin_amdgcn_sched_barrier(0);
      if (ks + 1 < 4) {
#pragma unroll
        for (int i = 0; i < C::FM; ++i)
          fa[n][i] = *reinterpret_cast<const bf16x8_t*>(st + a_row + i * 32 * C::BK + sw[ks + 1]);
#pragma unroll
        for (int j = 0; j < C::FN; ++j)
          fb[n][j] = *reinterpret_cast<const bf16x8_t*>(st + b_row + j * 32 * C::BK + sw[ks + 1]);
      }
#pragma unroll
      for (int i = 0; i < C::FM; ++i)
#pragma unroll
        for (int j = 0; j < C::FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c][i], fb[c][j], acc[i][j], 0, 0, 0);
      // keep the written order: the next step's LDS reads are issued before this step's MFMAs
      if (ks + 1 < 4) __builtin_amdgcn_sched_group_barrier(0x100, C::FM + C::FN, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, C::FM * C::FN, 0);
    }
  }
  dma::barrier();   // every wavefront is done reading before the caller reuses the LDS
}

}  // namespace llmc
