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
  static constexpr int LDS_STRIDE = BK + 8;             // bf16 elements; +16 B keeps 16-lane groups on distinct banks
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
#pragma unroll
    for (int ks = 0; ks < C::BK / 16; ++ks) {
      bf16x8_t fa[C::FM], fb[C::FN];
#pragma unroll
      for (int i = 0; i < C::FM; ++i)
        fa[i] = *reinterpret_cast<const bf16x8_t*>(sA[cur] + a_read + i * 32 * C::LDS_STRIDE + ks * 16);
#pragma unroll
      for (int j = 0; j < C::FN; ++j)
        fb[j] = *reinterpret_cast<const bf16x8_t*>(sB[cur] + b_read + j * 32 * C::LDS_STRIDE + ks * 16);
#pragma unroll
      for (int i = 0; i < C::FM; ++i)
#pragma unroll
        for (int j = 0; j < C::FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
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

}  // namespace llmc
