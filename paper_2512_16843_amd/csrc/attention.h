// Softmax attention of the miss path on the bf16 matrix cores (head size 64).
//
// A workgroup of 4 wavefronts owns 128 consecutive queries of one (sequence, head); each
// wavefront owns 32 of them and walks the keys in tiles of 64 with an online softmax.
// Both products are computed transposed so that a lane always holds ONE query column:
//   S^T [kv, q] = K [kv, dh] * Q [q, dh]^T          (A = K rows from LDS, B = Q in registers)
//   O^T [dh, q] += V^T [dh, kv] * P^T [kv, q]       (A = V^T rows from LDS, B = P from registers)
// The row maximum and row sum of a query are then per-lane reductions over registers plus
// one exchange between the two lane halves, and the probabilities of S^T feed the second
// product as its B operand without leaving registers: the k index of the instruction is a
// free permutation as long as both operands use the same one, so V^T fragments are read in
// the order in which the accumulator layout delivers the key rows
//   (half * 4 + 0..3, 8 + half * 4 + 0..3 within each block of 16 keys).
// V tiles are transposed on their way into LDS.
#pragma once
#include "common.h"
#include "mma.h"

namespace llmc {

struct AttnCfg {
  static constexpr int DH = 64, QB = 128, KT = 64, THREADS = 256;
  static constexpr int K_STRIDE = DH + 8;    // elements per K row in LDS (144 B: conflict-free 16-byte reads)
  static constexpr int V_STRIDE = KT + 4;    // elements per V^T row in LDS (136 B: conflict-free 8-byte reads)
  static constexpr int K_ELEMS = KT * K_STRIDE, V_ELEMS = DH * V_STRIDE;
};

typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) { return f32x2_to_bf16x2(a, b); }

// qkv [T, 3d] (compact token rows), ctx [T, d].  1-D grid, capped: workgroups walk the
// (sequence, head, query block) items with a grid stride; sequences beyond *count are skipped.
template <bool CAUSAL>
__global__ __launch_bounds__(AttnCfg::THREADS) void attention_mfma_kernel(const uint16_t* __restrict__ qkv,
                                                                          uint16_t* __restrict__ ctx, int S, int d,
                                                                          int n_heads, float scale_log2e,
                                                                          const int32_t* count, int max_seqs) {
  using C = AttnCfg;
  __shared__ __attribute__((aligned(16))) uint16_t sK[2][C::K_ELEMS];
  __shared__ __attribute__((aligned(16))) uint16_t sV[2][C::V_ELEMS];
  const int n_seq = count ? min(*count, max_seqs) : max_seqs;
  const int n_qb = (S + C::QB - 1) / C::QB;
  const int total = n_seq * n_heads * n_qb;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
  const size_t ld = 3 * (size_t)d;
  // staging role of this thread: two 16-byte vectors of K and of V per tile
  const int st_row = tid >> 3, st_chunk = tid & 7;      // rows st_row and st_row + 32, dh chunk of 8

  for (int item = blockIdx.x; item < total; item += gridDim.x) {
    const int qb = item % n_qb, head = (item / n_qb) % n_heads, seq = item / (n_qb * n_heads);
    const int q0 = qb * C::QB;
    const uint16_t* base = qkv + (size_t)seq * S * ld + head * C::DH;
    const int kv_end = CAUSAL ? min(S, q0 + C::QB) : S;
    const int n_tiles = (kv_end + C::KT - 1) / C::KT;

    // this wavefront's queries as B-operand fragments: column lane % 32, dh = ks * 16 + half * 8 ..
    const int q_lane = q0 + wave * 32 + (lane & 31);
    const int q_clamped = min(q_lane, S - 1);
    bf16x8_t fq[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      fq[ks] = *reinterpret_cast<const bf16x8_t*>(base + (size_t)q_clamped * ld + ks * 16 + half * 8);

    f32x16_t o[2];
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[f][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    uint4 rk[2], rv[2];
    auto load_tile = [&](int t) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int kr = min(t * C::KT + st_row + u * 32, S - 1);
        rk[u] = *reinterpret_cast<const uint4*>(base + (size_t)kr * ld + d + st_chunk * 8);
        rv[u] = *reinterpret_cast<const uint4*>(base + (size_t)kr * ld + 2 * d + st_chunk * 8);
      }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int row = st_row + u * 32;
        *reinterpret_cast<uint4*>(&sK[buf][row * C::K_STRIDE + st_chunk * 8]) = rk[u];
        const uint32_t w[4] = {rv[u].x, rv[u].y, rv[u].z, rv[u].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          sV[buf][(st_chunk * 8 + 2 * e) * C::V_STRIDE + row] = (uint16_t)(w[e] & 0xFFFFu);
          sV[buf][(st_chunk * 8 + 2 * e + 1) * C::V_STRIDE + row] = (uint16_t)(w[e] >> 16);
        }
      }
    };
    __syncthreads();            // the previous item's readers are done with both buffers
    load_tile(0);
    store_tile(0);
    __syncthreads();

    for (int t = 0; t < n_tiles; ++t) {
      const int buf = t & 1;
      if (t + 1 < n_tiles) load_tile(t + 1);
      // ---- S^T = K * Q^T for 64 keys x 32 queries ----
      f32x16_t s[2];
#pragma unroll
      for (int f = 0; f < 2; ++f) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[f][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const bf16x8_t fk = *reinterpret_cast<const bf16x8_t*>(
              &sK[buf][(f * 32 + (lane & 31)) * C::K_STRIDE + ks * 16 + half * 8]);
          s[f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk, fq[ks], s[f], 0, 0, 0);
        }
      }
      // ---- online softmax over this lane's 32 keys (base-2 exponent, scale folded in) ----
      const int kv0 = t * C::KT;
      const bool edge = (kv0 + C::KT > S) || (CAUSAL && kv0 + C::KT > q0 + wave * 32);
      // the maximum is taken over the raw scores (the scale is positive), the scale enters the exponent as one fma
      float mx = -INFINITY;
#pragma unroll
      for (int f = 0; f < 2; ++f)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float v = s[f][r];
          if (edge) {
            const int kv = kv0 + f * 32 + frag_row(lane, r);
            if (kv >= S || (CAUSAL && kv > q_lane)) v = -INFINITY;
            s[f][r] = v;
          }
          mx = fmaxf(mx, v);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run, mx * scale_log2e);          // finite: key 0 is visible to every query
      // the accumulators are rescaled only when some query of the wavefront met a larger score
      if (__any(m_new > m_run)) {
        const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
        l_run *= corr;
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[f][r] *= corr;
      }
      m_run = m_new;
      uint32_t pk[2][8];
#pragma unroll
      for (int f = 0; f < 2; ++f)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(s[f][r], scale_log2e, -m_new));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(s[f][r + 1], scale_log2e, -m_new));
          l_run += p0 + p1;
          pk[f][r >> 1] = pack_bf16x2(p0, p1);
        }
      // ---- O^T += V^T * P^T : 4 k-steps of 16 keys, 2 fragments of 32 dh rows ----
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        // keys of this k-step, in accumulator order: registers (ks % 2) * 8 .. + 8 of fragment ks / 2
        const int f = ks >> 1, rb = (ks & 1) * 4;
        union { uint32_t u[4]; bf16x8_t v; } pb;
#pragma unroll
        for (int e = 0; e < 4; ++e) pb.u[e] = pk[f][rb + e];
#pragma unroll
        for (int df = 0; df < 2; ++df) {
          const uint16_t* vrow = &sV[buf][(df * 32 + (lane & 31)) * C::V_STRIDE + ks * 16 + half * 4];
          union { uint2 u[2]; bf16x8_t v; } va;
          va.u[0] = *reinterpret_cast<const uint2*>(vrow);
          va.u[1] = *reinterpret_cast<const uint2*>(vrow + 8);
          o[df] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va.v, pb.v, o[df], 0, 0, 0);
        }
      }
      if (t + 1 < n_tiles) store_tile(buf ^ 1);
      __syncthreads();
    }
    // ---- normalise and store: lane holds query q_lane, dh rows df * 32 + half * 4 + 8 g + i ----
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_tot;
    if (q_lane < S) {
      uint16_t* dst = ctx + ((size_t)seq * S + q_lane) * d + head * C::DH;
#pragma unroll
      for (int df = 0; df < 2; ++df)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          uint2 w;
          w.x = pack_bf16x2(o[df][4 * g] * inv, o[df][4 * g + 1] * inv);
          w.y = pack_bf16x2(o[df][4 * g + 2] * inv, o[df][4 * g + 3] * inv);
          *reinterpret_cast<uint2*>(dst + df * 32 + half * 4 + 8 * g) = w;
        }
    }
  }
}

}  // namespace llmc
