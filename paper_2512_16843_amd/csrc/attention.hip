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
//
// The kernel is bound by its vector-ALU work (one exponential, one scale-and-shift, one
// maximum and one sum per score against 4 matrix-core flops per score and head dimension),
// so everything else is kept off the vector pipe:
//   * this file is compiled with the matrix instructions' accumulators in ordinary vector
//     registers (the scores are consumed by vector instructions straight away) and without
//     NaN handling (no score is a NaN for finite inputs; masked scores are -inf, which stays
//     exact), so a maximum is one instruction instead of a quieting copy per operand;
//   * V tiles are transposed on their way into LDS two keys at a time (one 32-bit store per
//     head dimension and key pair), the groups of four keys XOR-swizzled by the half of the
//     head dimension so that the 64 stores of a wavefront fall into 64 different banks;
//   * the two lane halves exchange their maxima with one lane-swap instruction;
//   * the row sum adds the ROUNDED probabilities, two per instruction, so the normaliser is
//     the sum of exactly the weights the second product uses.
#include "common.h"
#include "mma.h"

namespace llmc {

namespace {

struct AttnCfg {
  static constexpr int DH = 64, QB = 128, KT = 64, THREADS = 256;
  static constexpr int K_STRIDE = DH + 8;    // elements per K row in LDS (144 B: conflict-free 16-byte reads)
  static constexpr int V_STRIDE = KT + 4;    // elements per V^T row in LDS (136 B: conflict-free 8-byte reads)
  static constexpr int K_ELEMS = KT * K_STRIDE, V_ELEMS = DH * V_STRIDE;
};

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
constexpr int kMaxAttnGrid = 1024;   // four workgroups per compute unit; larger jobs walk the items with a grid stride

// maximum over the two lane halves (lane i and lane i ^ 32), in every lane
__device__ __forceinline__ float max_across_halves(float v) {
  const uint32_t u = __builtin_bit_cast(uint32_t, v);
  // the swap leaves one half's values in both halves of the first result and the other half's in the second
  const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__builtin_bit_cast(float, (uint32_t)sw[0]), __builtin_bit_cast(float, (uint32_t)sw[1]));
}

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
  // Causal: query block qb reads qb + 1 key blocks, so a work item is the PAIR (n_qb - 1 - x, x) of query blocks of
  // one (sequence, head): every item then costs the same number of key tiles and the grid stays balanced.
  const int per = CAUSAL ? (n_qb + 1) / 2 : n_qb;
  const int total = n_seq * n_heads * per;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
  const size_t ld = 3 * (size_t)d;
  // staging role of this thread, K: rows st_row and st_row + 32, dh chunk of 8
  const int st_row = tid >> 3, st_chunk = tid & 7;
  const int k_off = st_row * C::K_STRIDE + st_chunk * 8;
  // V: keys 2 * st_row and 2 * st_row + 1, dh chunk of 8; key group of four swizzled by the dh half
  const int v_key = ((((st_row >> 1) ^ ((st_chunk >> 2) * 4)) << 2) | ((st_row & 1) << 1));
  const int v_off = st_chunk * 8 * C::V_STRIDE + v_key;
  // fragment bases: K rows / V^T rows lane % 32, the lane half picks the second 8 (K) or 4 (V) of a k-step
  const int fk_off = (lane & 31) * C::K_STRIDE + half * 8;
  const int fv_off = (lane & 31) * C::V_STRIDE + half * 4;
  const bf16x2_t ones = {(__bf16)1.0f, (__bf16)1.0f};

  // one flat loop: step `it` of a workgroup is half it % 2 of its (it / 2)-th item (non-causal: every step an item)
  for (int it = 0;; ++it) {
    const int item = blockIdx.x + (CAUSAL ? it >> 1 : it) * gridDim.x;
    if (item >= total) break;
    const int x = item % per, head = (item / per) % n_heads, seq = item / (per * n_heads);
    const bool second = CAUSAL && (it & 1);
    if (second && n_qb - 1 - x == x) continue;                      // the middle block of an odd count pairs with itself
    const int qb = CAUSAL ? (second ? x : n_qb - 1 - x) : x;        // the longer block of a pair first
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

    f32x16_t o0, o1;
#pragma unroll
    for (int r = 0; r < 16; ++r) { o0[r] = 0.f; o1[r] = 0.f; }
    float m_run = -INFINITY, l_run = 0.f;

    uint4 rk0, rk1, rv0, rv1;
#define LLMC_ATTN_LOAD(T_)                                                                              \
    {                                                                                                   \
      const int ka_ = min((T_) * C::KT + st_row, S - 1), kb_ = min((T_) * C::KT + st_row + 32, S - 1);  \
      const int va_ = min((T_) * C::KT + 2 * st_row, S - 1), vb_ = min((T_) * C::KT + 2 * st_row + 1, S - 1); \
      rk0 = *reinterpret_cast<const uint4*>(base + (size_t)ka_ * ld + d + st_chunk * 8);                \
      rk1 = *reinterpret_cast<const uint4*>(base + (size_t)kb_ * ld + d + st_chunk * 8);                \
      rv0 = *reinterpret_cast<const uint4*>(base + (size_t)va_ * ld + 2 * d + st_chunk * 8);            \
      rv1 = *reinterpret_cast<const uint4*>(base + (size_t)vb_ * ld + 2 * d + st_chunk * 8);            \
    }
#define LLMC_ATTN_VPAIR(E_, A_, B_)                                                                              \
    *reinterpret_cast<uint32_t*>(&sV[buf_][v_off + (E_) * C::V_STRIDE]) = ((A_) & 0xFFFFu) | ((B_) << 16);       \
    *reinterpret_cast<uint32_t*>(&sV[buf_][v_off + ((E_) + 1) * C::V_STRIDE]) = ((A_) >> 16) | ((B_) & 0xFFFF0000u);
#define LLMC_ATTN_STORE(BUF_)                                                               \
    {                                                                                       \
      const int buf_ = (BUF_);                                                              \
      *reinterpret_cast<uint4*>(&sK[buf_][k_off]) = rk0;                                    \
      *reinterpret_cast<uint4*>(&sK[buf_][k_off + 32 * C::K_STRIDE]) = rk1;                 \
      LLMC_ATTN_VPAIR(0, rv0.x, rv1.x)                                                      \
      LLMC_ATTN_VPAIR(2, rv0.y, rv1.y)                                                      \
      LLMC_ATTN_VPAIR(4, rv0.z, rv1.z)                                                      \
      LLMC_ATTN_VPAIR(6, rv0.w, rv1.w)                                                      \
    }

    __syncthreads();            // the previous item's readers are done with both buffers
    LLMC_ATTN_LOAD(0)
    LLMC_ATTN_STORE(0)
    __syncthreads();

    for (int t = 0; t < n_tiles; ++t) {
      const int buf = t & 1;
      if (t + 1 < n_tiles) LLMC_ATTN_LOAD(t + 1)
      // a key tile that lies wholly behind this wavefront's 32 queries contributes nothing: only stage the next one
      const bool masked_out = CAUSAL && t * C::KT > q0 + wave * 32 + 31;
      if (!masked_out) {
      // ---- S^T = K * Q^T for 64 keys x 32 queries ----
      const uint16_t* kf = &sK[buf][fk_off];
      const f32x16_t zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      f32x16_t s0 = zero, s1 = zero;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const bf16x8_t fk0 = *reinterpret_cast<const bf16x8_t*>(kf + ks * 16);
        const bf16x8_t fk1 = *reinterpret_cast<const bf16x8_t*>(kf + 32 * C::K_STRIDE + ks * 16);
        s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk0, fq[ks], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk1, fq[ks], s1, 0, 0, 0);
      }
      // ---- online softmax over this lane's 32 keys (base-2 exponent, scale folded in) ----
      const int kv0 = t * C::KT;
      const bool edge = (kv0 + C::KT > S) || (CAUSAL && kv0 + C::KT > q0 + wave * 32);
      if (edge) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kv = kv0 + frag_row(lane, r);
          if (kv >= S || (CAUSAL && kv > q_lane)) s0[r] = -INFINITY;
          if (kv + 32 >= S || (CAUSAL && kv + 32 > q_lane)) s1[r] = -INFINITY;
        }
      }
      // the maximum is taken over the raw scores (the scale is positive), the scale enters the exponent as one fma
      float mx = fmaxf(s0[0], s1[0]);
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(fmaxf(mx, s0[r]), s1[r]);      // one three-way maximum each
      mx = max_across_halves(mx);
      const float m_new = fmaxf(m_run, mx * scale_log2e);          // finite: key 0 is visible to every query
      // the accumulators are rescaled only when some query of the wavefront met a larger score
      if (__any(m_new > m_run)) {
        const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
        l_run *= corr;
#pragma unroll
        for (int r = 0; r < 16; ++r) { o0[r] *= corr; o1[r] *= corr; }
      }
      m_run = m_new;
      uint32_t pk0[8], pk1[8];
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        pk0[r >> 1] = f32x2_to_bf16x2(__builtin_amdgcn_exp2f(fmaf(s0[r], scale_log2e, -m_new)),
                                      __builtin_amdgcn_exp2f(fmaf(s0[r + 1], scale_log2e, -m_new)));
        pk1[r >> 1] = f32x2_to_bf16x2(__builtin_amdgcn_exp2f(fmaf(s1[r], scale_log2e, -m_new)),
                                      __builtin_amdgcn_exp2f(fmaf(s1[r + 1], scale_log2e, -m_new)));
      }
      // row sum of the rounded probabilities, two per instruction
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pk0[e]), ones, l_run, false);
        l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pk1[e]), ones, l_run, false);
      }
      // ---- O^T += V^T * P^T : 4 k-steps of 16 keys, 2 fragments of 32 dh rows ----
      const uint16_t* vf = &sV[buf][fv_off];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        // keys of this k-step, in accumulator order: registers (ks % 2) * 8 .. + 8 of fragment ks / 2
        const int rb = (ks & 1) * 4;
        union { uint32_t u[4]; bf16x8_t v; } pb;
#pragma unroll
        for (int e = 0; e < 4; ++e) pb.u[e] = (ks >> 1) ? pk1[rb + e] : pk0[rb + e];
        // dh rows 0..31 keep the key groups in place, rows 32..63 have them XORed by 4 (one k-step over)
        union { uint2 u[2]; bf16x8_t v; } va, vb;
        va.u[0] = *reinterpret_cast<const uint2*>(vf + ks * 16);
        va.u[1] = *reinterpret_cast<const uint2*>(vf + ks * 16 + 8);
        vb.u[0] = *reinterpret_cast<const uint2*>(vf + 32 * C::V_STRIDE + (ks ^ 1) * 16);
        vb.u[1] = *reinterpret_cast<const uint2*>(vf + 32 * C::V_STRIDE + (ks ^ 1) * 16 + 8);
        o0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va.v, pb.v, o0, 0, 0, 0);
        o1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vb.v, pb.v, o1, 0, 0, 0);
      }
      }
      if (t + 1 < n_tiles) LLMC_ATTN_STORE(buf ^ 1)
      __syncthreads();
    }
#undef LLMC_ATTN_LOAD
#undef LLMC_ATTN_VPAIR
#undef LLMC_ATTN_STORE
    // ---- normalise and store: lane holds query q_lane, dh rows df * 32 + half * 4 + 8 g + i ----
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_tot;
    if (q_lane < S) {
      uint16_t* dst = ctx + ((size_t)seq * S + q_lane) * d + head * C::DH;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = f32x2_to_bf16x2(o0[4 * g] * inv, o0[4 * g + 1] * inv);
        w.y = f32x2_to_bf16x2(o0[4 * g + 2] * inv, o0[4 * g + 3] * inv);
        *reinterpret_cast<uint2*>(dst + half * 4 + 8 * g) = w;
        w.x = f32x2_to_bf16x2(o1[4 * g] * inv, o1[4 * g + 1] * inv);
        w.y = f32x2_to_bf16x2(o1[4 * g + 2] * inv, o1[4 * g + 3] * inv);
        *reinterpret_cast<uint2*>(dst + 32 + half * 4 + 8 * g) = w;
      }
    }
  }
}

}  // namespace

llmc_status_t launch_attention_bf16(const void* qkv, void* ctx, int S, int d, int n_heads, bool causal,
                                    const int32_t* count, int max_seqs, hipStream_t st) {
  if (d != n_heads * AttnCfg::DH) return LLMC_ERR_SHAPE;
  // base-2 softmax with log2(e) folded into the score scale
  const float scale_log2e = (1.0f / sqrtf((float)AttnCfg::DH)) * 1.4426950408889634f;
  const int n_qb = (S + AttnCfg::QB - 1) / AttnCfg::QB;
  const int items = (causal ? (n_qb + 1) / 2 : n_qb) * n_heads * max_seqs;   // causal: pairs of query blocks
  if (items <= 0) return LLMC_OK;
  const dim3 grid(std::min(items, kMaxAttnGrid));
  ProfScope ps_("attention_kernel", st);
  if (causal)
    LLMC_KERNEL_GGL(attention_mfma_kernel<true>, grid, dim3(AttnCfg::THREADS), 0, st, (const uint16_t*)qkv,
                    (uint16_t*)ctx, S, d, n_heads, scale_log2e, count, max_seqs);
  else
    LLMC_KERNEL_GGL(attention_mfma_kernel<false>, grid, dim3(AttnCfg::THREADS), 0, st, (const uint16_t*)qkv,
                    (uint16_t*)ctx, S, d, n_heads, scale_log2e, count, max_seqs);
  LLMC_LAUNCH_CHECK("attention");
  return LLMC_OK;
}

}  // namespace llmc
