// Hamming match of sign-bit keys (Section IV-B: SimHash keys, compared by cosine similarity or by
// LSH; Section III-A: hashing keeps the comparison cheap): for each query key the
// valid bank key at the smallest Hamming distance H, lowest slot among equals.  cos(pi H / k) stands
// for the cosine of the case equation, so the threshold becomes H <= max_hamming.
//
// Integer ALU work (XOR + popcount), laid out so that it costs two vector instructions per 32 bit
// pairs and nothing else:
//   * a lane owns ONE query key, held in registers for the whole kernel (k / 32 words);
//   * bank keys are the same for every lane, so they are read through the scalar data path (uniform
//     addresses, read-only) and enter the XOR as scalar operands: no LDS, no vector loads;
//   * the popcount instruction adds into an accumulator; its start value is a per-slot penalty word
//     (0 for a valid slot, 2048 for a free one), so validity costs no instruction;
//   * (H << 20 | row within the split) is one 32-bit key, so the running best -- and the lowest slot
//     among equal distances -- is a single unsigned minimum.
// A workgroup of 4 wavefronts owns 256 queries and a range of at most 2^20 bank rows; a second
// kernel merges the ranges per query in ascending row order.
#include "common.h"

namespace llmc {

constexpr uint32_t kFreePenalty = 2048;      // above any distance of keys of at most 1024 bits
constexpr int kBitsThreads = 256;
constexpr int kRowUnroll = 8;

// pen[j] = 0 for a valid slot, kFreePenalty for a free one and for the padding up to n_pad
__global__ void bits_penalty_kernel(const uint8_t* __restrict__ valid, int N, int n_pad, uint32_t* __restrict__ pen) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < n_pad) pen[j] = (j < N && valid[j] != 0) ? 0u : kFreePenalty;
}

// grid (n_split, query blocks)
template <int W>
__global__ __launch_bounds__(kBitsThreads) void match_bits_kernel(const uint32_t* __restrict__ bank,
                                                                  const uint32_t* __restrict__ pen, int N,
                                                                  const uint32_t* __restrict__ queries, int B,
                                                                  int rows_per_split, uint32_t* __restrict__ partial) {
  const int b = min((int)(blockIdx.y * kBitsThreads + threadIdx.x), B - 1);
  uint32_t q[W];
#pragma unroll
  for (int w = 0; w < W; ++w) q[w] = queries[(size_t)b * W + w];
  const int r0 = blockIdx.x * rows_per_split;
  const int r1 = min(N, r0 + rows_per_split);
  uint32_t best = 0xFFFFFFFFu;
  for (int r = r0; r < r1; r += kRowUnroll) {
    // rows past the end are clamped for the key read and carry the penalty of the padding (pen has N + kRowUnroll
    // entries and r is a multiple of kRowUnroll)
    uint32_t key[kRowUnroll];
#pragma unroll
    for (int u = 0; u < kRowUnroll; ++u) {
      const int row = r + u;
      const uint32_t* kp = bank + (size_t)min(row, N - 1) * W;
      uint32_t h = pen[row];
#pragma unroll
      for (int w = 0; w < W; ++w) h = __builtin_popcount(q[w] ^ kp[w]) + h;
      key[u] = (h << 20) | (uint32_t)(row - r0);
    }
#pragma unroll
    for (int u = 0; u < kRowUnroll; ++u) best = min(best, key[u]);
  }
  const int bq = blockIdx.y * kBitsThreads + threadIdx.x;
  if (bq < B) partial[(size_t)blockIdx.x * B + bq] = best;
}

// generic key length: words in a loop (same scheme, query words re-read from registers is not possible, so LDS)
__global__ __launch_bounds__(kBitsThreads) void match_bits_generic_kernel(const uint32_t* __restrict__ bank,
                                                                          const uint32_t* __restrict__ pen, int N, int W,
                                                                          const uint32_t* __restrict__ queries, int B,
                                                                          int rows_per_split,
                                                                          uint32_t* __restrict__ partial) {
  extern __shared__ uint32_t sq[];               // [W][kBitsThreads]: word w of this lane's query
  const int b = min((int)(blockIdx.y * kBitsThreads + threadIdx.x), B - 1);
  for (int w = 0; w < W; ++w) sq[w * kBitsThreads + threadIdx.x] = queries[(size_t)b * W + w];
  const int r0 = blockIdx.x * rows_per_split;
  const int r1 = min(N, r0 + rows_per_split);
  uint32_t best = 0xFFFFFFFFu;
  for (int row = r0; row < r1; ++row) {
    const uint32_t* kp = bank + (size_t)row * W;
    uint32_t h = pen[row];
    for (int w = 0; w < W; ++w) h = __builtin_popcount(sq[w * kBitsThreads + threadIdx.x] ^ kp[w]) + h;
    best = min(best, (h << 20) | (uint32_t)(row - r0));
  }
  const int bq = blockIdx.y * kBitsThreads + threadIdx.x;
  if (bq < B) partial[(size_t)blockIdx.x * B + bq] = best;
}

// one thread per query: merge the splits in ascending row order (a strictly smaller distance wins, so the
// lowest slot is kept among equals), then apply the threshold
__global__ void match_bits_finalize_kernel(const uint32_t* __restrict__ partial, int n_split, int rows_per_split, int B,
                                           int max_hamming, int32_t* __restrict__ idx_out,
                                           int32_t* __restrict__ dist_out, uint8_t* __restrict__ hit_out,
                                           float* __restrict__ sim_out, int k) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  uint32_t best_h = 0xFFFFFFFFu;
  int best_row = -1;
  constexpr int U = 8;
  for (int s0 = 0; s0 < n_split; s0 += U) {
    uint32_t k[U];
#pragma unroll
    for (int u = 0; u < U; ++u) k[u] = s0 + u < n_split ? partial[(size_t)(s0 + u) * B + b] : 0xFFFFFFFFu;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t h = k[u] >> 20;
      if (s0 + u < n_split && h < best_h) {
        best_h = h;
        best_row = (s0 + u) * rows_per_split + (int)(k[u] & 0xFFFFFu);
      }
    }
  }
  const bool found = best_row >= 0 && best_h < kFreePenalty;
  idx_out[b] = found ? best_row : -1;
  if (dist_out) dist_out[b] = found ? (int32_t)best_h : 0x7FFFFFFF;
  if (hit_out) hit_out[b] = (found && (int32_t)best_h <= max_hamming) ? 1 : 0;
  // the cosine that the distance stands for (informative: the decision above is the integer one)
  if (sim_out) sim_out[b] = found ? cosf(3.14159265358979323846f * (float)best_h / (float)k) : -INFINITY;
}

static void bits_plan(int N, int B, int* n_split, int* rows_per_split) {
  const int qb = (B + kBitsThreads - 1) / kBitsThreads;
  int want = (2048 + qb - 1) / qb;                          // about eight workgroups per compute unit
  const int max_split = (N + 63) / 64;
  if (want > max_split) want = max_split;
  if (want < 1) want = 1;
  int per = (N + want - 1) / want;
  per = (per + kRowUnroll - 1) / kRowUnroll * kRowUnroll;
  if (per > (1 << 20)) per = 1 << 20;
  *rows_per_split = per;
  *n_split = (N + per - 1) / per;
}

size_t match_bits_ws_bytes(int N, int k, int B) {
  int ns, per;
  bits_plan(N, B, &ns, &per);
  return align_up((size_t)ns * B * sizeof(uint32_t), 256) + align_up((size_t)(N + kRowUnroll) * sizeof(uint32_t), 256);
}

// d_pen: ready-made penalty words [N + kRowUnroll] (a bank's mirror), or NULL to derive them from d_valid into ws
llmc_status_t launch_match_bits(const uint32_t* d_bank_bits, const uint8_t* d_valid, int N, int k,
                                const uint32_t* d_query_bits, int B, int max_hamming, int32_t* d_idx, int32_t* d_dist,
                                uint8_t* d_hit, void* ws, hipStream_t st, const uint32_t* d_pen, float* d_sim) {
  int ns, per;
  bits_plan(N, B, &ns, &per);
  uint32_t* partial = (uint32_t*)ws;
  const uint32_t* pen = d_pen;
  if (!pen) {
    uint32_t* mine = (uint32_t*)((char*)ws + align_up((size_t)ns * B * sizeof(uint32_t), 256));
    const int n_pad = N + kRowUnroll;
    { ProfScope ps_("bits_penalty_kernel", st);
      LLMC_KERNEL_GGL(bits_penalty_kernel, dim3((n_pad + 255) / 256), dim3(256), 0, st, d_valid, N, n_pad, mine); }
    LLMC_LAUNCH_CHECK("bits_penalty_kernel");
    pen = mine;
  }
  const int W = k / 32;
  dim3 grid(ns, (B + kBitsThreads - 1) / kBitsThreads);
  {
    ProfScope ps_("match_bits_kernel", st);
#define LLMC_BITS_CASE(W_) LLMC_KERNEL_GGL(match_bits_kernel<W_>, grid, dim3(kBitsThreads), 0, st, d_bank_bits, pen, \
                                              N, d_query_bits, B, per, partial)
    if (W == 2) LLMC_BITS_CASE(2);
    else if (W == 4) LLMC_BITS_CASE(4);
    else if (W == 8) LLMC_BITS_CASE(8);
    else if (W == 16) LLMC_BITS_CASE(16);
    else
      LLMC_KERNEL_GGL(match_bits_generic_kernel, grid, dim3(kBitsThreads), (size_t)W * kBitsThreads * sizeof(uint32_t),
                         st, d_bank_bits, pen, N, W, d_query_bits, B, per, partial);
#undef LLMC_BITS_CASE
  }
  LLMC_LAUNCH_CHECK("match_bits_kernel");
  { ProfScope ps_("match_bits_finalize_kernel", st);
    LLMC_KERNEL_GGL(match_bits_finalize_kernel, dim3((B + 255) / 256), dim3(256), 0, st, partial, ns, per, B,
                       max_hamming, d_idx, d_dist, d_hit, d_sim, k); }
  LLMC_LAUNCH_CHECK("match_bits_finalize_kernel");
  return LLMC_OK;
}

}  // namespace llmc
