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
#include "mma.h"

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

// ---- matrix-core variant: many queries, 256-bit keys ------------------------------------------------
// The number of common set bits of two keys is a dot product of their bits, and
//   H(q, b) = |q| + |b| - 2 * common(q, b),
// so the scan becomes an int8 matrix product (v_mfma_i32_32x32x32_i8) of bank rows by queries.
// Bank bits are expanded to bytes on their way into LDS, query bits in registers.  Bit j of a byte of
// the key becomes a byte of value 2^j on the bank side (one byte-replicating permute per eight bits and
// one AND per four) and -128 / 2^j on the query side (+1 for j = 7, where the bank byte reads as -128),
// so the product of two set bits is -128 wherever they sit, and an accumulator that STARTS at
//   start[row] = 64 * (|b_row| + penalty_row) + (row within its 64-row tile)
// ends at 64 * (H - |q|) + (row within the tile).  The smallest accumulator of a lane is therefore
// its nearest row, lowest row among equals, and the whole reduction is one three-way minimum per two
// scores; validity, the key's own popcount and the row number cost no instruction.
// A workgroup of 4 wavefronts owns 256 queries (64 per wavefront, fragments in registers) and a range
// of 64-row tiles; three workgroups share a compute unit so that one's expansion and reduction run
// under the others' matrix instructions.  The bank is read as bits (32 bytes per key).
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x16_t __attribute__((ext_vector_type(16)));

struct BitsMma {
  static constexpr int K = 256, W = 8, RB = 64, NW = 4, THREADS = NW * 64, QW = 64, QB = NW * QW;
  static constexpr int ROWB = K + 16;                    // one byte per bit; rows padded by one 16-byte chunk, so that
                                                         // the same chunk of 16 consecutive rows covers all banks
  static constexpr int TILE_BYTES = RB * ROWB;
  static constexpr int STAGE_BYTES = TILE_BYTES + RB * 4;   // + the tile's start words
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
  static constexpr int SCALE = 64;                       // accumulator units per bit of distance (two set bits: -128)
};

// start[j] for every row of the padded bank (n_pad: a whole number of tiles)
__global__ void bits_start_kernel(const uint32_t* __restrict__ bank, const uint8_t* __restrict__ valid, int N, int n_pad,
                                  int32_t* __restrict__ start) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n_pad) return;
  // rows past the end read the last key (as the scan does) and carry the penalty of a free slot
  const int jr = min(j, N - 1);
  const uint4* kp = reinterpret_cast<const uint4*>(bank + (size_t)jr * BitsMma::W);
  const uint4 a = kp[0], b = kp[1];
  uint32_t h = __builtin_popcount(a.x) + __builtin_popcount(a.y) + __builtin_popcount(a.z) + __builtin_popcount(a.w) +
               __builtin_popcount(b.x) + __builtin_popcount(b.y) + __builtin_popcount(b.z) + __builtin_popcount(b.w);
  if (j >= N || valid[j] == 0) h += kFreePenalty;
  start[j] = (int32_t)(h * BitsMma::SCALE + (uint32_t)(j & (BitsMma::RB - 1)));
}

// byte m of w -> two words of four bytes: byte j of `lo` holds bit j of that byte at its own position
// (value 2^j), byte j of `hi` holds bit 4 + j (value 2^(4 + j))
__device__ __forceinline__ void spread_byte(uint32_t w, int m, uint32_t& lo, uint32_t& hi) {
  const uint32_t r = __builtin_amdgcn_perm(w, w, 0x01010101u * (uint32_t)m);   // the byte, four times
  lo = r & 0x08040201u;
  hi = r & 0x80402010u;
}

// every non-zero byte -> 0xFF
__device__ __forceinline__ uint32_t bytes_to_mask(uint32_t x) {
  uint32_t m = 0;
#pragma unroll
  for (int b = 0; b < 4; ++b)
    if ((x >> (8 * b)) & 0xFFu) m |= 0xFFu << (8 * b);
  return m;
}

// grid: 1-D; workgroup -> (split, query block) as in the cosine kernels (the query blocks of a split on one XCD)
__global__ __launch_bounds__(BitsMma::THREADS, 3) void match_bits_mma_kernel(
    const uint32_t* __restrict__ bank, const int32_t* __restrict__ start, int N, const uint32_t* __restrict__ queries,
    int B, int n_qb, int n_split, int tiles_per_split, uint32_t* __restrict__ partial) {
  using C = BitsMma;
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_bits[];
  const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int split = (local / n_qb) * 8 + xcd, qb = local % n_qb;
  if (split >= n_split) return;
  const int n_tiles = (N + C::RB - 1) / C::RB;
  const int t_begin = split * tiles_per_split;
  const int t_end = min(n_tiles, t_begin + tiles_per_split);
  const int q_base = qb * C::QB + wave * C::QW;

  // query fragments: column (lane % 32) of fragment j; step ks covers bits 32 ks .. 32 ks + 31, this lane
  // half's 16 of them as 16 bytes
  i32x4_t bq[2][C::W];
  int pq[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int q = min(q_base + j * 32 + (lane & 31), B - 1);
    const uint4* qp = reinterpret_cast<const uint4*>(queries + (size_t)q * C::W);
    const uint4 a = qp[0], b = qp[1];
    const uint32_t w[C::W] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    pq[j] = 0;
#pragma unroll
    for (int ks = 0; ks < C::W; ++ks) {
      pq[j] += __builtin_popcount(w[ks]);
#pragma unroll
      for (int m = 0; m < 2; ++m) {
        uint32_t lo, hi;
        spread_byte(w[ks], 2 * half + m, lo, hi);
        // a set bit j of the byte: -128 / 2^j for j < 7, +1 for j = 7
        bq[j][ks][2 * m] = (int)(bytes_to_mask(lo) & 0xF0E0C080u);
        bq[j][ks][2 * m + 1] = (int)(bytes_to_mask(hi) & 0x01FEFCF8u);
      }
    }
  }

  // staging: thread (row, part) expands bits 64 part .. 64 part + 63 of tile row `row` into four 16-byte
  // chunks.  Lanes are dealt so that any 8 consecutive ones (4 rows x 2 parts) write 8 different chunk
  // positions and any 16 write 16.
  const int s_row = ((tid >> 1) & 3) | ((tid >> 4) << 2), s_part = (tid & 1) | (((tid >> 3) & 1) << 1);
  auto load_bits = [&](int t) {
    const int r = min(t * C::RB + s_row, N - 1);
    return *reinterpret_cast<const uint2*>(bank + (size_t)r * C::W + s_part * 2);
  };
  auto expand = [&](uint2 w, int sv, int stage) {
    uint8_t* st = lds_bits + stage * C::STAGE_BYTES;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t word = c < 2 ? w.x : w.y;
      uint32_t v0, v1, v2, v3;
      spread_byte(word, 2 * (c & 1), v0, v1);
      spread_byte(word, 2 * (c & 1) + 1, v2, v3);
      i32x4_t v;
      v[0] = (int)v0; v[1] = (int)v1; v[2] = (int)v2; v[3] = (int)v3;
      *reinterpret_cast<i32x4_t*>(st + s_row * C::ROWB + (s_part * 4 + c) * 16) = v;
    }
    if (tid < C::RB) *reinterpret_cast<int*>(st + C::TILE_BYTES + tid * 4) = sv;
  };
  // start has a whole number of tiles, so every thread's read is in bounds (only the first 64 are used)
  expand(load_bits(t_begin), start[(size_t)t_begin * C::RB + lane], 0);
  uint2 nb = make_uint2(0u, 0u);
  int nsv = 0;
  if (t_begin + 1 < t_end) {
    nb = load_bits(t_begin + 1);
    nsv = start[(size_t)(t_begin + 1) * C::RB + lane];
  }

  int best_v[2] = {0x7FFFFFFF, 0x7FFFFFFF}, best_row[2] = {0, 0};
  const int frag_off = (lane & 31) * C::ROWB + half * 16;

  for (int t = t_begin; t < t_end; ++t) {
    const int cur = (t - t_begin) & 1;
    LLMC_WAIT_LGKM(0);                     // this thread's part of tile t is in LDS
    dma::barrier();                        // ... and everybody's; the other stage is no longer read
    if (t + 1 < t_end) {
      expand(nb, nsv, cur ^ 1);
      if (t + 2 < t_end) {
        nb = load_bits(t + 2);
        nsv = start[(size_t)(t + 2) * C::RB + lane];
      }
    }
    const uint8_t* stg = lds_bits + cur * C::STAGE_BYTES;
    const int* sst = reinterpret_cast<const int*>(stg + C::TILE_BYTES);
    i32x16_t acc[2][2];
    i32x16_t c0[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const i32x4_t v = *reinterpret_cast<const i32x4_t*>(sst + i * 32 + half * 4 + 8 * c);
        c0[i][4 * c] = v[0]; c0[i][4 * c + 1] = v[1]; c0[i][4 * c + 2] = v[2]; c0[i][4 * c + 3] = v[3];
      }
    // bank fragments of step ks + 1 are requested before step ks multiplies
    i32x4_t fa[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
      fa[0][i] = *reinterpret_cast<const i32x4_t*>(stg + i * 32 * C::ROWB + frag_off);
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
    for (int ks = 0; ks < C::W; ++ks) {
      const int c = ks & 1, n = c ^ 1;
      // the fragments of this step were requested one step ago: wait for them BEFORE requesting the next
      // ones, so that the wait does not cover a request that has only just been issued
      __builtin_amdgcn_sched_barrier(0);
      LLMC_WAIT_LGKM(0);
      __builtin_amdgcn_sched_barrier(0);
      if (ks + 1 < C::W) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
          fa[n][i] = *reinterpret_cast<const i32x4_t*>(stg + i * 32 * C::ROWB + frag_off + (ks + 1) * 32);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[c][i], bq[j][ks], ks == 0 ? c0[i] : acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      int m = min(acc[0][j][0], acc[1][j][0]);
#pragma unroll
      for (int r = 1; r < 16; ++r) m = min(min(m, acc[0][j][r]), acc[1][j][r]);
      // tiles ascend: a strictly smaller distance wins, so the lowest row is kept among equals
      const int v = m >> 6;                  // SCALE = 64
      if (v < best_v[j]) {
        best_v[j] = v;
        best_row[j] = t * C::RB + (m & (C::SCALE - 1));
      }
    }
  }
  // the two lane halves saw different rows of the same query column
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int ov = __shfl_xor(best_v[j], 32, 64), orow = __shfl_xor(best_row[j], 32, 64);
    if (ov < best_v[j] || (ov == best_v[j] && orow < best_row[j])) {
      best_v[j] = ov;
      best_row[j] = orow;
    }
    const int q = q_base + j * 32 + (lane & 31);
    if (half == 0 && q < B) {
      const uint32_t h = (uint32_t)(pq[j] + best_v[j]);     // the distance (+ the penalty of a free slot)
      partial[(size_t)split * B + q] = (h << 20) | (uint32_t)(best_row[j] - t_begin * C::RB);
    }
  }
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

// the matrix-core scan pays once a query block fills its workgroups and the bank is worth the set-up
static bool bits_use_mma(int N, int k, int B) { return k == BitsMma::K && B >= 2 * BitsMma::QB && N >= 4096; }

static void bits_mma_plan(int N, int B, int* n_qb, int* n_split, int* tiles_per_split) {
  const int qb = (B + BitsMma::QB - 1) / BitsMma::QB;
  const int n_tiles = (N + BitsMma::RB - 1) / BitsMma::RB;
  int want = (3072 + qb - 1) / qb;                          // four rounds of three workgroups per compute unit
  want = (want + 7) / 8 * 8;                                // splits are dealt to the 8 XCDs
  if (want > n_tiles) want = n_tiles;
  int per = (n_tiles + want - 1) / want;
  if (per * BitsMma::RB > (1 << 20)) per = (1 << 20) / BitsMma::RB;
  *n_qb = qb;
  *tiles_per_split = per;
  *n_split = (n_tiles + per - 1) / per;
}

size_t match_bits_ws_bytes(int N, int k, int B) {
  int ns, per;
  bits_plan(N, B, &ns, &per);
  size_t words = (size_t)N + kRowUnroll;
  if (bits_use_mma(N, k, B)) {
    int nqb, ns2, tps;
    bits_mma_plan(N, B, &nqb, &ns2, &tps);
    if (ns2 > ns) ns = ns2;
    words = (size_t)N + BitsMma::RB;
  }
  return align_up((size_t)ns * B * sizeof(uint32_t), 256) + align_up(words * sizeof(uint32_t), 256);
}

static llmc_status_t launch_match_bits_mma(const uint32_t* d_bank_bits, const uint8_t* d_valid, int N, int k,
                                           const uint32_t* d_query_bits, int B, int max_hamming, int32_t* d_idx,
                                           int32_t* d_dist, uint8_t* d_hit, void* ws, hipStream_t st, float* d_sim) {
  using C = BitsMma;
  int nqb, ns, tps;
  bits_mma_plan(N, B, &nqb, &ns, &tps);
  uint32_t* partial = (uint32_t*)ws;
  int32_t* start = (int32_t*)((char*)ws + align_up((size_t)ns * B * sizeof(uint32_t), 256));
  const int n_pad = (N + C::RB - 1) / C::RB * C::RB;
  { ProfScope ps_("bits_start_kernel", st);
    LLMC_KERNEL_GGL(bits_start_kernel, dim3((n_pad + 255) / 256), dim3(256), 0, st, d_bank_bits, d_valid, N, n_pad,
                    start); }
  LLMC_LAUNCH_CHECK("bits_start_kernel");
  const int grid = (ns + 7) / 8 * 8 * nqb;
  { ProfScope ps_("match_bits_mma_kernel", st);
    LLMC_KERNEL_GGL(match_bits_mma_kernel, dim3(grid), dim3(C::THREADS), (size_t)C::LDS_BYTES, st, d_bank_bits, start,
                    N, d_query_bits, B, nqb, ns, tps, partial); }
  LLMC_LAUNCH_CHECK("match_bits_mma_kernel");
  { ProfScope ps_("match_bits_finalize_kernel", st);
    LLMC_KERNEL_GGL(match_bits_finalize_kernel, dim3((B + 255) / 256), dim3(256), 0, st, partial, ns, tps * C::RB, B,
                    max_hamming, d_idx, d_dist, d_hit, d_sim, k); }
  LLMC_LAUNCH_CHECK("match_bits_finalize_kernel");
  return LLMC_OK;
}

// d_pen: ready-made penalty words [N + kRowUnroll] (a bank's mirror), or NULL to derive them from d_valid into ws.
// The matrix-core scan derives its own start words from d_valid into ws and is taken only when the caller sized
// ws with match_bits_ws_bytes (d_pen == NULL).
llmc_status_t launch_match_bits(const uint32_t* d_bank_bits, const uint8_t* d_valid, int N, int k,
                                const uint32_t* d_query_bits, int B, int max_hamming, int32_t* d_idx, int32_t* d_dist,
                                uint8_t* d_hit, void* ws, hipStream_t st, const uint32_t* d_pen, float* d_sim) {
  const bool aligned16 = (((uintptr_t)d_bank_bits | (uintptr_t)d_query_bits) & 15) == 0;   // 16-byte key reads
  if (!d_pen && aligned16 && bits_use_mma(N, k, B))
    return launch_match_bits_mma(d_bank_bits, d_valid, N, k, d_query_bits, B, max_hamming, d_idx, d_dist, d_hit, ws, st,
                                 d_sim);
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
