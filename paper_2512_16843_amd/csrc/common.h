// Internal helpers shared by the llmc kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <atomic>
#include <stdint.h>
#include <stddef.h>
#include <math.h>
#include "../../include/llmc.h"

namespace llmc {

// ---- element types ---------------------------------------------------------
// bf16 values travel as raw 16-bit patterns; arithmetic is always fp32.
struct bf16_t {
  uint16_t bits;
};

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}
// round to nearest, ties to even; NaN stays NaN.  Written as conversions to the compiler's bfloat type, which
// gfx950 performs in hardware, two values per instruction (same bits as the integer add-and-shift formula,
// ties, infinities and denormals included).
typedef __bf16 llmc_bf16x2_t __attribute__((ext_vector_type(2)));
typedef float llmc_f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
  const llmc_f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, llmc_bf16x2_t));
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kVec = 4;  // elements per 16-byte vector
  __device__ static __forceinline__ float load(const float* p) { return *p; }
  __device__ static __forceinline__ void store(float* p, float v) { *p = v; }
  __device__ static __forceinline__ float round(float v) { return v; }
};
template <> struct Elem<bf16_t> {
  static constexpr int kVec = 8;
  __device__ static __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(p->bits); }
  __device__ static __forceinline__ void store(bf16_t* p, float v) { p->bits = f32_to_bf16(v); }
  __device__ static __forceinline__ float round(float v) { return bf16_to_f32(f32_to_bf16(v)); }
};

// 16-byte vector of T unpacked to fp32
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  __device__ static __forceinline__ void load(const float* p, float* out) {
    float4 v = *reinterpret_cast<const float4*>(p);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
  }
  __device__ static __forceinline__ void store(float* p, const float* in) {
    *reinterpret_cast<float4*>(p) = make_float4(in[0], in[1], in[2], in[3]);
  }
};
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  __device__ static __forceinline__ void load(const bf16_t* p, float* out) {
    uint4 v = *reinterpret_cast<const uint4*>(p);
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = __uint_as_float(w[i] << 16);
      out[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
  }
  __device__ static __forceinline__ void store(bf16_t* p, const float* in) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = f32x2_to_bf16x2(in[2 * i], in[2 * i + 1]);
    *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
  }
};

// ---- wavefront (64 lanes) reductions with a fixed order -------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---- host-side error plumbing ------------------------------------------------------
llmc_status_t set_error(llmc_status_t st, const char* fmt, ...);
llmc_status_t hip_error(hipError_t e, const char* what);

#define LLMC_HIP(call)                                   \
  do {                                                   \
    hipError_t e_ = (call);                              \
    if (e_ != hipSuccess) return hip_error(e_, #call);   \
  } while (0)
#define LLMC_LAUNCH_CHECK(what)                          \
  do {                                                   \
    hipError_t e_ = hipGetLastError();                   \
    if (e_ != hipSuccess) return hip_error(e_, what);    \
  } while (0)
#define LLMC_KERNEL_GGL(KERNEL, GRID, BLOCK, LDS, ST, ...)                                              \
  do {                                                                                                   \
    ::llmc::ProfScope* p_ = ::llmc::prof_current();                                                      \
    if (p_ && p_->rec >= 0)                                                                              \
      hipExtLaunchKernelGGL(KERNEL, GRID, BLOCK, (std::uint32_t)(LDS), ST, p_->a, p_->b, 0, __VA_ARGS__); \
    else                                                                                                 \
      hipLaunchKernelGGL(KERNEL, GRID, BLOCK, LDS, ST, __VA_ARGS__);                                     \
  } while (0)
#define LLMC_TRY(expr)                                   \
  do {                                                   \
    llmc_status_t s_ = (expr);                           \
    if (s_ != LLMC_OK) return s_;                        \
  } while (0)

// Optional per-kernel timing.  A ProfScope names the launch that follows it; while recording is on it claims a pair
// of events, and LLMC_KERNEL_GGL hands them to the launch itself (hipExtLaunchKernelGGL), so that the pair carries
// the start and the end of that kernel's execution on the device -- the duration a kernel trace reports -- and
// not the gaps between dispatches.  One launch per scope.
struct ProfScope {
  ProfScope(const char* name, hipStream_t st);
  ~ProfScope();
  int rec;
  hipEvent_t a, b;
  ProfScope* outer;
};
ProfScope* prof_current();

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline size_t elem_size(int dtype) { return dtype == LLMC_F32 ? 4 : 2; }

// ---- the bank object ------------------------------------------------------------------
}  // namespace llmc

namespace llmc {
// Raise a kernel's dynamic-LDS limit once per device (the setting is per function AND per device).
// `done` is a per-call-site table; calls on one device from several host threads at once may set it twice, harmlessly.
inline llmc_status_t ensure_dynamic_lds(const void* fn, size_t bytes, std::atomic<bool>* done) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
  if (done[dev].load(std::memory_order_acquire)) return LLMC_OK;
  hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e != hipSuccess) return hip_error(e, "hipFuncSetAttribute(MaxDynamicSharedMemorySize)");
  done[dev].store(true, std::memory_order_release);
  return LLMC_OK;
}
}  // namespace llmc

struct llmc_bank {
  llmc_bank_desc_t desc;
  // Library-owned mirror [n_slots]: inv_norm of valid slots, NaN for free ones.  The match
  // epilogue multiplies scores by it and takes maxima with NaN-ignoring max, so free
  // slots never win and never mask a valid entry.
  float* d_binv_eff;
  int device;
  int64_t epoch;      // DECAYED_HITS: tick / half_life of the latest update (host side, in call order)
  // compressed values: library-owned transpose [d, rank] of the basis, and a list of value rows per hit (65536 entries)
  void* d_basis_t;
  int32_t* d_hit_slots;
};

namespace llmc {

// ---- kernel launchers (one per translation unit) ------------------------------------------
// fingerprint.hip
size_t fingerprint_ws_bytes(int B, int S, int d);
llmc_status_t launch_fingerprint(const void* d_h, const int32_t* d_rowmap_unused, int B, int S, int d, int dtype,
                                 const void* d_proj, const float* d_bias, int k, void* d_fp, float* d_inv, void* ws,
                                 hipStream_t st, const float* pooled_in = nullptr,
                                 const uint8_t* pooled_valid = nullptr, const void* key_in = nullptr,
                                 const float* key_inv_in = nullptr, bool few_uncarried = false,
                                 const int32_t* key_index = nullptr);
llmc_status_t launch_project_rows(const float* d_means, int n_max, int d, int dtype, const void* d_proj,
                                  const float* d_bias, int k, const int32_t* d_rows, const int32_t* d_count, void* d_fp,
                                  float* d_inv, hipStream_t st);
// token means of B whole sequences, wide form (ws_partials: fingerprint_ws_bytes(B, S, d) bytes), same bits as above
llmc_status_t launch_pool_means(const void* d_h, int B, int S, int d, int dtype, void* ws_partials, float* d_out,
                                int ld_out, hipStream_t st);
// ld_out: floats between consecutive output rows (0: d)
llmc_status_t launch_pool_rows(const void* d_h, int n_max, int S, int d, int dtype, const int32_t* d_rows,
                               const int32_t* d_count, const int32_t* d_dst, float* d_out, hipStream_t st,
                               int ld_out = 0);
llmc_status_t launch_fingerprint_bits(const void* d_h, int B, int S, int d, int dtype, const void* d_proj,
                                      const float* d_bias, int k, uint32_t* d_bits, void* ws, hipStream_t st,
                                      const float* pooled_in = nullptr, const uint8_t* pooled_valid = nullptr,
                                      bool few_uncarried = false);
size_t match_bits_ws_bytes(int N, int k, int B);
size_t lsh_index_bytes(int N, int k);
// d_changed (optional, device): the index is left as it is when *d_changed == 0
llmc_status_t launch_lsh_build(const uint32_t* d_bank_bits, const uint8_t* d_valid, int N, int k, void* d_index,
                               hipStream_t st, const int32_t* d_changed = nullptr);
llmc_status_t launch_lsh_match(const uint32_t* d_bank_bits, int N, int k, const void* d_index,
                               const uint32_t* d_query_bits, int B, int max_hamming, int32_t* d_idx, int32_t* d_dist,
                               uint8_t* d_hit, int32_t* d_compared, hipStream_t st, float* d_sim = nullptr);
llmc_status_t launch_match_bits(const uint32_t* d_bank_bits, const uint8_t* d_valid, int N, int k,
                                const uint32_t* d_query_bits, int B, int max_hamming, int32_t* d_idx, int32_t* d_dist,
                                uint8_t* d_hit, void* ws, hipStream_t st, const uint32_t* d_pen = nullptr,
                                float* d_sim = nullptr);
llmc_status_t launch_inv_norm(const void* d_fp, int64_t n, int k, int dtype, float* d_out, hipStream_t st);

// match.hip
size_t match_ws_bytes(int n_slots, int k, int dtype, int B);
size_t match_ws_max_bytes(int B);
llmc_status_t launch_match(const llmc_bank* bank, const void* d_fp, const float* d_inv, int B, float tau,
                           int32_t* d_idx, float* d_sim, uint8_t* d_hit, uint8_t* d_near_tie, void* ws,
                           hipStream_t st);

llmc_status_t match_static_scratch(void** out, size_t* bytes);

// gate.hip
llmc_status_t launch_compact(const uint8_t* d_hit, const int32_t* d_idx, const float* d_sim,
                             const uint8_t* d_near_tie, int B, float tau, int32_t* d_hit_rows,
                             int32_t* d_miss_rows, int32_t* d_reval_tmp, int32_t* d_counters, llmc_bank* bank,
                             uint32_t flags, uint64_t tick, hipStream_t st, uint8_t* d_pooled_valid_out = nullptr,
                             int has_pool = 0, int32_t* d_ref_out = nullptr);
// within-batch reuse (LLMC_DEDUP): scratch size, the decision among the rows to compute (before the dense block),
// and the copies / bookkeeping of the followers (after the insertion)
size_t dedup_ws_bytes(int B);
llmc_status_t launch_dedup_resolve(const void* d_keys, const float* d_inv, int k, int dtype, int B, float tau,
                                   int32_t* d_miss_rows, int32_t* d_counters, void* ws, hipStream_t st);
llmc_status_t launch_dedup_finish(llmc_bank* bank, void* d_h_out, int B, const int32_t* d_slots, int32_t* d_idx,
                                  float* d_sim, uint8_t* d_hit, int32_t* d_counters, uint32_t flags, void* ws,
                                  hipStream_t st);
llmc_status_t launch_materialize(const llmc_bank* bank, const int32_t* d_ref, const int32_t* d_rows, const int32_t* d_n,
                                 int n_max, void* d_h, hipStream_t st);
llmc_status_t launch_divergence(llmc_bank* bank, const void* d_h_out, const int32_t* d_idx, const int32_t* d_rows,
                                int32_t* d_counters, int B, hipStream_t st);
llmc_status_t launch_all_miss(int B, int32_t* d_miss_rows, int32_t* d_counters, int32_t* d_idx, float* d_sim,
                              uint8_t* d_hit, hipStream_t st, uint8_t* d_pooled_valid_out = nullptr);
llmc_status_t launch_gather(const llmc_bank* bank, const int32_t* d_idx, const int32_t* d_rows,
                            const int32_t* d_n, int n_max, void* d_h_out, hipStream_t st,
                            float* d_pooled_out = nullptr, void* d_key_out = nullptr, float* d_key_inv_out = nullptr);

// bank.hip
llmc_status_t launch_bank_refresh(llmc_bank* bank, hipStream_t st);
llmc_status_t launch_transpose(const void* in, void* out, int r, int d, int e, hipStream_t st);
// DECAYED_HITS: halve the hit counts once per epoch gone by since the bank's latest update
llmc_status_t launch_bank_advance(llmc_bank* bank, uint64_t tick, hipStream_t st);
llmc_status_t launch_bank_insert(llmc_bank* bank, const void* d_fp, const float* d_inv, const void* d_act,
                                 const int32_t* d_rows, const int32_t* d_m, int m_max, uint64_t tick,
                                 int32_t* d_slots_out, int32_t* d_counters, hipStream_t st);
llmc_status_t launch_bank_evict(llmc_bank* bank, const int32_t* d_m, int m_max, int32_t* d_victims,
                                hipStream_t st);

// layer.hip
struct LayerWs {
  void* qkv;   // [T, 3d]
  void* ctx;   // [T, d]
  void* t0;    // [T, d]
  void* t1;    // [T, d]
  void* ff;    // [T, d_ff]
};
size_t layer_ws_bytes(const llmc_layer_desc_t* L, int B, int S);
// Computes f_l for the sequences listed in d_rows[0 .. *d_count) of d_h_in and writes each
// result to the same row of d_h_out.  d_count / d_rows live on the device.
// out[o_rows] = A[a_rows] * W^T (+ bias): the layer's GEMM on plain arguments (W [N, K], K contiguous; sequences of S rows)
llmc_status_t launch_linear(const void* A, int lda, const int32_t* a_rows, const void* W, const void* bias, int N, int K,
                            void* out, int ldo, const int32_t* o_rows, int S, const int32_t* count, int max_seqs,
                            int dtype, hipStream_t st);
// pool_partial / pooled_flags (both or neither): the block's last LayerNorm also leaves the chunk sums of its
// outputs in the fingerprint's partials buffer and sets pooled_flags[row] = 2 (post-LayerNorm blocks whose rows fit)
// bf16 softmax attention on the matrix cores (head size 64): qkv [T, 3d] -> ctx [T, d]; sequences beyond *count skipped
llmc_status_t launch_attention_bf16(const void* qkv, void* ctx, int S, int d, int n_heads, bool causal,
                                    const int32_t* count, int max_seqs, hipStream_t st);
// Section IV-B, prefix attention statistics: the block's self-attention sub-layer run over the first n_prefix tokens of
// every sequence alone; the mean of its outputs over those tokens goes to out[b * ld_out ..] [d] fp32
size_t prefix_attention_ws_bytes(const llmc_layer_desc_t* L, int B, int n_prefix);
llmc_status_t launch_prefix_attention_mean(const llmc_layer_desc_t* L, const void* d_h, int B, int S, int n_prefix,
                                           void* ws, float* d_out, int ld_out, hipStream_t st);
llmc_status_t launch_layer(const llmc_layer_desc_t* L, const void* d_h_in, void* d_h_out, int B, int S,
                           const int32_t* d_rows, const int32_t* d_count, void* ws, hipStream_t st,
                           float* pool_partial = nullptr, uint8_t* pooled_flags = nullptr);

}  // namespace llmc
