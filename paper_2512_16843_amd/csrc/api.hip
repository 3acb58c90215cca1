// C ABI of libllmc.so: argument validation (before any HIP call) and the host-side
// orchestration of the gated layer, which only enqueues kernels on the caller's stream.
#include <algorithm>
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include <atomic>
#include <map>
#include <new>
#include <string>
#include <vector>
#include "common.h"

namespace llmc {

static thread_local char g_err[512] = "";

llmc_status_t set_error(llmc_status_t st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}
llmc_status_t hip_error(hipError_t e, const char* what) {
  return set_error(LLMC_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

// ---- per-kernel event timing ---------------------------------------------------------------
struct ProfRec { const char* name; hipEvent_t a, b; };
static std::vector<ProfRec> g_prof;
static std::atomic<int> g_prof_used{0};
static std::atomic<bool> g_prof_on{false};

static thread_local ProfScope* g_prof_cur = nullptr;
ProfScope* prof_current() { return g_prof_cur; }

ProfScope::ProfScope(const char* name, hipStream_t) : rec(-1), a(nullptr), b(nullptr), outer(g_prof_cur) {
  g_prof_cur = this;
  if (!g_prof_on.load(std::memory_order_relaxed)) return;
  const int i = g_prof_used.fetch_add(1);
  if (i >= (int)g_prof.size()) return;
  g_prof[i].name = name;
  a = g_prof[i].a;
  b = g_prof[i].b;
  rec = i;
}
ProfScope::~ProfScope() { g_prof_cur = outer; }

static bool dtype_ok(int dt) { return dt == LLMC_F32 || dt == LLMC_BF16; }

#define REQUIRE(cond, st, ...)                      \
  do {                                              \
    if (!(cond)) return set_error(st, __VA_ARGS__); \
  } while (0)

static llmc_status_t check_layer(const llmc_layer_desc_t* L) {
  REQUIRE(L, LLMC_ERR_INVALID_ARG, "layer descriptor is NULL");
  REQUIRE(dtype_ok(L->dtype), LLMC_ERR_DTYPE, "layer dtype %d unknown", L->dtype);
  REQUIRE(L->arch == 0 || L->arch == 1, LLMC_ERR_INVALID_ARG, "layer arch %d unknown", L->arch);
  REQUIRE(L->gelu == 0 || L->gelu == 1, LLMC_ERR_INVALID_ARG, "gelu kind %d unknown", L->gelu);
  REQUIRE(L->d > 0 && L->n_heads > 0 && L->d_ff > 0, LLMC_ERR_SHAPE, "non-positive layer size");
  REQUIRE(L->d % 64 == 0 && L->d_ff % 64 == 0, LLMC_ERR_SHAPE, "d=%d and d_ff=%d must be multiples of 64", L->d,
          L->d_ff);
  REQUIRE(L->d % L->n_heads == 0 && L->d / L->n_heads == 64, LLMC_ERR_SHAPE, "head size d/n_heads must be 64, got %d/%d",
          L->d, L->n_heads);
  REQUIRE(L->ln_eps > 0.f && L->ln_eps == L->ln_eps, LLMC_ERR_INVALID_ARG, "ln_eps must be positive");
  const void* ptrs[] = {L->d_wqkv, L->d_bqkv, L->d_wo, L->d_bo, L->d_w1, L->d_b1, L->d_w2, L->d_b2,
                        L->d_ln1_g, L->d_ln1_b, L->d_ln2_g, L->d_ln2_b};
  for (const void* p : ptrs) {
    REQUIRE(p, LLMC_ERR_INVALID_ARG, "a layer weight pointer is NULL");
    REQUIRE(aligned16(p), LLMC_ERR_SHAPE, "layer weight pointers must be 16-byte aligned");
  }
  return LLMC_OK;
}

static size_t gate_small_bytes(int B, int k, int dtype) {
  // keys, inverse norms, idx, sim, hit, tie, hit_rows, miss_rows, slots, recomputed-row scratch, counters
  return align_up((size_t)B * k * elem_size(dtype), 256) + 7 * align_up((size_t)B * 4, 256) +
         2 * align_up((size_t)B, 256) + 256;
}

}  // namespace llmc

using namespace llmc;

extern "C" {

const char* llmc_last_error(void) { return g_err; }
const char* llmc_version(void) { return "llmc 0.1 (gfx950)"; }

static bool lsh_k_ok(int k) { return k == 64 || k == 128 || k == 256 || k == 512; }

llmc_status_t llmc_bank_create(const llmc_bank_desc_t* desc, llmc_bank_t** out) {
  REQUIRE(desc && out, LLMC_ERR_INVALID_ARG, "desc/out is NULL");
  *out = nullptr;
  REQUIRE(dtype_ok(desc->dtype), LLMC_ERR_DTYPE, "bank dtype %d unknown", desc->dtype);
  REQUIRE(desc->policy == LLMC_EVICT_NONE || desc->policy == LLMC_EVICT_LRU ||
              desc->policy == LLMC_EVICT_DECAYED_HITS,
          LLMC_ERR_INVALID_ARG, "eviction policy %d unknown", desc->policy);
  if (desc->policy == LLMC_EVICT_DECAYED_HITS) {
    REQUIRE(desc->half_life >= 0, LLMC_ERR_INVALID_ARG, "half_life must not be negative");
    REQUIRE(desc->n_slots <= (1 << 24), LLMC_ERR_SHAPE, "a bank ranked by decayed hits holds at most 2^24 slots");
  }
  REQUIRE(desc->n_slots > 0 && desc->k > 0 && desc->S > 0 && desc->d > 0 && desc->n_act_slots > 0, LLMC_ERR_SHAPE,
          "non-positive bank size");
  REQUIRE(desc->k % 32 == 0 && desc->k <= 1024, LLMC_ERR_SHAPE, "k=%d must be a multiple of 32, at most 1024", desc->k);
  REQUIRE(desc->d % 64 == 0, LLMC_ERR_SHAPE, "d=%d must be a multiple of 64", desc->d);
  REQUIRE(desc->n_act_slots <= desc->n_slots, LLMC_ERR_SHAPE, "n_act_slots > n_slots");
  REQUIRE(desc->d_act_slot || desc->n_act_slots == desc->n_slots, LLMC_ERR_SHAPE,
          "identity value map needs n_act_slots == n_slots");
  REQUIRE(desc->key_bits == 0 || desc->key_bits == 1, LLMC_ERR_INVALID_ARG, "key_bits must be 0 or 1");
  REQUIRE(desc->d_fp && desc->d_act && (desc->d_inv_norm || desc->key_bits) && desc->d_last_used && desc->d_hits &&
              desc->d_valid,
          LLMC_ERR_INVALID_ARG, "a bank array pointer is NULL");
  REQUIRE(!(desc->key_bits && desc->d_next_fp), LLMC_ERR_INVALID_ARG,
          "stored next-layer keys are refused on a bank of sign-bit keys");
  if (desc->d_lsh_index) {
    REQUIRE(desc->key_bits, LLMC_ERR_INVALID_ARG, "a bucket index needs sign-bit keys");
    REQUIRE(lsh_k_ok(desc->k), LLMC_ERR_SHAPE, "bucketed lookup supports k = 64, 128, 256 or 512 bits");
    REQUIRE(((uintptr_t)desc->d_lsh_index & 255) == 0, LLMC_ERR_SHAPE, "d_lsh_index must be 256-byte aligned");
    REQUIRE(desc->lsh_index_bytes >= lsh_index_bytes(desc->n_slots, desc->k), LLMC_ERR_WORKSPACE,
            "the bucket index needs %zu bytes", lsh_index_bytes(desc->n_slots, desc->k));
  }
  REQUIRE(aligned16(desc->d_fp) && aligned16(desc->d_act), LLMC_ERR_SHAPE, "bank arrays must be 16-byte aligned");
  REQUIRE(!(desc->d_act_pool && desc->rank > 0), LLMC_ERR_INVALID_ARG,
          "stored token means are refused together with compressed values");
  REQUIRE(!(desc->d_act_pool && desc->d_act_slot), LLMC_ERR_INVALID_ARG,
          "stored token means need keys that own their value rows");
  if (desc->d_next_fp || desc->d_next_inv || desc->d_next_proj) {
    REQUIRE(desc->d_next_fp && desc->d_next_inv && desc->d_next_proj && desc->d_act_pool, LLMC_ERR_INVALID_ARG,
            "stored next-layer keys need d_next_proj, d_next_fp, d_next_inv and d_act_pool");
    REQUIRE(desc->next_k > 0 && desc->next_k % 32 == 0 && desc->next_k <= 1024, LLMC_ERR_SHAPE,
            "next_k=%d must be a multiple of 32, at most 1024", desc->next_k);
    REQUIRE(aligned16(desc->d_next_proj) && aligned16(desc->d_next_fp), LLMC_ERR_SHAPE,
            "next-layer key arrays must be 16-byte aligned");
  }
  REQUIRE(desc->rank >= 0, LLMC_ERR_SHAPE, "rank must not be negative");
  if (desc->rank > 0) {
    REQUIRE(desc->rank % 64 == 0 && desc->rank <= desc->d, LLMC_ERR_SHAPE,
            "rank=%d must be a multiple of 64, at most d", desc->rank);
    REQUIRE(desc->d_basis && aligned16(desc->d_basis), LLMC_ERR_INVALID_ARG, "d_basis is NULL or misaligned");
    REQUIRE(desc->policy != LLMC_EVICT_NONE, LLMC_ERR_INVALID_ARG, "compressed values need a replacing policy");
  }
  llmc_bank* b = new (std::nothrow) llmc_bank();
  REQUIRE(b, LLMC_ERR_INVALID_ARG, "out of host memory");
  b->desc = *desc;
  b->d_binv_eff = nullptr;
  b->epoch = 0;
  hipError_t e = hipGetDevice(&b->device);
  b->d_basis_t = nullptr;
  b->d_hit_slots = nullptr;
  if (e == hipSuccess) e = hipMalloc((void**)&b->d_binv_eff, align_up((size_t)desc->n_slots + 8, 256) * sizeof(float));
  if (e == hipSuccess && desc->rank > 0) {
    e = hipMalloc(&b->d_basis_t, (size_t)desc->rank * desc->d * elem_size(desc->dtype));
    if (e == hipSuccess) e = hipMalloc((void**)&b->d_hit_slots, 65536 * sizeof(int32_t));
  }
  if (e != hipSuccess) {
    (void)hipFree(b->d_binv_eff);
    (void)hipFree(b->d_basis_t);
    (void)hipFree(b->d_hit_slots);
    delete b;
    return hip_error(e, "llmc_bank_create: hipMalloc");
  }
  llmc_status_t st = launch_bank_refresh(b, nullptr);
  if (st == LLMC_OK && desc->rank > 0)
    st = launch_transpose(desc->d_basis, b->d_basis_t, desc->rank, desc->d, (int)elem_size(desc->dtype), nullptr);
  if (st == LLMC_OK) {
    e = hipStreamSynchronize(nullptr);
    if (e != hipSuccess) st = hip_error(e, "llmc_bank_create: sync");
  }
  if (st != LLMC_OK) {
    (void)hipFree(b->d_binv_eff);
    (void)hipFree(b->d_basis_t);
    (void)hipFree(b->d_hit_slots);
    delete b;
    return st;
  }
  *out = b;
  return LLMC_OK;
}

llmc_status_t llmc_bank_destroy(llmc_bank_t* bank) {
  if (!bank) return LLMC_OK;
  hipError_t e = hipDeviceSynchronize();
  hipError_t e2 = hipFree(bank->d_binv_eff);
  (void)hipFree(bank->d_basis_t);
  (void)hipFree(bank->d_hit_slots);
  delete bank;
  if (e != hipSuccess) return hip_error(e, "llmc_bank_destroy: sync");
  if (e2 != hipSuccess) return hip_error(e2, "llmc_bank_destroy: hipFree");
  return LLMC_OK;
}

llmc_status_t llmc_bank_refresh(llmc_bank_t* bank, llmc_stream_t stream) {
  REQUIRE(bank, LLMC_ERR_INVALID_ARG, "bank is NULL");
  return launch_bank_refresh(bank, (hipStream_t)stream);
}

llmc_status_t llmc_bank_insert(llmc_bank_t* bank, const void* d_fp, const float* d_inv_norm, const void* d_act,
                               const int32_t* d_rows, const int32_t* d_m, int32_t m_max, uint64_t tick,
                               int32_t* d_slots_out, int32_t* d_counters, llmc_stream_t stream) {
  REQUIRE(bank && d_fp && d_act && d_slots_out, LLMC_ERR_INVALID_ARG, "NULL argument");
  REQUIRE(d_inv_norm || bank->desc.key_bits, LLMC_ERR_INVALID_ARG, "d_inv_norm is NULL");
  REQUIRE(m_max > 0 && m_max <= LLMC_MAX_UPDATE_ROWS, LLMC_ERR_SHAPE, "m_max=%d out of range 1..%d", m_max,
          LLMC_MAX_UPDATE_ROWS);
  REQUIRE(tick <= LLMC_MAX_TICK, LLMC_ERR_INVALID_ARG, "tick out of range");
  REQUIRE(bank->desc.policy != LLMC_EVICT_DECAYED_HITS || tick <= LLMC_MAX_TICK_DECAYED, LLMC_ERR_INVALID_ARG,
          "tick out of range for a bank ranked by decayed hits");
  REQUIRE(bank->desc.n_act_slots == bank->desc.n_slots, LLMC_ERR_SHAPE,
          "insertion into a bank whose keys share value rows is refused");
  REQUIRE(aligned16(d_fp) && aligned16(d_act), LLMC_ERR_SHAPE, "arrays must be 16-byte aligned");
  REQUIRE(bank->desc.rank == 0 || m_max <= bank->desc.n_slots, LLMC_ERR_SHAPE,
          "a bank with compressed values places at most n_slots rows per call");
  return launch_bank_insert(bank, d_fp, d_inv_norm, d_act, d_rows, d_m, m_max, tick, d_slots_out, d_counters,
                            (hipStream_t)stream);
}

llmc_status_t llmc_bank_pool_values(llmc_bank_t* bank, llmc_stream_t stream) {
  REQUIRE(bank, LLMC_ERR_INVALID_ARG, "bank is NULL");
  const llmc_bank_desc_t& D = bank->desc;
  REQUIRE(D.d_act_pool, LLMC_ERR_INVALID_ARG, "the bank keeps no token means");
  for (int s0 = 0; s0 < D.n_act_slots; s0 += 32768) {
    const int n = std::min(32768, D.n_act_slots - s0);
    const char* src = (const char*)D.d_act + (size_t)s0 * D.S * D.d * elem_size(D.dtype);
    LLMC_TRY(launch_pool_rows(src, n, D.S, D.d, D.dtype, nullptr, nullptr, nullptr, D.d_act_pool + (size_t)s0 * D.d,
                              (hipStream_t)stream));
    if (D.d_next_fp)
      LLMC_TRY(launch_project_rows(D.d_act_pool + (size_t)s0 * D.d, n, D.d, D.dtype, D.d_next_proj, D.d_next_bias,
                                   D.next_k, nullptr, nullptr,
                                   (char*)D.d_next_fp + (size_t)s0 * D.next_k * elem_size(D.dtype), D.d_next_inv + s0,
                                   (hipStream_t)stream));
  }
  return LLMC_OK;
}

llmc_status_t llmc_bank_evict(llmc_bank_t* bank, const int32_t* d_m, int32_t m_max, int32_t* d_victims_out,
                              llmc_stream_t stream) {
  REQUIRE(bank && d_victims_out, LLMC_ERR_INVALID_ARG, "NULL argument");
  REQUIRE(m_max > 0 && m_max <= LLMC_MAX_UPDATE_ROWS, LLMC_ERR_SHAPE, "m_max=%d out of range 1..%d", m_max,
          LLMC_MAX_UPDATE_ROWS);
  return launch_bank_evict(bank, d_m, m_max, d_victims_out, (hipStream_t)stream);
}

size_t llmc_fingerprint_workspace_bytes(int32_t B, int32_t S, int32_t d) {
  if (B <= 0 || S <= 0 || d <= 0) return 0;
  return fingerprint_ws_bytes(B, S, d);
}

static llmc_status_t check_fp_shape(int B, int S, int d, int dtype, int k) {
  REQUIRE(dtype_ok(dtype), LLMC_ERR_DTYPE, "dtype %d unknown", dtype);
  REQUIRE(B > 0 && S > 0 && d > 0 && k > 0, LLMC_ERR_INVALID_ARG, "non-positive size");
  REQUIRE(B <= 65535, LLMC_ERR_SHAPE, "B=%d exceeds 65535", B);
  REQUIRE(d % 64 == 0 && d <= 8192, LLMC_ERR_SHAPE, "d=%d must be a multiple of 64, at most 8192", d);
  REQUIRE((size_t)d * elem_size(dtype) <= 16384, LLMC_ERR_SHAPE, "d=%d is too wide for fp32 pooling (at most 4096)", d);
  REQUIRE(k % 32 == 0 && k <= 1024, LLMC_ERR_SHAPE, "k=%d must be a multiple of 32, at most 1024", k);
  return LLMC_OK;
}

llmc_status_t llmc_fingerprint(const void* d_h, int32_t B, int32_t S, int32_t d, int32_t dtype, const void* d_proj,
                               const float* d_bias, int32_t k, void* d_fp_out, float* d_inv_norm_out,
                               void* d_workspace, size_t workspace_bytes, llmc_stream_t stream) {
  REQUIRE(d_h && d_proj && d_fp_out && d_inv_norm_out, LLMC_ERR_INVALID_ARG, "NULL argument");
  LLMC_TRY(check_fp_shape(B, S, d, dtype, k));
  REQUIRE(aligned16(d_h) && aligned16(d_proj) && aligned16(d_fp_out), LLMC_ERR_SHAPE, "arrays must be 16-byte aligned");
  REQUIRE(d_workspace && workspace_bytes >= fingerprint_ws_bytes(B, S, d), LLMC_ERR_WORKSPACE,
          "fingerprint workspace needs %zu bytes", fingerprint_ws_bytes(B, S, d));
  return launch_fingerprint(d_h, nullptr, B, S, d, dtype, d_proj, d_bias, k, d_fp_out, d_inv_norm_out, d_workspace,
                            (hipStream_t)stream);
}

size_t llmc_fingerprint_prefix_workspace_bytes(const llmc_layer_desc_t* layer, int32_t B, int32_t S, int32_t n_prefix) {
  if (!layer || check_layer(layer) != LLMC_OK || B <= 0 || S <= 0 || n_prefix <= 0 || n_prefix > S) return 0;
  // the two features | the dense block over the prefix, which shares its space with the pooling's chunk sums
  return align_up((size_t)B * 2 * layer->d * sizeof(float), 256) +
         std::max(prefix_attention_ws_bytes(layer, B, n_prefix), fingerprint_ws_bytes(B, S, layer->d));
}

llmc_status_t llmc_fingerprint_prefix(const llmc_layer_desc_t* layer, const void* d_h, int32_t B, int32_t S,
                                      int32_t n_prefix, const void* d_proj2, const float* d_bias, int32_t k,
                                      void* d_fp_out, float* d_inv_norm_out, void* d_workspace, size_t workspace_bytes,
                                      llmc_stream_t stream) {
  REQUIRE(layer && d_h && d_proj2 && d_fp_out && d_inv_norm_out, LLMC_ERR_INVALID_ARG, "NULL argument");
  LLMC_TRY(check_layer(layer));
  LLMC_TRY(check_fp_shape(B, S, layer->d, layer->dtype, k));
  REQUIRE(n_prefix >= 1 && n_prefix <= S, LLMC_ERR_INVALID_ARG, "n_prefix=%d must lie in 1..S=%d", n_prefix, S);
  REQUIRE(2 * layer->d <= 8192, LLMC_ERR_SHAPE, "d=%d: the two features together exceed 8192 values", layer->d);
  REQUIRE(aligned16(d_h) && aligned16(d_proj2) && aligned16(d_fp_out), LLMC_ERR_SHAPE, "arrays must be 16-byte aligned");
  const size_t need = llmc_fingerprint_prefix_workspace_bytes(layer, B, S, n_prefix);
  REQUIRE(d_workspace && workspace_bytes >= need, LLMC_ERR_WORKSPACE, "prefix fingerprint workspace needs %zu bytes", need);
  REQUIRE(((uintptr_t)d_workspace & 255) == 0, LLMC_ERR_SHAPE, "workspace must be 256-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  const int d = layer->d;
  float* feat = (float*)d_workspace;                                                   // [B, 2 d]: token mean | prefix attention mean
  void* ws_attn = (char*)d_workspace + align_up((size_t)B * 2 * d * sizeof(float), 256);
  LLMC_TRY(launch_pool_means(d_h, B, S, d, layer->dtype, ws_attn, feat, 2 * d, st));
  LLMC_TRY(launch_prefix_attention_mean(layer, d_h, B, S, n_prefix, ws_attn, feat + d, 2 * d, st));
  return launch_project_rows(feat, B, 2 * d, layer->dtype, d_proj2, d_bias, k, nullptr, nullptr, d_fp_out, d_inv_norm_out, st);
}

llmc_status_t llmc_fingerprint_bits(const void* d_h, int32_t B, int32_t S, int32_t d, int32_t dtype, const void* d_proj,
                                    const float* d_bias, int32_t k, uint32_t* d_bits_out, void* d_workspace,
                                    size_t workspace_bytes, llmc_stream_t stream) {
  REQUIRE(d_h && d_proj && d_bits_out, LLMC_ERR_INVALID_ARG, "NULL argument");
  LLMC_TRY(check_fp_shape(B, S, d, dtype, k));
  REQUIRE(aligned16(d_h) && aligned16(d_proj), LLMC_ERR_SHAPE, "arrays must be 16-byte aligned");
  REQUIRE(d_workspace && workspace_bytes >= fingerprint_ws_bytes(B, S, d), LLMC_ERR_WORKSPACE,
          "fingerprint workspace needs %zu bytes", fingerprint_ws_bytes(B, S, d));
  return launch_fingerprint_bits(d_h, B, S, d, dtype, d_proj, d_bias, k, d_bits_out, d_workspace, (hipStream_t)stream);
}

size_t llmc_match_bits_workspace_bytes(int32_t N, int32_t k, int32_t B) {
  if (N <= 0 || B <= 0 || k <= 0 || k % 32 != 0 || k > 1024 || N > (1 << 30)) return 0;
  return match_bits_ws_bytes(N, k, B);
}


size_t llmc_lsh_index_bytes(int32_t N, int32_t k) {
  if (N <= 0 || N > (1 << 30) || !lsh_k_ok(k)) return 0;
  return lsh_index_bytes(N, k);
}

llmc_status_t llmc_lsh_build(const uint32_t* d_bank_bits, const uint8_t* d_valid, int32_t N, int32_t k, void* d_index,
                             size_t index_bytes, llmc_stream_t stream) {
  REQUIRE(d_bank_bits && d_valid && d_index, LLMC_ERR_INVALID_ARG, "NULL argument");
  REQUIRE(N > 0 && N <= (1 << 30), LLMC_ERR_INVALID_ARG, "N out of range");
  REQUIRE(lsh_k_ok(k), LLMC_ERR_SHAPE, "bucketed lookup supports k = 64, 128, 256 or 512 bits");
  REQUIRE(((uintptr_t)d_index & 255) == 0, LLMC_ERR_SHAPE, "index must be 256-byte aligned");
  REQUIRE(index_bytes >= lsh_index_bytes(N, k), LLMC_ERR_WORKSPACE, "index needs %zu bytes", lsh_index_bytes(N, k));
  return launch_lsh_build(d_bank_bits, d_valid, N, k, d_index, (hipStream_t)stream);
}

llmc_status_t llmc_match_bits_lsh(const uint32_t* d_bank_bits, int32_t N, int32_t k, const void* d_index,
                                  size_t index_bytes, const uint32_t* d_query_bits, int32_t B, int32_t max_hamming,
                                  int32_t* d_idx, int32_t* d_dist, uint8_t* d_hit, int32_t* d_compared,
                                  llmc_stream_t stream) {
  REQUIRE(d_bank_bits && d_index && d_query_bits && d_idx, LLMC_ERR_INVALID_ARG, "NULL argument");
  REQUIRE(N > 0 && N <= (1 << 30) && B > 0, LLMC_ERR_INVALID_ARG, "N or B out of range");
  REQUIRE(lsh_k_ok(k), LLMC_ERR_SHAPE, "bucketed lookup supports k = 64, 128, 256 or 512 bits");
  REQUIRE(((uintptr_t)d_index & 255) == 0, LLMC_ERR_SHAPE, "index must be 256-byte aligned");
  REQUIRE(index_bytes >= lsh_index_bytes(N, k), LLMC_ERR_WORKSPACE, "index needs %zu bytes", lsh_index_bytes(N, k));
  return launch_lsh_match(d_bank_bits, N, k, d_index, d_query_bits, B, max_hamming, d_idx, d_dist, d_hit, d_compared,
                          (hipStream_t)stream);
}

int32_t llmc_max_hamming(float tau, int32_t k) {
  int32_t best = -1;
  for (int32_t H = 0; H <= k; ++H)
    if (cos(3.141592653589793238462643383279502884 * (double)H / (double)k) > (double)tau) best = H;
  return best;
}

llmc_status_t llmc_match_bits(const uint32_t* d_bank_bits, const uint8_t* d_valid, int32_t N, int32_t k,
                              const uint32_t* d_query_bits, int32_t B, int32_t max_hamming, int32_t* d_idx,
                              int32_t* d_dist, uint8_t* d_hit, void* d_workspace, size_t workspace_bytes,
                              llmc_stream_t stream) {
  REQUIRE(d_bank_bits && d_valid && d_query_bits && d_idx, LLMC_ERR_INVALID_ARG, "NULL argument");
  REQUIRE(N > 0 && B > 0, LLMC_ERR_INVALID_ARG, "N and B must be positive");
  REQUIRE(k > 0 && k % 32 == 0 && k <= 1024, LLMC_ERR_SHAPE, "k=%d must be a multiple of 32, at most 1024", k);
  REQUIRE(N <= (1 << 30), LLMC_ERR_SHAPE, "N=%d exceeds 2^30", N);
  REQUIRE(B <= 65535 * 256, LLMC_ERR_SHAPE, "B=%d too large", B);
  const size_t need = match_bits_ws_bytes(N, k, B);
  REQUIRE(d_workspace && workspace_bytes >= need, LLMC_ERR_WORKSPACE, "bit-match workspace needs %zu bytes", need);
  REQUIRE(((uintptr_t)d_workspace & 255) == 0, LLMC_ERR_SHAPE, "workspace must be 256-byte aligned");
  return launch_match_bits(d_bank_bits, d_valid, N, k, d_query_bits, B, max_hamming, d_idx, d_dist, d_hit, d_workspace,
                           (hipStream_t)stream);
}

llmc_status_t llmc_inv_norm(const void* d_fp, int64_t n, int32_t k, int32_t dtype, float* d_inv_norm_out,
                            llmc_stream_t stream) {
  REQUIRE(d_fp && d_inv_norm_out, LLMC_ERR_INVALID_ARG, "NULL argument");
  REQUIRE(dtype_ok(dtype), LLMC_ERR_DTYPE, "dtype %d unknown", dtype);
  REQUIRE(n > 0 && k > 0 && n <= (int64_t)4 * 0x7FFFFFFF, LLMC_ERR_INVALID_ARG, "size out of range");
  return launch_inv_norm(d_fp, n, k, dtype, d_inv_norm_out, (hipStream_t)stream);
}

size_t llmc_match_workspace_bytes(const llmc_bank_t* bank, int32_t B) {
  if (!bank || B <= 0) return 0;
  return match_ws_bytes(bank->desc.n_slots, bank->desc.k, bank->desc.dtype, B);
}

llmc_status_t llmc_match(const llmc_bank_t* bank, const void* d_fp, const float* d_inv_norm, int32_t B, float tau,
                         int32_t* d_idx, float* d_sim, uint8_t* d_hit, uint8_t* d_near_tie, void* d_workspace,
                         size_t workspace_bytes, llmc_stream_t stream) {
  REQUIRE(bank && d_fp && d_inv_norm && d_idx, LLMC_ERR_INVALID_ARG, "NULL argument");
  REQUIRE(!bank->desc.key_bits, LLMC_ERR_DTYPE, "the bank holds sign-bit keys: use llmc_match_bits");
  REQUIRE(B > 0, LLMC_ERR_INVALID_ARG, "B must be positive");
  REQUIRE(B <= 65535 * 128, LLMC_ERR_SHAPE, "B=%d too large", B);
  REQUIRE(tau == tau, LLMC_ERR_INVALID_ARG, "tau is NaN");
  REQUIRE(aligned16(d_fp), LLMC_ERR_SHAPE, "query keys must be 16-byte aligned");
  const size_t need = match_ws_bytes(bank->desc.n_slots, bank->desc.k, bank->desc.dtype, B);
  REQUIRE(d_workspace && workspace_bytes >= need, LLMC_ERR_WORKSPACE, "match workspace needs %zu bytes", need);
  return launch_match(bank, d_fp, d_inv_norm, B, tau, d_idx, d_sim, d_hit, d_near_tie, d_workspace,
                      (hipStream_t)stream);
}

llmc_status_t llmc_match_noalloc(const llmc_bank_t* bank, const void* d_fp, const float* d_inv_norm, int32_t B,
                                 float tau, int32_t* d_idx, float* d_sim, uint8_t* d_hit, uint8_t* d_near_tie,
                                 llmc_stream_t stream) {
  REQUIRE(bank && d_fp && d_inv_norm && d_idx, LLMC_ERR_INVALID_ARG, "NULL argument");
  REQUIRE(!bank->desc.key_bits, LLMC_ERR_DTYPE, "the bank holds sign-bit keys: use llmc_match_bits");
  REQUIRE(B > 0, LLMC_ERR_INVALID_ARG, "B must be positive");
  REQUIRE(B <= 65535 * 128, LLMC_ERR_SHAPE, "B=%d too large", B);
  REQUIRE(tau == tau, LLMC_ERR_INVALID_ARG, "tau is NaN");
  REQUIRE(aligned16(d_fp), LLMC_ERR_SHAPE, "query keys must be 16-byte aligned");
  const size_t need = match_ws_bytes(bank->desc.n_slots, bank->desc.k, bank->desc.dtype, B);
  REQUIRE(need <= (size_t)LLMC_MATCH_STATIC_SCRATCH_BYTES, LLMC_ERR_WORKSPACE,
          "llmc_match_noalloc: %d queries against %d slots need %zu bytes of scratch, the library's fixed scratch "
          "holds %zu: use llmc_match with a workspace",
          B, bank->desc.n_slots, need, (size_t)LLMC_MATCH_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  size_t have = 0;
  LLMC_TRY(match_static_scratch(&ws, &have));
  return launch_match(bank, d_fp, d_inv_norm, B, tau, d_idx, d_sim, d_hit, d_near_tie, ws, (hipStream_t)stream);
}

llmc_status_t llmc_gather_hits(const llmc_bank_t* bank, const int32_t* d_idx, const int32_t* d_rows, const int32_t* d_n,
                               int32_t n_max, void* d_h_out, llmc_stream_t stream) {
  REQUIRE(bank && d_idx && d_h_out, LLMC_ERR_INVALID_ARG, "NULL argument");
  REQUIRE(n_max > 0 && n_max <= 65535, LLMC_ERR_SHAPE, "n_max=%d out of range 1..65535", n_max);
  REQUIRE(aligned16(d_h_out), LLMC_ERR_SHAPE, "output must be 16-byte aligned");
  return launch_gather(bank, d_idx, d_rows, d_n, n_max, d_h_out, (hipStream_t)stream);
}

llmc_status_t llmc_materialize(const llmc_bank_t* bank, const int32_t* d_ref, int32_t B, void* d_h,
                               llmc_stream_t stream) {
  REQUIRE(bank && d_ref && d_h, LLMC_ERR_INVALID_ARG, "NULL argument");
  REQUIRE(B > 0 && B <= 65535, LLMC_ERR_SHAPE, "B=%d out of range 1..65535", B);
  REQUIRE(aligned16(d_h), LLMC_ERR_SHAPE, "output must be 16-byte aligned");
  REQUIRE(bank->desc.rank == 0, LLMC_ERR_INVALID_ARG, "the bank holds compressed values");
  return launch_materialize(bank, d_ref, nullptr, nullptr, B, d_h, (hipStream_t)stream);
}

llmc_status_t llmc_profile_begin(int32_t max_records) {
  REQUIRE(max_records > 0 && max_records <= (1 << 20), LLMC_ERR_INVALID_ARG, "max_records out of range");
  REQUIRE(!g_prof_on.load() && g_prof.empty(), LLMC_ERR_INVALID_ARG, "profiling already on");
  g_prof.resize(max_records);
  for (int i = 0; i < max_records; ++i) {
    g_prof[i].name = nullptr;
    hipError_t e = hipEventCreate(&g_prof[i].a);
    if (e == hipSuccess) {
      e = hipEventCreate(&g_prof[i].b);
      if (e != hipSuccess) (void)hipEventDestroy(g_prof[i].a);
    }
    if (e != hipSuccess) {
      g_prof.resize(i);
      llmc_profile_end();
      return hip_error(e, "hipEventCreate");
    }
  }
  g_prof_used.store(0);
  g_prof_on.store(true);
  return LLMC_OK;
}

int32_t llmc_profile_report(char* buf, size_t cap) {
  if (!buf || cap == 0) return 0;
  buf[0] = 0;
  (void)hipDeviceSynchronize();
  const int n = std::min((int)g_prof.size(), g_prof_used.load());
  std::map<std::string, std::pair<int, double>> agg;
  for (int i = 0; i < n; ++i) {
    float ms = 0.f;
    if (!g_prof[i].name || hipEventElapsedTime(&ms, g_prof[i].a, g_prof[i].b) != hipSuccess) continue;
    auto& a = agg[g_prof[i].name];
    a.first += 1;
    a.second += ms;
  }
  size_t off = 0;
  for (auto& kv : agg) {
    int w = snprintf(buf + off, cap - off, "%s %d %.6f\n", kv.first.c_str(), kv.second.first, kv.second.second);
    if (w < 0 || (size_t)w >= cap - off) break;
    off += (size_t)w;
  }
  g_prof_used.store(0);
  return n;
}

llmc_status_t llmc_profile_end(void) {
  g_prof_on.store(false);
  (void)hipDeviceSynchronize();
  for (auto& r : g_prof) {
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
  }
  g_prof.clear();
  g_prof_used.store(0);
  return LLMC_OK;
}

size_t llmc_layer_workspace_bytes(const llmc_layer_desc_t* layer, int32_t B, int32_t S, int32_t k) {
  if (!layer || B <= 0 || S <= 0 || k < 0 || !dtype_ok(layer->dtype)) return 0;
  return fingerprint_ws_bytes(B, S, layer->d) + gate_small_bytes(B, k > 0 ? k : 32, layer->dtype) +
         match_ws_max_bytes(B) + dedup_ws_bytes(B) + layer_ws_bytes(layer, B, S);
}

llmc_status_t llmc_layer_forward_gated(const llmc_layer_desc_t* layer, llmc_bank_t* bank, const llmc_fp_desc_t* fp,
                                       const void* d_h_in, void* d_h_out, int32_t B, int32_t S, float tau,
                                       uint32_t flags, uint64_t tick, const void* d_fp_given,
                                       const float* d_inv_norm_given, const llmc_gate_out_t* out, void* d_workspace,
                                       size_t workspace_bytes, llmc_stream_t stream) {
  LLMC_TRY(check_layer(layer));
  REQUIRE(d_h_in && d_h_out, LLMC_ERR_INVALID_ARG, "d_h_in/d_h_out is NULL");
  REQUIRE(d_h_in != d_h_out, LLMC_ERR_INVALID_ARG, "d_h_in and d_h_out must not overlap");
  REQUIRE(aligned16(d_h_in) && aligned16(d_h_out), LLMC_ERR_SHAPE, "activations must be 16-byte aligned");
  REQUIRE(B > 0 && S > 0, LLMC_ERR_INVALID_ARG, "B and S must be positive");
  REQUIRE(B <= 65535, LLMC_ERR_SHAPE, "B=%d exceeds 65535", B);
  REQUIRE((int64_t)B * S <= 0x7FFFFFFF / 4, LLMC_ERR_SHAPE, "B*S too large");
  REQUIRE(tau == tau, LLMC_ERR_INVALID_ARG, "tau is NaN");
  REQUIRE(tick <= LLMC_MAX_TICK, LLMC_ERR_INVALID_ARG, "tick out of range");
  REQUIRE((flags & ~(LLMC_INSERT_ON_MISS | LLMC_UPDATE_LRU | LLMC_REVALIDATE | LLMC_HINT_MOSTLY_CARRIED | LLMC_DEFER_COPY |
                     LLMC_DEDUP | LLMC_LOOKUP_LSH)) == 0,
          LLMC_ERR_INVALID_ARG,
          "unknown flag bits");
  int k = 0;
  if (bank) {
    const llmc_bank_desc_t& D = bank->desc;
    REQUIRE(D.dtype == layer->dtype, LLMC_ERR_DTYPE, "bank and layer element types differ");
    REQUIRE(D.d == layer->d && D.S == S, LLMC_ERR_SHAPE, "bank value shape [%d,%d] does not fit [S=%d,d=%d]", D.S, D.d,
            S, layer->d);
    k = D.k;
    if (d_fp_given) {
      REQUIRE(d_inv_norm_given || D.key_bits, LLMC_ERR_INVALID_ARG, "given keys need their inverse norms");
      REQUIRE(aligned16(d_fp_given), LLMC_ERR_SHAPE, "given keys must be 16-byte aligned");
    } else {
      REQUIRE(fp && fp->d_proj, LLMC_ERR_INVALID_ARG, "fingerprint descriptor is NULL");
      REQUIRE(fp->k == D.k, LLMC_ERR_SHAPE, "fingerprint length %d does not fit the bank's %d", fp->k, D.k);
      REQUIRE(aligned16(fp->d_proj), LLMC_ERR_SHAPE, "projection must be 16-byte aligned");
      LLMC_TRY(check_fp_shape(B, S, layer->d, layer->dtype, k));
    }
    REQUIRE(D.policy != LLMC_EVICT_DECAYED_HITS || !(flags & (LLMC_INSERT_ON_MISS | LLMC_UPDATE_LRU)) ||
                tick <= LLMC_MAX_TICK_DECAYED,
            LLMC_ERR_INVALID_ARG, "tick out of range for a bank ranked by decayed hits");
    REQUIRE(!(flags & LLMC_INSERT_ON_MISS) || D.rank == 0 || B <= D.n_slots, LLMC_ERR_SHAPE,
            "a bank with compressed values places at most n_slots rows per call");
    REQUIRE(!(flags & LLMC_REVALIDATE) || D.rank == 0, LLMC_ERR_INVALID_ARG,
            "the divergence monitor is refused on a bank with compressed values");
    REQUIRE(!(flags & LLMC_REVALIDATE) || !D.d_act_pool, LLMC_ERR_INVALID_ARG,
            "the divergence monitor is refused on a bank that keeps token means");
    if (flags & LLMC_DEFER_COPY) {
      REQUIRE(out && out->d_ref_out, LLMC_ERR_INVALID_ARG, "LLMC_DEFER_COPY needs out->d_ref_out");
      REQUIRE(!(flags & (LLMC_INSERT_ON_MISS | LLMC_REVALIDATE)), LLMC_ERR_INVALID_ARG,
              "LLMC_DEFER_COPY is refused with LLMC_INSERT_ON_MISS and LLMC_REVALIDATE");
      REQUIRE(D.rank == 0, LLMC_ERR_INVALID_ARG, "LLMC_DEFER_COPY is refused on a bank with compressed values");
    }
    if (!d_fp_given && fp && fp->d_ref_in) {
      REQUIRE(fp->prev_bank, LLMC_ERR_INVALID_ARG, "d_ref_in needs prev_bank");
      const llmc_bank_desc_t& Pb = fp->prev_bank->desc;
      REQUIRE(Pb.d_next_fp && Pb.next_k == D.k && Pb.dtype == D.dtype && !D.key_bits, LLMC_ERR_SHAPE,
              "prev_bank must keep next-layer keys of this bank's length and type");
      REQUIRE(Pb.S == S && Pb.d == layer->d && Pb.rank == 0, LLMC_ERR_SHAPE, "prev_bank's value shape does not fit");
    }
    if (flags & LLMC_REVALIDATE) {
      REQUIRE(D.reval_every >= 0 && D.drift_bound == D.drift_bound && D.drift_bound >= 0.f, LLMC_ERR_INVALID_ARG,
              "reval_every and drift_bound must not be negative");
      REQUIRE(D.n_act_slots == D.n_slots, LLMC_ERR_SHAPE,
              "the divergence monitor is refused on a bank whose keys share value rows");
    }
    if (flags & LLMC_LOOKUP_LSH)
      REQUIRE(D.key_bits && D.d_lsh_index, LLMC_ERR_INVALID_ARG,
              "LLMC_LOOKUP_LSH needs a bank of sign-bit keys created with d_lsh_index");
    if (flags & LLMC_DEDUP) {
      REQUIRE(flags & LLMC_INSERT_ON_MISS, LLMC_ERR_INVALID_ARG, "LLMC_DEDUP needs LLMC_INSERT_ON_MISS");
      REQUIRE(!(flags & LLMC_REVALIDATE), LLMC_ERR_INVALID_ARG, "LLMC_DEDUP is refused with LLMC_REVALIDATE");
      REQUIRE(B <= LLMC_MAX_DEDUP_ROWS, LLMC_ERR_SHAPE, "LLMC_DEDUP handles at most %d rows per call", LLMC_MAX_DEDUP_ROWS);
      REQUIRE(D.policy != LLMC_EVICT_NONE, LLMC_ERR_INVALID_ARG, "LLMC_DEDUP needs a replacing policy");
      REQUIRE(D.rank == 0 && !D.key_bits, LLMC_ERR_INVALID_ARG,
              "LLMC_DEDUP is refused on banks with compressed values or sign-bit keys");
    }
    if (flags & LLMC_INSERT_ON_MISS) {
      REQUIRE(B <= LLMC_MAX_UPDATE_ROWS, LLMC_ERR_SHAPE, "insertion handles at most %d rows per call",
              LLMC_MAX_UPDATE_ROWS);
      REQUIRE(D.n_act_slots == D.n_slots, LLMC_ERR_SHAPE,
              "insertion into a bank whose keys share value rows is refused");
    }
  }
  const size_t need = llmc_layer_workspace_bytes(layer, B, S, k);
  REQUIRE(d_workspace && workspace_bytes >= need, LLMC_ERR_WORKSPACE, "layer workspace needs %zu bytes", need);
  REQUIRE(aligned16(d_workspace), LLMC_ERR_SHAPE, "workspace must be 16-byte aligned");
  REQUIRE(!out || !out->d_fp_used || aligned16(out->d_fp_used), LLMC_ERR_SHAPE, "d_fp_used must be 16-byte aligned");

  hipStream_t st = (hipStream_t)stream;
  char* p = (char*)d_workspace;
  auto take = [&](size_t bytes) { char* r = p; p += align_up(bytes, 256); return (void*)r; };
  void* ws_fp = take(fingerprint_ws_bytes(B, S, layer->d));
  void* keys = take((size_t)B * (k > 0 ? k : 32) * elem_size(layer->dtype));
  float* inv = (float*)take((size_t)B * 4);
  int32_t* idx = (int32_t*)take((size_t)B * 4);
  float* sim = (float*)take((size_t)B * 4);
  int32_t* hit_rows = (int32_t*)take((size_t)B * 4);
  int32_t* miss_rows = (int32_t*)take((size_t)B * 4);
  int32_t* slots = (int32_t*)take((size_t)B * 4);
  int32_t* reval_tmp = (int32_t*)take((size_t)B * 4);
  uint8_t* hit = (uint8_t*)take((size_t)B);
  uint8_t* tie = (uint8_t*)take((size_t)B);
  int32_t* counters = (int32_t*)take(LLMC_CNT_WORDS * 4);
  void* ws_match = take(match_ws_max_bytes(B));
  void* ws_dedup = take(dedup_ws_bytes(B));
  void* ws_layer = (void*)p;
  if (out) {
    if (out->d_idx) idx = out->d_idx;
    if (out->d_sim) sim = out->d_sim;
    if (out->d_hit) hit = out->d_hit;
    if (out->d_counters) counters = out->d_counters;
    if (out->d_slots) slots = out->d_slots;
    if (out->d_fp_used) keys = out->d_fp_used;
    if (out->d_inv_norm_used) inv = out->d_inv_norm_used;
  }
  if (!bank) {
    LLMC_TRY(launch_all_miss(B, miss_rows, counters, out ? out->d_idx : nullptr, out ? out->d_sim : nullptr,
                             out ? out->d_hit : nullptr, st, out ? out->d_pooled_out_valid : nullptr));
    uint8_t* flags_out = out ? out->d_pooled_out_valid : nullptr;
    return launch_layer(layer, d_h_in, d_h_out, B, S, miss_rows, counters + LLMC_CNT_COMPUTED, ws_layer, st,
                        flags_out ? (float*)ws_fp : nullptr, flags_out);
  }
  if (flags & (LLMC_INSERT_ON_MISS | LLMC_UPDATE_LRU)) LLMC_TRY(launch_bank_advance(bank, tick, st));
  const void* q = d_fp_given;
  const float* qinv = d_inv_norm_given;
  const bool bits = bank->desc.key_bits != 0;
  if (!q && bits) {
    // sign-bit keys (the words live in the key buffer); carried token means are honoured, carried keys are not
    const bool carried = fp->d_pooled_in && fp->d_pooled_in_valid;
    LLMC_TRY(launch_fingerprint_bits(d_h_in, B, S, layer->d, layer->dtype, fp->d_proj, fp->d_bias, k, (uint32_t*)keys,
                                     ws_fp, st, carried ? fp->d_pooled_in : nullptr,
                                     carried ? fp->d_pooled_in_valid : nullptr,
                                     (flags & LLMC_HINT_MOSTLY_CARRIED) != 0));
    q = keys;
  } else if (!q && fp->d_ref_in) {
    // rows that are references to the producing layer's bank take their key from its stored next-layer keys
    const llmc_bank_desc_t& Pb = fp->prev_bank->desc;
    LLMC_TRY(launch_fingerprint(d_h_in, nullptr, B, S, layer->d, layer->dtype, fp->d_proj, fp->d_bias, k, keys, inv,
                                ws_fp, st, nullptr, fp->d_pooled_in_valid, Pb.d_next_fp, Pb.d_next_inv,
                                (flags & LLMC_HINT_MOSTLY_CARRIED) != 0, fp->d_ref_in));
    q = keys;
    qinv = inv;
  } else if (!q) {
    const bool keys_in = fp->d_key_in && fp->d_key_inv_in && fp->d_pooled_in_valid;
    const bool carried = (fp->d_pooled_in || keys_in) && fp->d_pooled_in_valid;
    LLMC_TRY(launch_fingerprint(d_h_in, nullptr, B, S, layer->d, layer->dtype, fp->d_proj, fp->d_bias, k, keys, inv,
                                ws_fp, st, carried ? fp->d_pooled_in : nullptr,
                                carried ? fp->d_pooled_in_valid : nullptr, keys_in ? fp->d_key_in : nullptr,
                                keys_in ? fp->d_key_inv_in : nullptr, (flags & LLMC_HINT_MOSTLY_CARRIED) != 0));
    q = keys;
    qinv = inv;
  }
  if (bits && (flags & LLMC_LOOKUP_LSH)) {
    LLMC_TRY(launch_lsh_match((const uint32_t*)bank->desc.d_fp, bank->desc.n_slots, k, bank->desc.d_lsh_index,
                              (const uint32_t*)q, B, llmc_max_hamming(tau, k), idx, nullptr, hit, nullptr, st, sim));
    tie = nullptr;
  } else if (bits) {
    LLMC_TRY(launch_match_bits((const uint32_t*)bank->desc.d_fp, bank->desc.d_valid, bank->desc.n_slots, k,
                               (const uint32_t*)q, B, llmc_max_hamming(tau, k), idx, nullptr, hit, ws_match, st,
                               (const uint32_t*)bank->d_binv_eff, sim));
    tie = nullptr;
  }
  float* pooled_out = nullptr;
  uint8_t* pooled_valid_out = nullptr;
  void* key_out = nullptr;
  float* key_inv_out = nullptr;
  if (out && out->d_pooled_out_valid) {
    pooled_valid_out = out->d_pooled_out_valid;                       // always written: zeros if nothing is carried
    if (out->d_pooled_out && bank->desc.d_act_pool) pooled_out = out->d_pooled_out;
    if (pooled_out && out->d_key_out && out->d_key_inv_out && bank->desc.d_next_fp) {
      key_out = out->d_key_out;
      key_inv_out = out->d_key_inv_out;
    }
  }
  int32_t* ref_out = (flags & LLMC_DEFER_COPY) ? out->d_ref_out : nullptr;
  if (!bits) LLMC_TRY(launch_match(bank, q, qinv, B, tau, idx, sim, hit, tie, ws_match, st));
  LLMC_TRY(launch_compact(hit, idx, sim, tie, B, tau, hit_rows, miss_rows, reval_tmp, counters, bank, flags, tick, st,
                          pooled_valid_out, pooled_out ? 1 : 0, ref_out));
  // rows to compute that arrived as references get their content now (the only reader of a referenced row)
  if (!d_fp_given && fp && fp->d_ref_in)
    LLMC_TRY(launch_materialize(fp->prev_bank, fp->d_ref_in, miss_rows, counters + LLMC_CNT_COMPUTED, B,
                                const_cast<void*>(d_h_in), st));
  if (!(flags & LLMC_DEFER_COPY))
    LLMC_TRY(launch_gather(bank, idx, hit_rows, counters + LLMC_CNT_HIT, B, d_h_out, st, pooled_out, key_out, key_inv_out));
  // within-batch reuse: the rows to compute shrink to the leaders (after the gather, which reads the hit count)
  if (flags & LLMC_DEDUP) LLMC_TRY(launch_dedup_resolve(q, qinv, k, layer->dtype, B, tau, miss_rows, counters, ws_dedup, st));
  // the rows to compute: the misses, then (divergence monitor) the sampled hit rows, whose copies are overwritten
  // (the last LayerNorm of a post-LayerNorm block also leaves the chunk sums of the computed rows for the next call)
  LLMC_TRY(launch_layer(layer, d_h_in, d_h_out, B, S, miss_rows, counters + LLMC_CNT_COMPUTED, ws_layer, st,
                        pooled_valid_out ? (float*)ws_fp : nullptr, pooled_valid_out));
  if ((flags & LLMC_REVALIDATE) && bank->desc.reval_every > 0)
    LLMC_TRY(launch_divergence(bank, d_h_out, idx, miss_rows, counters, B, st));
  if (flags & LLMC_INSERT_ON_MISS)
    LLMC_TRY(launch_bank_insert(bank, q, qinv, d_h_out, miss_rows, counters + LLMC_CNT_MISS, B, tick, slots, counters,
                                st));
  if (flags & LLMC_DEDUP)
    LLMC_TRY(launch_dedup_finish(bank, d_h_out, B, slots, idx, sim, hit, counters, flags, ws_dedup, st));
  return LLMC_OK;
}

}  // extern "C"
