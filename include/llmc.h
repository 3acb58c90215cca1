/*
 * llmc -- the cache-gated transformer layer of LLMCache on one AMD MI355X (gfx950).
 *
 * C ABI of libllmc.so.  Plain pointers and sizes only.
 *
 * Conventions that hold for every call
 * ------------------------------------
 *  - A pointer whose name starts with d_ is DEVICE memory owned by the caller
 *    (allocated by whatever the caller uses for device memory); every other
 *    pointer is HOST memory.  The library never frees caller memory.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Every call that takes a stream only ENQUEUES work on it and returns
 *    without synchronising; results, including all counts, stay on the device.
 *    No call with a stream argument allocates or frees device memory.
 *  - Errors are return codes.  Arguments are validated before the first HIP
 *    call, so argument errors are reported on a host without a GPU as well.
 *    llmc_last_error() gives a thread-local description of the last failure.
 *  - Matrices are row-major.  Element type is given by llmc_dtype_t: LLMC_F32
 *    (IEEE binary32) or LLMC_BF16 (bfloat16, 2 bytes).  Device pointers must be
 *    16-byte aligned; d (model width) must be a multiple of 64 and k
 *    (fingerprint length) a multiple of 32.
 *  - Batch semantics: all B sequences of a call are matched against the bank as
 *    it stands when the call's kernels run; insertions of this batch are seen
 *    by later calls on the same stream (Algorithm 1 applied batch-wise).
 *  - Results for one sequence do not depend on its row in the batch, on B, or
 *    on which other rows hit or miss: every reduction has a fixed order.
 *  - Two calls that touch the same bank, or share a workspace, must not overlap
 *    on different streams.  A bank handle also carries host-side state (the decay
 *    epoch of LLMC_EVICT_DECAYED_HITS) and library-owned device scratch (the value-row
 *    list of a bank with compressed values): calls on one bank must come from one host
 *    thread at a time, in the order in which their work is to run.
 *  - llmc_profile_* is process-wide and not synchronised: switch it on and off while
 *    no other thread is inside the library.
 */
#ifndef LLMC_H
#define LLMC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct llmc_bank llmc_bank_t; /* opaque handle of one layer's bank C_l */
typedef void* llmc_stream_t;          /* hipStream_t */

typedef enum {
  LLMC_OK = 0,
  LLMC_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, NaN threshold, tick out of range */
  LLMC_ERR_SHAPE = 2,       /* k / S / d / alignment do not fit the bank, the layer or the kernels */
  LLMC_ERR_DTYPE = 3,       /* unknown element type, or operands of different element types */
  LLMC_ERR_BANK_FULL = 4,   /* reserved: a full bank with eviction off is reported on the device, see llmc_bank_insert */
  LLMC_ERR_WORKSPACE = 5,   /* workspace missing or smaller than the matching *_workspace_bytes() */
  LLMC_ERR_HIP = 6          /* a HIP runtime call failed; llmc_last_error() names it */
} llmc_status_t;

typedef enum { LLMC_F32 = 0, LLMC_BF16 = 1 } llmc_dtype_t;

/* Replacement policy (Section III-E / IV-D of the paper).  LRU is the first
 * policy the paper names: remove the entries unused for the longest time.
 * DECAYED_HITS is the staleness-aware policy of Section IV-D (entries whose rate of matches has
 * faded with time go first; Section III-E: frequency-based policy with temporal decay): an entry's
 * standing is its hit count d_hits, and every hit count of the bank is halved (integer
 * shift) each time the tick crosses a multiple of half_life (half_life 0: never, i.e. plain
 * least-frequently-used).  Victims are taken by ascending (min(hits, 65535), last_used,
 * slot).  The halving is applied by the library, before anything else, in every call that
 * takes a tick and updates the bank (llmc_bank_insert, llmc_layer_forward_gated with
 * LLMC_INSERT_ON_MISS or LLMC_UPDATE_LRU); ticks must not decrease.  A bank under this
 * policy holds at most 2^24 slots and takes ticks below LLMC_MAX_TICK_DECAYED.  Whether a call
 * halves is decided on the HOST from the tick it is given, so a recorded HIP graph of such a
 * call repeats the decision taken at capture time: do not replay a graph of a call that updates
 * a DECAYED_HITS bank across a multiple of half_life (record it again, or launch that call eagerly). */
typedef enum { LLMC_EVICT_NONE = 0, LLMC_EVICT_LRU = 1, LLMC_EVICT_DECAYED_HITS = 2 } llmc_evict_t;
#define LLMC_MAX_TICK_DECAYED 0xFFFFFEull

/* Flags of llmc_layer_forward_gated. */
#define LLMC_INSERT_ON_MISS 1u /* Algorithm 1: store (f_X, h_l) of every computed row */
#define LLMC_UPDATE_LRU 2u     /* record hits: last_used = tick, hits += 1 */
#define LLMC_REVALIDATE 4u     /* divergence monitor (Section IV-D, third item; Section III-E): with the bank's
                                  reval_every = r >= 1, a hit row b with (tick + b) % r == 0 is computed anyway and
                                  returns the fresh f_l(h_in[b]); its divergence max|fresh - cached| / max|cached| is
                                  compared with the bank's drift_bound and, if larger, the entry's cached value is
                                  replaced by the fresh output (the key stays).  When several sampled rows of a batch
                                  matched one entry, the lowest row alone decides.  Such rows count as hits and are
                                  not inserted again.  Needs a bank whose keys own their value rows. */

#define LLMC_HINT_MOSTLY_CARRIED 8u /* a hint about cost, never about results: the caller expects nearly every row to arrive
                                       with a carried mean or key (llmc_fp_desc_t), so the separate pooling launch is
                                       dropped and the few other rows are pooled inside the projection's workgroups
                                       (one workgroup per row: slower per row, one launch fewer).  Same bits either way. */

#define LLMC_DEFER_COPY 16u    /* rows answered from the bank are NOT copied into d_h_out; out->d_ref_out[b] receives the
                                  value row of the matched entry instead (-1 for computed rows, whose d_h_out row is
                                  written as usual).  The content of such a row is bank->d_act[d_ref_out[b]] until
                                  someone needs it: the next layer's call (llmc_fp_desc_t.d_ref_in) copies it only if it
                                  has to compute that row, and llmc_materialize copies what is still outstanding at the
                                  end.  A row that keeps hitting is thus never copied.  Needs out->d_ref_out; refused
                                  with LLMC_INSERT_ON_MISS and LLMC_REVALIDATE (the bank must not change while rows
                                  refer to it) and on banks with compressed values. */

#define LLMC_DEDUP 32u         /* within-batch reuse: Algorithm 1 handles inputs one after the other and stores each miss
                                  before the next input is looked up, so an input can hit what an earlier one has just
                                  stored.  With this flag the rows of a batch that miss the bank get that behaviour among
                                  themselves: taken in ascending order, a row is a LEADER unless its key is more similar
                                  than tau to the key of an earlier leader; otherwise it FOLLOWS the most similar earlier
                                  leader (the earliest among equals): it is not computed, returns the leader's output as
                                  stored, is reported as a hit on the leader's new entry (d_idx = that slot, d_sim = the
                                  similarity of the two keys; with LLMC_UPDATE_LRU the entry's hit count grows) and is not
                                  stored again.  Rows that hit the bank as it stood are untouched.  Needs
                                  LLMC_INSERT_ON_MISS and a replacing policy; B <= LLMC_MAX_DEDUP_ROWS; refused with
                                  LLMC_REVALIDATE, compressed values and sign-bit keys. */
#define LLMC_MAX_DEDUP_ROWS 1024
#define LLMC_LOOKUP_LSH 64u    /* sign-bit keys only: the lookup goes through the bank's bucket index (d_lsh_index) instead
                                  of comparing the query with every slot: a query is compared with the slots that share
                                  one whole 16-bit band with it and gets the nearest of those (see llmc_match_bits_lsh);
                                  a row whose nearest neighbour shares no band with it is a miss.  The library keeps the
                                  index current: every call that stores or replaces keys rebuilds it on the device
                                  before it returns (and does nothing of the kind when the batch stored nothing). */

/* Largest tick accepted (recency keys are packed into 32 bits on the device). */
#define LLMC_MAX_TICK 0x7FFFFFFEull
/* Largest number of rows one insert/evict call may place. */
#define LLMC_MAX_UPDATE_ROWS 4096

/* Layout of the device counters written by llmc_layer_forward_gated. */
enum {
  LLMC_CNT_HIT = 0,      /* rows answered from the bank */
  LLMC_CNT_MISS = 1,     /* rows computed */
  LLMC_CNT_NEAR_TAU = 2, /* rows with |sim - tau| < 1e-3 */
  LLMC_CNT_NEAR_TIE = 3, /* rows whose two best candidate groups (or all groups, see below) were re-evaluated exactly */
  LLMC_CNT_INSERTED = 4,
  LLMC_CNT_EVICTED = 5,  /* insertions that replaced a valid entry */
  LLMC_CNT_DROPPED = 6,  /* insertions skipped: bank full and policy NONE */
  LLMC_CNT_COMPUTED = 7, /* rows that went through f_l: misses + revalidated hits */
  LLMC_CNT_REVALIDATED = 8, /* hit rows recomputed by the divergence monitor */
  LLMC_CNT_DIVERGED = 9,    /* of those, entries whose cached value was replaced */
  LLMC_CNT_TIE_OVERFLOW = 10, /* rows with three or more candidate groups within 1e-5 of the best: decided among the two
                                 best groups, so the slot is within that margin of the arg-max but possibly not it */
  LLMC_CNT_DEDUP = 11,      /* LLMC_DEDUP: rows that followed an earlier row of the batch (they are counted as hits too) */
  LLMC_CNT_WORDS = 12
};

/*
 * One layer's bank C_l = {(f, h_l)} (Section III-B): N keys of length k and
 * the cached layer outputs, each [S, d].  All arrays are caller-owned device
 * memory that the library reads and updates in place:
 *   d_fp        [n_slots, k]        keys, element type `dtype`, k contiguous
 *   d_inv_norm  [n_slots]           1 / |key| of the stored (rounded) key, 0 for a zero key
 *   d_act       [n_act_slots, S, d] cached outputs, element type `dtype`
 *   d_act_slot  [n_slots] or NULL   value row of each key; NULL = identity (needs n_act_slots == n_slots)
 *   d_last_used [n_slots]           tick of insertion or latest hit
 *   d_hits      [n_slots]           hits since insertion
 *   d_valid     [n_slots]           1 = slot holds an entry, 0 = free
 * n_act_slots < n_slots lets several keys share one value row (a bounded value
 * store); such a bank is read-only: insertion into it is refused.
 */
typedef struct {
  int32_t n_slots, k, S, d;
  int32_t n_act_slots;
  int32_t dtype;  /* llmc_dtype_t */
  int32_t policy; /* llmc_evict_t */
  void* d_fp;
  void* d_act;
  float* d_inv_norm;
  int32_t* d_act_slot;
  uint64_t* d_last_used;
  uint32_t* d_hits;
  uint8_t* d_valid;
  int32_t half_life; /* LLMC_EVICT_DECAYED_HITS: ticks per halving of the hit counts, 0 = never; else ignored */
  int32_t reval_every; /* LLMC_REVALIDATE: sampling period r of the divergence monitor, 0 = off */
  float drift_bound;   /* LLMC_REVALIDATE: divergence above which a cached value is replaced */
  /* Compressed cached values (Section III-B: cached representations may be stored compressed, by PCA).
   * rank = 0: d_act holds the outputs themselves, [n_act_slots, S, d].
   * rank = r > 0: d_basis [r, d] (element type `dtype`, d contiguous, rows = the directions kept) is given, d_act
   * is [n_act_slots, S, r] and holds the coefficients C = h U^T of each cached output, rounded to `dtype`; a hit
   * returns the reconstruction C U (rounded to `dtype`).  Both products run on the layer's GEMM kernels.
   * r % 64 == 0, r <= d; the policy must not be NONE; the divergence monitor is refused.  The basis is read at
   * llmc_bank_create (the library keeps a transposed copy) and must stay unchanged and alive afterwards. */
  int32_t rank;
  const void* d_basis;
  /* Optional [n_act_slots, d] fp32, caller-owned: the token mean (1/S) sum_t h[t,:] of each cached output, written
   * by the library whenever it stores an output (same arithmetic and order as the fingerprint's pooling), read by
   * llmc_layer_forward_gated to hand the next layer its pooled input without reading the output again.  NULL: not
   * kept.  Refused together with compressed values.  Entries written into d_act by the caller directly have no
   * mean until llmc_bank_pool_values() is called. */
  float* d_act_pool;
  /* Optional, needs d_act_pool: the KEY under which each cached output will be looked up by the next layer, i.e.
   * its fingerprint under that layer's map (d_next_proj [d, next_k], d_next_bias [next_k] or NULL), kept in
   * d_next_fp [n_act_slots, next_k] (element type `dtype`) and d_next_inv [n_act_slots].  Written by the library
   * whenever it stores an output (the same arithmetic as llmc_fingerprint, so the same bits), handed to the next
   * call through llmc_gate_out_t.d_key_out, which then neither pools nor projects the reused rows.  All NULL: not
   * kept.  The projection arrays must stay alive and unchanged. */
  const void* d_next_proj;
  const float* d_next_bias;
  int32_t next_k;
  void* d_next_fp;
  float* d_next_inv;
  /* key_bits = 1: the keys are SIGN BITS (SimHash, see llmc_fingerprint_bits): d_fp is uint32 [n_slots, k / 32],
   * d_inv_norm is not used (may be NULL), the match is by Hamming distance and the threshold of
   * llmc_layer_forward_gated is applied as H <= llmc_max_hamming(tau, k); the similarity reported is cos(pi H / k).
   * llmc_bank_insert and d_fp_given then take keys in that form (d_inv_norm / d_inv_norm_given ignored);
   * llmc_match refuses such a bank (use llmc_match_bits).  Refused together with stored next-layer keys. */
  int32_t key_bits;
  /* Optional, key_bits = 1 only: storage for the bucket index of the keys (Section IV-B, LSH), device memory of
   * lsh_index_bytes >= llmc_lsh_index_bytes(n_slots, k) bytes, 256-byte aligned, owned by the caller and written by
   * the library alone: llmc_bank_create and llmc_bank_refresh build it from the keys and validity flags as they
   * stand, llmc_bank_insert and the insertions of llmc_layer_forward_gated rebuild it after they changed a key.
   * LLMC_LOOKUP_LSH needs it.  k must be 64, 128, 256 or 512. */
  void* d_lsh_index;
  size_t lsh_index_bytes;
} llmc_bank_desc_t;

/*
 * One transformer block f_l (Section IV-A; model families of Section V-A).
 * arch 0: encoder, post-LayerNorm, bidirectional attention:
 *     x1 = LN1(x + MHA(x));  y = LN2(x1 + W2 act(W1 x1 + b1) + b2)
 * arch 1: decoder, pre-LayerNorm, causal attention:
 *     x1 = x + MHA(LN1(x));  y = x1 + W2 act(W1 LN2(x1) + b1) + b2
 * Linear weights are [out_features, in_features] (input index contiguous):
 * d_wqkv [3d, d] with rows 0..d-1 = Q, d..2d-1 = K, 2d..3d-1 = V and head h
 * owning features h*dh..(h+1)*dh-1 of each; d_wo [d, d]; d_w1 [d_ff, d];
 * d_w2 [d, d_ff].  Biases and LayerNorm parameters are vectors of the same
 * element type.  Attention scores are scaled by 1/sqrt(dh), dh = d / n_heads
 * (the kernels support dh = 64).  gelu 0 = exact erf form, 1 = tanh form.
 */
typedef struct {
  int32_t arch;
  int32_t d, n_heads, d_ff;
  int32_t gelu;
  float ln_eps;
  int32_t dtype; /* llmc_dtype_t */
  const void *d_wqkv, *d_bqkv, *d_wo, *d_bo, *d_w1, *d_b1, *d_w2, *d_b2;
  const void *d_ln1_g, *d_ln1_b, *d_ln2_g, *d_ln2_b;
} llmc_layer_desc_t;

/* Fingerprint map of one layer (Section IV-B): projection P [d, k] (element
 * type of the run, k contiguous) and optional fp32 offset c [k] (NULL = 0). */
typedef struct {
  const void* d_proj;
  const float* d_bias;
  int32_t k;
  /* Optional carry from the call that produced this layer's input (see llmc_gate_out_t.d_pooled_out): for a
   * row b with d_pooled_in_valid[b] == 1, d_pooled_in[b] [d] fp32 is taken as the token mean of d_h_in[b] and the
   * row is not read again.  The carried mean is the one the library itself computes (same arithmetic, same
   * order), so keys do not depend on whether a mean was carried.  d_pooled_in_valid[b] == 2 says that the producing
   * call computed row b and its last LayerNorm already left the row's pooled chunk sums in the fingerprint part of
   * the workspace: the row is not read again either.  Flag 2 is only meaningful when this call is given the SAME
   * workspace, with the same B, S and d, as the producing call, and nothing wrote to it in between; a caller that
   * cannot promise that clears such flags to 0.  Both NULL: every row is pooled here. */
  const float* d_pooled_in;
  const uint8_t* d_pooled_in_valid;
  /* Optional, with d_pooled_in_valid: finished keys [B, k] + inverse norms [B] of the flagged rows (see
   * llmc_gate_out_t.d_key_out); those rows are then neither pooled nor projected.  k must be this map's k. */
  const void* d_key_in;
  const float* d_key_inv_in;
  /* Optional, from a producing call made with LLMC_DEFER_COPY: d_ref_in[b] >= 0 says that row b of d_h_in was not
   * written and stands for value row d_ref_in[b] of prev_bank (the producing layer's bank, which must keep
   * next-layer keys under THIS map: d_next_fp).  The key of such a row is taken from there.  If the row has to be
   * computed, this call first copies prev_bank's value row into d_h_in[b]: with d_ref_in the buffer behind d_h_in
   * is written to, its const notwithstanding.  The carry pointers above are ignored when d_ref_in is given. */
  const llmc_bank_t* prev_bank;
  const int32_t* d_ref_in;
} llmc_fp_desc_t;

/* Optional per-row results of the gate; any pointer may be NULL. */
typedef struct {
  int32_t* d_idx;      /* [B] best slot, -1 if the bank has no valid entry */
  float* d_sim;        /* [B] best cosine similarity, -inf if none */
  uint8_t* d_hit;      /* [B] 1 = reused, 0 = computed */
  int32_t* d_counters; /* [LLMC_CNT_WORDS], overwritten by the call */
  int32_t* d_slots;    /* [B] slots taken by this call's insertions, in ascending miss-row order */
  /* Reuse fused with the next layer's pooling: the cached output of a hit is the next layer's input, and its
   * token mean was stored with it (llmc_bank_desc_t.d_act_pool).  With a bank that has d_act_pool, and both
   * pointers given, the call writes d_pooled_out[b] [d] fp32 = that stored mean and d_pooled_out_valid[b] = 1 for
   * every row answered from the bank.  Computed rows get 0 (the next call pools them itself), or 2 when the block's
   * last LayerNorm pooled them on the way out (post-LayerNorm blocks: the chunk sums stay in the workspace, see
   * llmc_fp_desc_t.d_pooled_in_valid). */
  float* d_pooled_out;          /* [B, d] */
  uint8_t* d_pooled_out_valid;  /* [B] */
  /* With a bank that keeps d_next_fp: the stored next-layer key and inverse norm of every row answered from the
   * bank (same flags).  d_key_out [B, next_k] in the bank's element type, d_key_inv_out [B]. */
  void* d_key_out;
  float* d_key_inv_out;
  int32_t* d_ref_out;           /* [B], written with LLMC_DEFER_COPY: value row of the matched entry, or -1 */
  /* The keys the rows were matched with, [B, k] in the bank's key form (element type `dtype`, or uint32 words for a
   * bank of sign-bit keys), and their inverse norms [B] (real-valued keys only): whatever their source was --
   * computed here, carried, or taken from the producing bank's stored keys.  Not written when d_fp_given is used. */
  void* d_fp_used;
  float* d_inv_norm_used;
} llmc_gate_out_t;

/* ---- bank -------------------------------------------------------------- */

/*
 * Wrap caller-owned arrays as a bank (Section III-B).  Synchronous: allocates
 * a small device mirror of the validity/norm arrays ([n_slots] floats), fills
 * it from d_valid and d_inv_norm on the default stream and waits for that.
 * The arrays must hold a consistent state (all-zero d_valid = empty bank).
 * Errors: INVALID_ARG (null desc/out/array), SHAPE (sizes <= 0, k % 32, d % 64,
 * n_act_slots > n_slots, identity map with n_act_slots != n_slots), DTYPE, HIP.
 */
llmc_status_t llmc_bank_create(const llmc_bank_desc_t* desc, llmc_bank_t** out);

/* Free what llmc_bank_create allocated (never the caller's arrays).  Synchronous. */
llmc_status_t llmc_bank_destroy(llmc_bank_t* bank);

/*
 * If the caller wrote the bank arrays directly (e.g. loaded keys), rebuild the
 * library's mirror from d_valid / d_inv_norm.  Enqueued on `stream`.
 */
llmc_status_t llmc_bank_refresh(llmc_bank_t* bank, llmc_stream_t stream);

/*
 * Algorithm 1's store step, C_l[f_X] <- h_l, for a batch (Section III-C: a
 * computed result is added to the cache), with the replacement of Section IV-D.
 *   d_fp [*, k], d_inv_norm [*], d_act [*, S, d]: keys, their inverse norms and the values;
 *          the i-th stored entry is row d_rows[i] of all three (d_rows NULL: row i)
 *   d_m: device count m of rows to store (NULL: m = m_max); m is clamped to m_max
 *   tick: recency stamp given to the new entries (<= LLMC_MAX_TICK)
 *   d_slots_out [m_max]: slot taken by row i, -1 if the row was dropped
 *   d_counters: optional [LLMC_CNT_WORDS]; INSERTED / EVICTED / DROPPED are ADDED to
 * Rows take, in order, free slots by ascending index and then, the bank being
 * full, the valid entries in ascending (last_used, slot) order; a replaced
 * entry's hit count restarts at 0.  With policy NONE rows beyond the free
 * slots are dropped and counted.  m_max <= LLMC_MAX_UPDATE_ROWS.
 * Errors: INVALID_ARG, SHAPE (m_max out of range; bank with shared value rows).
 */
llmc_status_t llmc_bank_insert(llmc_bank_t* bank, const void* d_fp, const float* d_inv_norm,
                               const void* d_act, const int32_t* d_rows, const int32_t* d_m,
                               int32_t m_max, uint64_t tick, int32_t* d_slots_out,
                               int32_t* d_counters, llmc_stream_t stream);

/* Recompute d_act_pool (and d_next_fp / d_next_inv, if kept) from d_act for all value rows (after the caller wrote
 * values directly).
 * INVALID_ARG if the bank keeps no means. */
llmc_status_t llmc_bank_pool_values(llmc_bank_t* bank, llmc_stream_t stream);

/*
 * Section IV-D, LRU: invalidate the m least recently used valid entries.
 *   d_m: device count (NULL: m = m_max), clamped to m_max and to the number of valid entries
 *   d_victims_out [m_max]: evicted slots in ascending (last_used, slot) order, -1 beyond the count
 * The keys and values of evicted slots are left in place; only validity changes.
 */
llmc_status_t llmc_bank_evict(llmc_bank_t* bank, const int32_t* d_m, int32_t m_max,
                              int32_t* d_victims_out, llmc_stream_t stream);

/* ---- fingerprint --------------------------------------------------------- */

/*
 * Section IV-B: embedding aggregation then dimensionality reduction, giving the
 * fixed-length key of Section III-A.  For each sequence b of d_h [B, S, d]:
 *   p = (1/S) sum_t h[b,t,:];  v = P^T p + c;  u = v / max(|v|, 1e-12);
 *   d_fp_out[b] = u rounded to `dtype` (nearest even);  d_inv_norm_out[b] = 1/|rounded u| (0 if 0).
 * d_proj [d, k] has element type `dtype`; d_bias [k] fp32 or NULL.
 * d_workspace: at least llmc_fingerprint_workspace_bytes(B, S, d) bytes.
 * Accumulation is fp32 in a fixed order that depends on S and d only.
 */
llmc_status_t llmc_fingerprint(const void* d_h, int32_t B, int32_t S, int32_t d, int32_t dtype,
                               const void* d_proj, const float* d_bias, int32_t k,
                               void* d_fp_out, float* d_inv_norm_out, void* d_workspace,
                               size_t workspace_bytes, llmc_stream_t stream);
size_t llmc_fingerprint_workspace_bytes(int32_t B, int32_t S, int32_t d);

/* d_inv_norm_out[i] = 1 / |d_fp[i]| for n stored keys [n, k] (0 for a zero key):
 * the norm that the cosine of Section III-C divides by, for keys supplied directly. */
llmc_status_t llmc_inv_norm(const void* d_fp, int64_t n, int32_t k, int32_t dtype,
                            float* d_inv_norm_out, llmc_stream_t stream);

/* ---- match ------------------------------------------------------------------ */

/*
 * Section III-C with the test of Section IV-A / Algorithm 1: for each query
 * key, the valid bank entry of largest cosine similarity, and whether that
 * similarity strictly exceeds tau.
 *   d_fp [B, k] (bank's element type), d_inv_norm [B]
 *   d_idx [B]: best slot, lowest slot on exact ties, -1 if no valid entry
 *   d_sim [B]: its cosine (product of the stored vectors times both inverse norms), -inf if none
 *   d_hit [B]: sim > tau        (d_sim, d_hit may be NULL)
 *   d_near_tie: optional [B] flags: 1 where two candidate groups were compared exactly; 2 where three or more
 *               groups were within 1e-5 of the best (several near-identical keys): the winner of the two best
 *               groups is returned, which is within that margin of the maximum but need not be the arg-max
 * The bulk search runs on the matrix cores with fp32 accumulation; the winner
 * is then decided, and d_sim computed, in fp64 among the best candidate group
 * (and the runner-up group when the two are closer than 1e-5).
 * d_workspace: at least llmc_match_workspace_bytes(bank, B) bytes.
 * Errors: INVALID_ARG (null, B <= 0, tau NaN), WORKSPACE.
 */
llmc_status_t llmc_match(const llmc_bank_t* bank, const void* d_fp, const float* d_inv_norm,
                         int32_t B, float tau, int32_t* d_idx, float* d_sim, uint8_t* d_hit,
                         uint8_t* d_near_tie, void* d_workspace, size_t workspace_bytes,
                         llmc_stream_t stream);
size_t llmc_match_workspace_bytes(const llmc_bank_t* bank, int32_t B);

/*
 * llmc_match for callers that cannot allocate device memory and have no workspace to pass: code running under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * the same results as llmc_match, but the per-split candidates of the bulk pass go to a fixed scratch array
 * inside the library (LLMC_MATCH_STATIC_SCRATCH_BYTES of device memory per GPU, held until the process ends)
 * instead of a caller's workspace.  The call allocates and frees nothing.
 * Errors: as llmc_match; WORKSPACE if llmc_match_workspace_bytes(bank, B) exceeds the fixed scratch (the
 * message names both sizes), nothing is enqueued then.
 * Every call on one GPU shares that GPU's scratch: two such calls must not overlap in time on one GPU
 * (different streams, or different host threads), or they race on it.  Calls on one stream are ordered and safe.
 */
#define LLMC_MATCH_STATIC_SCRATCH_BYTES (5u << 20)
llmc_status_t llmc_match_noalloc(const llmc_bank_t* bank, const void* d_fp, const float* d_inv_norm,
                                 int32_t B, float tau, int32_t* d_idx, float* d_sim, uint8_t* d_hit,
                                 uint8_t* d_near_tie, llmc_stream_t stream);

/* ---- sign-bit keys (SimHash) and their Hamming match ------------------------------ */

/*
 * Section IV-B names SimHash as the dimensionality reduction and Section III-A hashing as the
 * route to cheap comparison: the key is the SIGN of each of the k projections of the pooled
 * input.  For each sequence b of d_h [B, S, d]:  p = (1/S) sum_t h[b,t,:];  v = P^T p + c;
 * bit i of the key = (v_i >= 0).  d_bits_out [B, k / 32] uint32: bit i is word i / 32, position
 * i % 32 (least significant first).  Pooling and projection are those of llmc_fingerprint
 * (same workspace size, same fixed fp32 accumulation order); k % 32 == 0, k <= 1024.
 */
llmc_status_t llmc_fingerprint_bits(const void* d_h, int32_t B, int32_t S, int32_t d, int32_t dtype,
                                    const void* d_proj, const float* d_bias, int32_t k,
                                    uint32_t* d_bits_out, void* d_workspace, size_t workspace_bytes,
                                    llmc_stream_t stream);

/*
 * Section IV-B, the second fingerprint feature (prefix attention statistics: the mean of the first self-attention
 * outputs), taken together with the first (the token average) and reduced by ONE linear map:
 *   p = mean_t h[b, t, :]                                            (as in llmc_fingerprint)
 *   a = mean_{t < n_prefix} MHA_l(h[b, 0 .. n_prefix, :])[t, :]      the block's own self-attention sub-layer over the
 *       first n_prefix tokens ALONE (they attend to each other only; after LN1 and causal in the pre-LayerNorm decoder
 *       block), outputs taken after the output projection and before the residual
 *   v = P2^T [p; a] + c,  P2 [2 d, k] row-major (rows 0 .. d-1 act on p, rows d .. 2d-1 on a);  key = v / |v| rounded
 *       to the element type, inv_norm = 1 / |rounded key|, exactly as llmc_fingerprint does.
 * For a causal block the feature depends on the first n_prefix tokens only, so inputs sharing a prefix share it.
 *   layer: the block whose attention weights are used (its dtype is the element type of d_h, d_proj2 and d_fp_out)
 *   d_h [B, S, d], d_proj2 [2 d, k], d_bias [k] fp32 or NULL, d_fp_out [B, k], d_inv_norm_out [B] fp32: device memory
 *   of the caller; d_workspace: llmc_fingerprint_prefix_workspace_bytes(layer, B, S, n_prefix) bytes, 256-byte aligned.
 * The keys are for llmc_match / llmc_bank_insert or for llmc_layer_forward_gated's d_fp_given.  On return the first
 * B * 2 d floats of d_workspace hold the two features of every row, [p; a] row by row (fp32): what a caller needs to
 * centre the map (c = -P2^T mean[p; a] over the sequences a bank is built from).  Nothing is allocated or synchronised.  Errors: INVALID_ARG (null, n_prefix outside 1..S), SHAPE (layer, k, alignment), DTYPE, WORKSPACE.
 */
llmc_status_t llmc_fingerprint_prefix(const llmc_layer_desc_t* layer, const void* d_h, int32_t B, int32_t S,
                                      int32_t n_prefix, const void* d_proj2, const float* d_bias, int32_t k,
                                      void* d_fp_out, float* d_inv_norm_out, void* d_workspace,
                                      size_t workspace_bytes, llmc_stream_t stream);
size_t llmc_fingerprint_prefix_workspace_bytes(const llmc_layer_desc_t* layer, int32_t B, int32_t S, int32_t n_prefix);

/*
 * Section IV-B (keys are compared by cosine similarity or by LSH), with the test of the case equation
 * (Section IV-A): for each query key the valid bank key at the smallest Hamming distance H;
 * cos(pi H / k) stands for the cosine of the two pooled inputs, so  sim > tau  becomes
 * H <= max_hamming  with  max_hamming = llmc_max_hamming(tau, k).
 *   d_bank_bits [N, k / 32], d_valid [N] (0 = free slot), d_query_bits [B, k / 32]: device, uint32 words as above
 *   d_idx [B]: nearest valid slot, lowest slot among equal distances, -1 if no slot is valid
 *   d_dist [B]: its Hamming distance, 0x7FFFFFFF if none;  d_hit [B]: idx >= 0 and dist <= max_hamming
 *   (d_dist, d_hit may be NULL).  Integer work throughout: results are exact.  Which kernel scans the bank depends
 *   on the sizes only (512 queries or more of 256-bit keys in 16-byte aligned arrays: an int8 matrix-core product of
 *   the expanded bits; otherwise XOR + popcount on the vector ALU); the results do not.
 * d_workspace: at least llmc_match_bits_workspace_bytes(N, k, B) bytes.  Nothing is allocated or synchronised.
 * Errors: INVALID_ARG (null, sizes <= 0), SHAPE (k % 32 != 0 or k > 1024, N > 2^30), WORKSPACE.
 */
llmc_status_t llmc_match_bits(const uint32_t* d_bank_bits, const uint8_t* d_valid, int32_t N, int32_t k,
                              const uint32_t* d_query_bits, int32_t B, int32_t max_hamming,
                              int32_t* d_idx, int32_t* d_dist, uint8_t* d_hit, void* d_workspace,
                              size_t workspace_bytes, llmc_stream_t stream);
size_t llmc_match_bits_workspace_bytes(int32_t N, int32_t k, int32_t B);

/*
 * Bucketed lookup of sign-bit keys (Section IV-B, LSH; Section III-A asks for a comparison cost below linear in the bank size).  The key is
 * cut into k / 16 bands of 16 bits (band b = bits 16 b .. 16 b + 15).  llmc_lsh_build groups the valid slots of a
 * bank by the value of each band into d_index (caller-owned, llmc_lsh_index_bytes(N, k) bytes, 256-byte aligned);
 * it must be called again after the bank's keys or validity change.  llmc_match_bits_lsh compares a query only with
 * the slots that share at least one whole band with it and returns the nearest of those (lowest slot among equal
 * distances; -1 / 0x7FFFFFFF if there is none): the exact nearest neighbour whenever that neighbour shares a band
 * with the query, at a cost that grows with the bucket sizes and not with N.
 *   d_compared [B] (optional): bucket members visited per query (a slot in several of its buckets counts each time)
 * k must be 64, 128, 256 or 512.  Errors: INVALID_ARG, SHAPE, WORKSPACE (index too small).
 */
size_t llmc_lsh_index_bytes(int32_t N, int32_t k);
llmc_status_t llmc_lsh_build(const uint32_t* d_bank_bits, const uint8_t* d_valid, int32_t N, int32_t k,
                             void* d_index, size_t index_bytes, llmc_stream_t stream);
llmc_status_t llmc_match_bits_lsh(const uint32_t* d_bank_bits, int32_t N, int32_t k, const void* d_index,
                                  size_t index_bytes, const uint32_t* d_query_bits, int32_t B,
                                  int32_t max_hamming, int32_t* d_idx, int32_t* d_dist, uint8_t* d_hit,
                                  int32_t* d_compared, llmc_stream_t stream);

/* Host arithmetic, no device work: the largest H in 0..k with cos(pi * H / k) > tau, evaluated in
 * binary64 as written; -1 if there is none (tau >= 1) or k <= 0. */
int32_t llmc_max_hamming(float tau, int32_t k);

/* ---- gather ----------------------------------------------------------------- */

/*
 * Algorithm 1's reuse step h_l <- h' (Section IV-A, first case): for i < n,
 * copy the cached output of slot d_idx[d_rows[i]] into d_h_out[d_rows[i]].
 *   d_rows [n_max] row numbers, d_n device count (NULL: n = n_max), d_idx [B] slots
 * Exact copy (a bank with compressed values writes the reconstruction C U instead, see llmc_bank_desc_t).
 * d_h_out is [B, S, d] with the bank's S, d and element type.
 */
llmc_status_t llmc_gather_hits(const llmc_bank_t* bank, const int32_t* d_idx, const int32_t* d_rows,
                               const int32_t* d_n, int32_t n_max, void* d_h_out, llmc_stream_t stream);

/* Copy the rows that LLMC_DEFER_COPY left outstanding: d_h[b] = bank->d_act[d_ref[b]] for d_ref[b] >= 0 (other rows
 * untouched).  d_h [B, S, d] with the bank's S, d and element type. */
llmc_status_t llmc_materialize(const llmc_bank_t* bank, const int32_t* d_ref, int32_t B, void* d_h,
                               llmc_stream_t stream);

/* ---- the gated layer ---------------------------------------------------------- */

/*
 * One trip of Algorithm 1's loop body for a batch (case equation of Section
 * IV-A): fingerprint the layer input, match it against the layer's bank,
 * reuse the cached output where sim > tau and compute f_l only for the other
 * rows, then (by flag) record hits and store the computed rows.
 *   layer: f_l;  bank: C_l, or NULL = the layer is not cached and every row is
 *          computed (layer selection, Section VI-D);  fp: P_l, c_l (ignored if bank NULL)
 *   d_h_in, d_h_out [B, S, d], element type of the layer; they must not overlap
 *   d_fp_given / d_inv_norm_given: NULL, or keys [B, k] + norms to use instead of
 *          fingerprinting d_h_in (Algorithm 1 taken literally: one fingerprint of X for all layers)
 *   tau: threshold; flags: LLMC_INSERT_ON_MISS | LLMC_UPDATE_LRU | LLMC_REVALIDATE | LLMC_HINT_MOSTLY_CARRIED |
 *          LLMC_DEFER_COPY | LLMC_DEDUP | LLMC_LOOKUP_LSH;
 *          tick <= LLMC_MAX_TICK
 *   out: optional per-row results and counters (NULL or any member NULL)
 *   d_workspace: at least llmc_layer_workspace_bytes(layer, B, S, k) bytes
 * The number of misses never visits the host: the miss-path kernels read it on
 * the device.  Hit rows are exact copies of the cached values.
 * Errors: INVALID_ARG, SHAPE (layer/bank/fp disagree on d, S, k or dtype; dh != 64), DTYPE, WORKSPACE.
 */
llmc_status_t llmc_layer_forward_gated(const llmc_layer_desc_t* layer, llmc_bank_t* bank,
                                       const llmc_fp_desc_t* fp, const void* d_h_in, void* d_h_out,
                                       int32_t B, int32_t S, float tau, uint32_t flags, uint64_t tick,
                                       const void* d_fp_given, const float* d_inv_norm_given,
                                       const llmc_gate_out_t* out, void* d_workspace,
                                       size_t workspace_bytes, llmc_stream_t stream);
size_t llmc_layer_workspace_bytes(const llmc_layer_desc_t* layer, int32_t B, int32_t S, int32_t k);

/* ---- measurement aid ------------------------------------------------------------- */

/*
 * Per-kernel timing with HIP events on the launch stream: while recording is on, every kernel
 * the library enqueues is launched with a start and a stop event of its own (hipExtLaunchKernel),
 * which carry the begin and the end of that kernel's execution on the device, i.e. the duration a
 * kernel trace reports for the dispatch (gaps between dispatches are not included).
 * llmc_profile_begin creates `max_records` event pairs (it allocates; call it outside any timed or
 * captured region) and switches recording on; launches beyond max_records are not recorded.
 * llmc_profile_report synchronises the device and writes one text line per kernel name,
 * "name count total_ms", into buf (NUL-terminated, truncated to cap), restarts the record count and
 * returns the number of records it read.  llmc_profile_end switches recording off and destroys the
 * events.  Do not record inside a stream capture; time whole steps with recording off.
 */
llmc_status_t llmc_profile_begin(int32_t max_records);
int32_t llmc_profile_report(char* buf, size_t cap);
llmc_status_t llmc_profile_end(void);

/* ---- misc ---------------------------------------------------------------------- */

const char* llmc_last_error(void); /* thread-local, never NULL */
const char* llmc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LLMC_H */
