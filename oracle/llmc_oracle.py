"""Plain CPU oracle of the cache-gated transformer layer (LLMCache).

TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of
what the path computes, written from the paper; it is imported by the tests, by
the smoke check and by the benchmark's CPU-baseline leg, and by nothing else.
It shares no code with the HIP library and never imports it.

Everything is numpy in float64.  Inputs are the *stored* values of the run
(fp32, or bf16 widened exactly to fp32/fp64); no intermediate rounding of the
run dtype is emulated except where the method itself stores a rounded value
(the fingerprint key, Section III-B: the bank holds the key that is compared).

What follows the paper, and where:

* fingerprint  -- Section IV-B: average of the token vectors, then a linear
  dimensionality reduction; Section III-A: a fixed-length key.
* match        -- Section III-C / Algorithm 1: "exists an entry with
  sim > tau"  <=>  max_j sim_j > tau, sim = cosine similarity.
* threshold    -- Section IV-A case equation and Algorithm 1: strict ">".
* gated layer  -- Section IV-A case equation: cached h_l on a hit, f_l(h_{l-1})
  otherwise; Algorithm 1: store the computed h_l on a miss.
* sign-bit keys -- Section IV-B (SimHash), Section III-A: the sign of each
  projection, compared by Hamming distance; cos(pi H / k) stands for the cosine.
* compressed values -- Section III-B: cached outputs stored as coefficients on a
  PCA basis and reconstructed on a hit.
* eviction     -- Section IV-D, first policy: least recently used.
* within-batch reuse -- Algorithm 1 processes inputs one after the other and stores each
  miss before the next input is looked up; FLAG_DEDUP gives the rows of one batch that
  behaviour among themselves (pinned against a row-by-row run of the same function).
* f_l          -- Section V-A names the model families; the blocks themselves
  are the textbook post-LN encoder block and pre-LN causal decoder block.

Pins (see tests/test_oracle_*.py): closed forms for the pooling/projection,
brute-force nearest neighbour, threshold invariants, tau > 1 == plain forward,
resubmission hits at similarity 1, torch.nn.functional cross-check of f_l in
float64, scripted LRU trace against a list-based simulation; sign-bit keys:
bit order against a hand-made word, Hamming distance against Python's bit_count,
the angle law of random hyperplanes, monotone agreement with the cosine match.  The paper prints
no worked numerical example, so absolute values rest on those pins alone.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
from scipy.special import erf as _erf

ENCODER_POST_LN = 0
DECODER_PRE_LN = 1
GELU_ERF = 0
GELU_TANH = 1

FLAG_INSERT_ON_MISS = 1
FLAG_UPDATE_LRU = 2
FLAG_REVALIDATE = 4
FLAG_DEDUP = 32
FLAG_LOOKUP_LSH = 64

NORM_FLOOR = 1e-12


# ----------------------------------------------------------------------------
# rounding to the bank's storage type
# ----------------------------------------------------------------------------

def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bfloat16 (ties to even); result held in float32.

    The value is first rounded to float32, the precision the device computes
    the normalised vector in, then to bfloat16: the quantised code is decided
    in the kernel's precision.
    """
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    out = r.astype(np.uint32).view(np.float32).copy()
    nan = np.isnan(f)
    out[nan] = np.float32(np.nan)
    return out.reshape(f.shape)


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "f32":
        return np.asarray(x, dtype=np.float32)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------
# step 1: fingerprint (Section IV-B)
# ----------------------------------------------------------------------------

def fingerprint(h: np.ndarray, P: np.ndarray, c: Optional[np.ndarray], dtype: str
                ) -> Tuple[np.ndarray, np.ndarray]:
    """Fingerprint of each sequence in ``h [B, S, d]``.

    p = mean over tokens (embedding aggregation), v = P^T p + c (linear
    dimensionality reduction), u = v / max(|v|, 1e-12), q = u rounded to the
    bank's storage type, qinv = 1 / |q| of the *rounded* key (0 if q == 0).
    Returns (q [B, k] float32 holding storage-type values, qinv [B] float32).
    """
    h = np.asarray(h, dtype=np.float64)
    P = np.asarray(P, dtype=np.float64)
    B, S, d = h.shape
    p = h.sum(axis=1) / float(S)
    v = p @ P
    if c is not None:
        v = v + np.asarray(c, dtype=np.float64)[None, :]
    nrm = np.sqrt((v * v).sum(axis=1))
    u = v / np.maximum(nrm, NORM_FLOOR)[:, None]
    q = round_to_storage(u, dtype)
    return q, inv_norm(q)


def inv_norm(q: np.ndarray) -> np.ndarray:
    """1 / |q| of stored keys (float64 arithmetic, stored as float32); 0 for a zero key."""
    q64 = np.asarray(q, dtype=np.float64)
    n = np.sqrt((q64 * q64).sum(axis=-1))
    out = np.zeros_like(n)
    nz = n > 0
    out[nz] = 1.0 / n[nz]
    return out.astype(np.float32)


# ----------------------------------------------------------------------------
# step 2: match (Section III-C) and step 3: threshold (Section IV-A)
# ----------------------------------------------------------------------------

def similarities(q: np.ndarray, qinv: np.ndarray, bank_fp: np.ndarray, bank_inv_norm: np.ndarray
                 ) -> np.ndarray:
    """Cosine similarity of every query with every bank key, float64 [B, N].

    The cosine is that of the stored vectors: their dot product times both
    stored inverse norms.
    """
    q64 = np.asarray(q, dtype=np.float64)
    b64 = np.asarray(bank_fp, dtype=np.float64)
    dots = q64 @ b64.T
    return dots * np.asarray(qinv, dtype=np.float64)[:, None] * np.asarray(bank_inv_norm, dtype=np.float64)[None, :]


def match(q: np.ndarray, qinv: np.ndarray, bank_fp: np.ndarray, bank_inv_norm: np.ndarray,
          valid: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Best valid bank entry per query: (idx [B] int32, sim [B] float64).

    Lowest slot wins exact ties.  With no valid entry idx = -1 and sim = -inf.
    """
    B = np.asarray(q).shape[0]
    valid = np.asarray(valid).astype(bool)
    if bank_fp is None or valid.size == 0 or not valid.any():
        return np.full((B,), -1, dtype=np.int32), np.full((B,), -np.inf)
    s = similarities(q, qinv, bank_fp, bank_inv_norm)
    s[:, ~valid] = -np.inf
    idx = np.argmax(s, axis=1)           # first occurrence of the maximum
    sim = s[np.arange(B), idx]
    return idx.astype(np.int32), sim


def near_tie_sets(q, qinv, bank_fp, bank_inv_norm, valid, gap: float = 2e-6) -> List[np.ndarray]:
    """Per query, the valid slots whose similarity lies within ``gap`` of the best."""
    valid = np.asarray(valid).astype(bool)
    s = similarities(q, qinv, bank_fp, bank_inv_norm)
    s[:, ~valid] = -np.inf
    best = s.max(axis=1)
    return [np.nonzero(s[b] >= best[b] - gap)[0] for b in range(s.shape[0])]


def threshold(sim: np.ndarray, tau: float) -> np.ndarray:
    """Hit iff the best similarity strictly exceeds tau."""
    return (np.asarray(sim) > float(tau))


# ----------------------------------------------------------------------------
# f_l: transformer blocks (textbook definitions)
# ----------------------------------------------------------------------------

def gelu(x: np.ndarray, kind: int) -> np.ndarray:
    if kind == GELU_ERF:
        return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))
    if kind == GELU_TANH:
        return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))
    raise ValueError(kind)


def layer_norm(x: np.ndarray, g: np.ndarray, b: np.ndarray, eps: float) -> np.ndarray:
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g + b


def attention(x: np.ndarray, wqkv: np.ndarray, bqkv: np.ndarray, wo: np.ndarray, bo: np.ndarray,
              n_heads: int, causal: bool) -> np.ndarray:
    """Multi-head self-attention of one sequence ``x [S, d]`` -> [S, d].

    Linear weights are [out, in].  Rows 0..d-1 of wqkv give Q, d..2d-1 K,
    2d..3d-1 V; head h owns features h*dh..(h+1)*dh-1.  Scores are scaled by
    1/sqrt(dh); a causal mask lets token t see tokens <= t only.
    """
    S, d = x.shape
    dh = d // n_heads
    qkv = x @ wqkv.T + bqkv
    Q, K, V = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
    ctx = np.empty((S, d), dtype=np.float64)
    for hd in range(n_heads):
        sl = slice(hd * dh, (hd + 1) * dh)
        sc = (Q[:, sl] @ K[:, sl].T) / math.sqrt(dh)
        if causal:
            sc = np.where(np.tril(np.ones((S, S), dtype=bool)), sc, -np.inf)
        sc = sc - sc.max(axis=1, keepdims=True)
        e = np.exp(sc)
        p = e / e.sum(axis=1, keepdims=True)
        ctx[:, sl] = p @ V[:, sl]
    return ctx @ wo.T + bo


def _w64(w: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    return {k: np.asarray(v, dtype=np.float64) for k, v in w.items()}


def encoder_layer_post_ln(x: np.ndarray, w: Dict[str, np.ndarray], n_heads: int, eps: float,
                          gelu_kind: int = GELU_ERF) -> np.ndarray:
    """Post-LayerNorm encoder block on one sequence [S, d]:
    x1 = LN1(x + MHA(x)); y = LN2(x1 + W2 gelu(W1 x1 + b1) + b2)."""
    w = _w64(w)
    x = np.asarray(x, dtype=np.float64)
    a = attention(x, w["wqkv"], w["bqkv"], w["wo"], w["bo"], n_heads, causal=False)
    x1 = layer_norm(x + a, w["ln1_g"], w["ln1_b"], eps)
    ff = gelu(x1 @ w["w1"].T + w["b1"], gelu_kind) @ w["w2"].T + w["b2"]
    return layer_norm(x1 + ff, w["ln2_g"], w["ln2_b"], eps)


def decoder_layer_pre_ln(x: np.ndarray, w: Dict[str, np.ndarray], n_heads: int, eps: float,
                         gelu_kind: int = GELU_TANH) -> np.ndarray:
    """Pre-LayerNorm causal decoder block on one sequence [S, d]:
    x1 = x + MHA_causal(LN1(x)); y = x1 + W2 gelu(W1 LN2(x1) + b1) + b2."""
    w = _w64(w)
    x = np.asarray(x, dtype=np.float64)
    a = attention(layer_norm(x, w["ln1_g"], w["ln1_b"], eps), w["wqkv"], w["bqkv"], w["wo"], w["bo"],
                  n_heads, causal=True)
    x1 = x + a
    ff = gelu(layer_norm(x1, w["ln2_g"], w["ln2_b"], eps) @ w["w1"].T + w["b1"], gelu_kind) @ w["w2"].T + w["b2"]
    return x1 + ff


def layer_forward(x: np.ndarray, w: Dict[str, np.ndarray], arch: int, n_heads: int, eps: float,
                  gelu_kind: int) -> np.ndarray:
    """f_l applied to one sequence [S, d] (float64 result)."""
    if arch == ENCODER_POST_LN:
        return encoder_layer_post_ln(x, w, n_heads, eps, gelu_kind)
    if arch == DECODER_PRE_LN:
        return decoder_layer_pre_ln(x, w, n_heads, eps, gelu_kind)
    raise ValueError(arch)


# ----------------------------------------------------------------------------
# fingerprint with prefix attention statistics (Section IV-B, second feature)
# ----------------------------------------------------------------------------

def prefix_attention_mean(h: np.ndarray, w: Dict[str, np.ndarray], arch: int, n_heads: int, eps: float,
                          n_prefix: int) -> np.ndarray:
    """Section IV-B lists, beside the token average, the mean of the initial self-attention outputs as a
    fingerprint feature.  Reading taken here: for each sequence of ``h [B, S, d]`` the layer's own self-attention
    sub-layer is applied to the first ``n_prefix`` tokens ALONE (they attend to each other only; causal in the
    decoder block, after LN1 in the pre-LayerNorm block), and its outputs (after the output projection, before
    the residual) are averaged over those tokens.  Returns a [B, d] float64."""
    h = np.asarray(h, dtype=np.float64)
    w = _w64(w)
    B, S, d = h.shape
    assert 1 <= n_prefix <= S
    out = np.empty((B, d), dtype=np.float64)
    for b in range(B):
        x = h[b, :n_prefix]
        if arch == DECODER_PRE_LN:
            x = layer_norm(x, w["ln1_g"], w["ln1_b"], eps)
        a = attention(x, w["wqkv"], w["bqkv"], w["wo"], w["bo"], n_heads, causal=(arch == DECODER_PRE_LN))
        out[b] = a.sum(axis=0) / float(n_prefix)
    return out


def fingerprint_prefix(h: np.ndarray, P2: np.ndarray, c: Optional[np.ndarray], dtype: str, w: Dict[str, np.ndarray],
                       arch: int, n_heads: int, eps: float, n_prefix: int) -> Tuple[np.ndarray, np.ndarray]:
    """Fingerprint over the two features of Section IV-B: the token average p [d] and the prefix attention mean
    a [d], reduced together by one linear map: v = P2^T [p; a] + c with P2 [2 d, k]; normalisation, rounding and
    the inverse norm as in ``fingerprint``."""
    h = np.asarray(h, dtype=np.float64)
    P2 = np.asarray(P2, dtype=np.float64)
    B, S, d = h.shape
    assert P2.shape[0] == 2 * d
    p = h.sum(axis=1) / float(S)
    a = prefix_attention_mean(h, w, arch, n_heads, eps, n_prefix)
    v = np.concatenate([p, a], axis=1) @ P2
    if c is not None:
        v = v + np.asarray(c, dtype=np.float64)[None, :]
    nrm = np.sqrt((v * v).sum(axis=1))
    u = v / np.maximum(nrm, NORM_FLOOR)[:, None]
    q = round_to_storage(u, dtype)
    return q, inv_norm(q)


# ----------------------------------------------------------------------------
# the bank C_l (Section III-B) with insertion and LRU (Sections III-E, IV-D)
# ----------------------------------------------------------------------------
# sign-bit keys (Section IV-B names SimHash as a reduction, Section III-A MinHash- or SimHash-based
# hashing; Section IV-B: keys are compared by cosine similarity or by LSH)
# ----------------------------------------------------------------------------
#
# The real-valued key above is the SimHash projection before the sign is taken.
# Taking the sign of each of the k projections gives a k-bit key; two keys are
# compared by their Hamming distance H, and cos(pi * H / k) estimates the cosine
# of the angle between the pooled vectors (each random hyperplane separates two
# vectors with probability angle / pi).  The threshold of the case equation is
# applied to that estimate: hit  <=>  cos(pi * H / k) > tau  <=>  H <= max_hamming(tau, k).
# The paper fixes neither the bit order nor the sign of zero; here bit i of a key
# is word i // 32, position i % 32 (least significant first), and v_i >= 0 gives 1.

NO_MATCH_DIST = 0x7FFFFFFF


def simhash_projection(h: np.ndarray, P: np.ndarray, c: Optional[np.ndarray]) -> np.ndarray:
    """v = P^T mean_t(h) + c for each sequence, float64 [B, k] (the values whose signs are the key)."""
    h = np.asarray(h, dtype=np.float64)
    P = np.asarray(P, dtype=np.float64)
    p = h.sum(axis=1) / float(h.shape[1])
    v = p @ P
    if c is not None:
        v = v + np.asarray(c, dtype=np.float64)[None, :]
    return v


def pack_bits(bits: np.ndarray) -> np.ndarray:
    """[.., k] booleans -> [.., k / 32] uint32 words; bit i sits in word i // 32 at position i % 32."""
    bits = np.asarray(bits).astype(bool)
    k = bits.shape[-1]
    assert k % 32 == 0
    out = np.zeros(bits.shape[:-1] + (k // 32,), dtype=np.uint32)
    for i in range(k):
        out[..., i // 32] |= (bits[..., i].astype(np.uint32) << np.uint32(i % 32))
    return out


def unpack_bits(words: np.ndarray, k: int) -> np.ndarray:
    """Inverse of pack_bits: [.., k / 32] uint32 -> [.., k] booleans."""
    words = np.asarray(words, dtype=np.uint32)
    out = np.zeros(words.shape[:-1] + (k,), dtype=bool)
    for i in range(k):
        out[..., i] = ((words[..., i // 32] >> np.uint32(i % 32)) & np.uint32(1)).astype(bool)
    return out


def fingerprint_bits(h: np.ndarray, P: np.ndarray, c: Optional[np.ndarray]) -> np.ndarray:
    """Sign-bit key of each sequence: packed uint32 [B, k / 32]."""
    return pack_bits(simhash_projection(h, P, c) >= 0.0)


def hamming(q_words: np.ndarray, bank_words: np.ndarray, k: int) -> np.ndarray:
    """Hamming distance of every query key with every bank key, int64 [B, N]."""
    qb = unpack_bits(q_words, k)
    bb = unpack_bits(bank_words, k)
    out = np.zeros((qb.shape[0], bb.shape[0]), dtype=np.int64)
    for i in range(k):
        out += (qb[:, i][:, None] != bb[:, i][None, :])
    return out


def match_bits(q_words: np.ndarray, bank_words: np.ndarray, valid: np.ndarray, k: int
               ) -> Tuple[np.ndarray, np.ndarray]:
    """Nearest valid bank key per query by Hamming distance: (idx [B] int32, dist [B] int32).

    Lowest slot wins ties.  With no valid entry idx = -1 and dist = NO_MATCH_DIST.
    """
    B = np.asarray(q_words).shape[0]
    valid = np.asarray(valid).astype(bool)
    if valid.size == 0 or not valid.any():
        return np.full((B,), -1, np.int32), np.full((B,), NO_MATCH_DIST, np.int32)
    H = hamming(q_words, bank_words, k)
    H[:, ~valid] = NO_MATCH_DIST
    idx = np.argmin(H, axis=1)            # first occurrence of the minimum
    return idx.astype(np.int32), H[np.arange(B), idx].astype(np.int32)


def lsh_candidates(q_words: np.ndarray, bank_words: np.ndarray, valid: np.ndarray, k: int) -> np.ndarray:
    """Bucketed lookup (Section IV-B, LSH; Section III-A wants the comparison cost below linear): the key is cut into
    k / 16 bands of 16 bits (band b = bits 16 b .. 16 b + 15); a bank entry is a CANDIDATE for a query iff it is
    valid and at least one band is equal in both keys.  Returns the boolean [B, N] candidate matrix."""
    q16 = np.asarray(q_words, dtype=np.uint32)
    b16 = np.asarray(bank_words, dtype=np.uint32)
    valid = np.asarray(valid).astype(bool)
    cand = np.zeros((q16.shape[0], b16.shape[0]), dtype=bool)
    for band in range(k // 16):
        w, sh = band // 2, np.uint32(16 * (band % 2))
        qv = (q16[:, w] >> sh) & np.uint32(0xFFFF)
        bv = (b16[:, w] >> sh) & np.uint32(0xFFFF)
        cand |= (qv[:, None] == bv[None, :])
    return cand & valid[None, :]


def match_bits_lsh(q_words: np.ndarray, bank_words: np.ndarray, valid: np.ndarray, k: int
                   ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Nearest CANDIDATE by Hamming distance: (idx, dist, number of distinct candidates).  Lowest slot wins ties;
    no candidate: idx -1, dist NO_MATCH_DIST.  The result equals match_bits whenever the true nearest entry shares
    a whole band with the query, which is what makes the lookup sub-linear: only bucket members are compared."""
    cand = lsh_candidates(q_words, bank_words, valid, k)
    B = cand.shape[0]
    H = hamming(q_words, bank_words, k)
    H[~cand] = NO_MATCH_DIST
    idx = np.argmin(H, axis=1)
    dist = H[np.arange(B), idx]
    none = ~cand.any(axis=1)
    idx = np.where(none, -1, idx)
    return idx.astype(np.int32), dist.astype(np.int32), cand.sum(axis=1).astype(np.int32)


def cosine_estimate(dist: np.ndarray, k: int) -> np.ndarray:
    """cos(pi * H / k): the cosine that a Hamming distance H between k-bit sign keys stands for."""
    return np.cos(np.pi * np.asarray(dist, dtype=np.float64) / float(k))


def max_hamming(tau: float, k: int) -> int:
    """Largest H in 0..k with cos(pi * H / k) > tau; -1 if there is none (tau >= 1)."""
    best = -1
    for H in range(k + 1):
        if math.cos(math.pi * H / k) > tau:
            best = H
    return best


def threshold_bits(idx: np.ndarray, dist: np.ndarray, max_h: int) -> np.ndarray:
    """Hit iff a valid entry was found within max_h bits."""
    return (np.asarray(idx) >= 0) & (np.asarray(dist) <= int(max_h))


# ----------------------------------------------------------------------------

class Bank:
    """One layer's cache bank: keys ``fp [N, k]``, values ``act [A, S, d]``.

    ``act_slot[j]`` names the value row of key j (identity when A == N).
    ``last_used[j]`` is the tick of the entry's insertion or latest hit,
    ``hits[j]`` its number of hits since insertion.
    """

    def __init__(self, n_slots: int, k: int, S: int, d: int, dtype: str,
                 n_act_slots: Optional[int] = None, lru: bool = True, decayed_hits: bool = False,
                 half_life: int = 0, basis: Optional[np.ndarray] = None, key_bits: bool = False):
        A = n_slots if n_act_slots is None else n_act_slots
        # sign-bit keys: fp holds k / 32 uint32 words per entry, compared by Hamming distance
        self.key_bits = key_bits
        self.N, self.k, self.S, self.d, self.A = n_slots, k, S, d, A
        self.dtype = dtype
        # compressed cached values (Section III-B: cached representations may be stored compressed, by PCA):
        # with a basis U [r, d] (rows = principal directions) an entry stores the coefficients
        # C = h U^T [S, r] in the bank's storage type, and a hit returns the reconstruction C U
        self.basis = None if basis is None else np.asarray(basis, dtype=np.float64)
        self.rank = 0 if basis is None else int(self.basis.shape[0])
        self.lru = lru or decayed_hits
        # staleness-aware replacement (Section IV-D, second policy; Section III-E: frequency-based policy and
        # temporal decay): entries are ranked by their hit count, which is halved every `half_life` ticks
        # (0 = never), then by recency, then by slot
        self.decayed_hits = decayed_hits
        self.half_life = half_life
        self.epoch = 0
        self.fp = np.zeros((n_slots, k // 32), dtype=np.uint32) if key_bits else np.zeros((n_slots, k), dtype=np.float32)
        self.inv_norm = np.zeros((n_slots,), dtype=np.float32)
        self.act = np.zeros((A, S, d if basis is None else self.rank), dtype=np.float32)
        self.act_slot = np.arange(n_slots, dtype=np.int32) if A == n_slots else np.zeros((n_slots,), np.int32)
        self.last_used = np.zeros((n_slots,), dtype=np.uint64)
        self.hits = np.zeros((n_slots,), dtype=np.uint32)
        self.valid = np.zeros((n_slots,), dtype=np.uint8)

    # -- cached values -------------------------------------------------------
    def encode(self, h: np.ndarray) -> np.ndarray:
        """What is stored for an output h [S, d]: h itself, or its coefficients on the basis, rounded to storage."""
        if self.basis is None:
            return h
        return round_to_storage(np.asarray(h, dtype=np.float64) @ self.basis.T, self.dtype)

    def value(self, vslot: int) -> np.ndarray:
        """What a hit on value row ``vslot`` returns: the stored output, or its reconstruction C U (float64)."""
        if self.basis is None:
            return self.act[vslot]
        return np.asarray(self.act[vslot], dtype=np.float64) @ self.basis

    # -- temporal decay ------------------------------------------------------
    def advance(self, tick: int) -> None:
        """Bring the hit counts to the epoch of ``tick`` (epoch = tick // half_life): one halving per epoch
        gone by, at most 31.  Called with the tick of every update before the update itself."""
        if not self.decayed_hits or self.half_life <= 0:
            return
        e = int(tick) // self.half_life
        if e > self.epoch:
            sh = min(31, e - self.epoch)
            for j in range(self.N):
                if self.valid[j]:
                    self.hits[j] = np.uint32(int(self.hits[j]) >> sh)
            self.epoch = e

    def _victim_key(self, j: int):
        if self.decayed_hits:
            return (min(int(self.hits[j]), 65535), int(self.last_used[j]), j)
        return (int(self.last_used[j]), j)

    # -- selection -----------------------------------------------------------
    def select_slots(self, m: int) -> List[int]:
        """Slots that the next ``m`` insertions take, in order: free slots by
        ascending index, then -- bank full -- valid entries by ascending
        (last_used, slot).  Raises if the bank is full and eviction is off."""
        free = [j for j in range(self.N) if not self.valid[j]]
        out = free[:m]
        if len(out) < m:
            if not self.lru:
                raise RuntimeError("bank full and eviction disabled")
            order = sorted((j for j in range(self.N) if self.valid[j]), key=self._victim_key)
            out += order[:m - len(out)]
        return out

    def lru_victims(self, m: int) -> List[int]:
        """The ``m`` first victims among valid entries: ascending (last_used, slot), or with the decayed-hits
        policy ascending (min(hits, 65535), last_used, slot)."""
        order = sorted((j for j in range(self.N) if self.valid[j]), key=self._victim_key)
        return order[:m]

    # -- updates -------------------------------------------------------------
    def insert(self, q: np.ndarray, qinv: np.ndarray, acts: np.ndarray, tick: int) -> Tuple[List[int], int]:
        """Store ``m`` (key, value) pairs; returns (slots taken, number evicted)."""
        self.advance(tick)
        m = q.shape[0]
        slots = self.select_slots(m)
        n_evicted = 0
        for i, j in enumerate(slots):
            n_evicted += int(self.valid[j])
            self.fp[j] = q[i]
            self.inv_norm[j] = qinv[i]
            self.act[self.act_slot[j]] = self.encode(acts[i])
            self.last_used[j] = tick
            self.hits[j] = 0
            self.valid[j] = 1
        return slots, n_evicted

    def evict(self, m: int) -> List[int]:
        """Invalidate the ``m`` least recently used entries; returns them in eviction order."""
        v = self.lru_victims(m)
        for j in v:
            self.valid[j] = 0
        return v

    def touch(self, slots: Sequence[int], tick: int) -> None:
        """Record hits: refresh recency and count the hit."""
        self.advance(tick)
        for j in slots:
            self.last_used[j] = tick
            self.hits[j] += 1


# ----------------------------------------------------------------------------
# the gated layer (Section IV-A case equation, Algorithm 1 loop body)
# ----------------------------------------------------------------------------

@dataclass
class GateResult:
    h_out: np.ndarray          # [B, S, d] float64; hit rows hold the cached values exactly
    q: np.ndarray              # [B, k] stored-type fingerprint
    qinv: np.ndarray           # [B]
    idx: np.ndarray            # [B] int32 best slot (-1: empty bank)
    sim: np.ndarray            # [B] float64 best similarity
    hit: np.ndarray            # [B] bool
    slots: List[int]           # slots taken by this batch's insertions (ascending miss row order)
    n_evicted: int
    revalidated: List[int] = None   # hit rows that were re-computed (divergence monitor), ascending
    divergence: List[float] = None  # their divergence from the cached value
    refreshed: List[int] = None     # slots whose cached value was replaced by the fresh output
    follower_of: Dict[int, int] = None  # FLAG_DEDUP: row -> the earlier row of the batch whose fresh entry it reused


def gated_layer(h_in: np.ndarray, bank: Optional[Bank], P: Optional[np.ndarray], c: Optional[np.ndarray],
                w: Dict[str, np.ndarray], arch: int, n_heads: int, eps: float, gelu_kind: int,
                tau: float, flags: int = 0, tick: int = 0, out_dtype: Optional[str] = None,
                fp_override: Optional[Tuple[np.ndarray, np.ndarray]] = None, reval_every: int = 0,
                drift_bound: float = 0.0) -> GateResult:
    """One trip of Algorithm 1's loop body for a whole batch.

    The batch is matched against the bank as it stands on entry; insertions
    become visible to the next call.  ``bank is None`` means the layer is not
    cached and is computed plainly (Section VI-D, layer selection).
    ``out_dtype`` rounds the *stored* value on insertion (the bank holds
    storage-type values); h_out itself is returned unrounded for miss rows.
    ``fp_override`` supplies (q, qinv) instead of fingerprinting h_in
    (Algorithm 1 taken literally: one fingerprint of the input for all layers).

    Divergence monitor (Section IV-D third item; Section III-E: the outputs that successive
    calls produce for one fingerprint are compared), with FLAG_REVALIDATE and
    ``reval_every`` = r >= 1: a hit row b with (tick + b) % r == 0 is computed anyway; its
    output is the fresh f_l(h_in[b]); its divergence is max|fresh - cached| / max|cached|
    (1e-30 floor); above ``drift_bound`` the entry's cached value is replaced by the fresh
    output (stored in ``out_dtype``), the key stays; if several sampled rows of the batch
    matched one entry, the lowest row alone decides.  The row still counts as a hit and is
    not inserted again.
    """
    h_in = np.asarray(h_in, dtype=np.float64)
    B, S, d = h_in.shape
    h_out = np.empty((B, S, d), dtype=np.float64)
    if bank is None:
        for b in range(B):
            h_out[b] = layer_forward(h_in[b], w, arch, n_heads, eps, gelu_kind)
        return GateResult(h_out, np.zeros((B, 0), np.float32), np.zeros((B,), np.float32),
                          np.full((B,), -1, np.int32), np.full((B,), -np.inf), np.zeros((B,), bool), [], 0)
    if bank.key_bits:
        # sign-bit keys: Hamming match, threshold on the cosine that the distance stands for
        q = fp_override[0] if fp_override is not None else fingerprint_bits(h_in, P, c)
        qinv = np.zeros((B,), np.float32)
        if flags & FLAG_LOOKUP_LSH:
            # bucketed lookup (Section IV-B, LSH): only slots that share one whole band with the query are compared
            idx, dist, _ = match_bits_lsh(q, bank.fp, bank.valid, bank.k)
        else:
            idx, dist = match_bits(q, bank.fp, bank.valid, bank.k)
        hit = threshold_bits(idx, dist, max_hamming(tau, bank.k))
        sim = np.where(idx >= 0, cosine_estimate(np.minimum(dist, bank.k), bank.k), -np.inf)
    else:
        if fp_override is not None:
            q, qinv = fp_override
        else:
            q, qinv = fingerprint(h_in, P, c, bank.dtype)
        idx, sim = match(q, qinv, bank.fp, bank.inv_norm, bank.valid)
        hit = threshold(sim, tau)
    revalidated: List[int] = []
    divergence: List[float] = []
    refreshed: List[int] = []
    # Within-batch reuse (Algorithm 1 run over the rows of the batch one after the other: a row can hit what an
    # EARLIER row of the same batch has just stored).  Rows that miss the bank as it stood are taken in ascending
    # order; a row is a LEADER unless its key is more similar than tau to the key of an earlier leader, in which
    # case it FOLLOWS the most similar earlier leader (the earliest one among equals): it is not computed, it returns
    # the leader's stored output, counts as a hit on the leader's new entry and is not stored again.
    follower_of: Dict[int, int] = {}
    if (flags & FLAG_DEDUP) and (flags & FLAG_INSERT_ON_MISS):
        assert not bank.key_bits and bank.basis is None and not (flags & FLAG_REVALIDATE)
        leaders: List[int] = []
        q64 = np.asarray(q, dtype=np.float64)
        for b in range(B):
            if hit[b]:
                continue
            best, best_s = -1, -np.inf
            for a in leaders:
                s_ab = float(q64[b] @ q64[a]) * float(qinv[b]) * float(qinv[a])
                if s_ab > float(tau) and s_ab > best_s:
                    best, best_s = a, s_ab
            if best < 0:
                leaders.append(b)
            else:
                follower_of[b] = best
                sim[b] = best_s
    for b in range(B):
        if hit[b]:
            h_out[b] = bank.value(int(bank.act_slot[idx[b]]))
        elif b not in follower_of:
            h_out[b] = layer_forward(h_in[b], w, arch, n_heads, eps, gelu_kind)
    if (flags & FLAG_REVALIDATE) and reval_every >= 1:
        assert bank.basis is None, "the divergence monitor is not defined for compressed values"
        for b in range(B):
            if hit[b] and (int(tick) + b) % int(reval_every) == 0:
                vslot = int(bank.act_slot[idx[b]])
                cached = np.asarray(bank.act[vslot], dtype=np.float64)
                fresh = layer_forward(h_in[b], w, arch, n_heads, eps, gelu_kind)
                div = float(np.abs(fresh - cached).max() / max(float(np.abs(cached).max()), 1e-30))
                revalidated.append(b)
                divergence.append(div)
                h_out[b] = fresh
        # all comparisons are against the bank as it stood; replacements happen afterwards.  When several
        # sampled rows matched one entry, the lowest row alone decides about that entry.
        decided = set()
        for b, div in zip(revalidated, divergence):
            if int(idx[b]) in decided:
                continue
            decided.add(int(idx[b]))
            if div > float(drift_bound):
                vslot = int(bank.act_slot[idx[b]])
                val = h_out[b]
                if out_dtype is not None:
                    val = round_to_storage(val, out_dtype)
                bank.act[vslot] = val
                refreshed.append(int(idx[b]))
    if flags & FLAG_UPDATE_LRU:
        bank.touch([int(idx[b]) for b in range(B) if hit[b]], tick)
    slots: List[int] = []
    n_evicted = 0
    if flags & FLAG_INSERT_ON_MISS:
        miss = [b for b in range(B) if not hit[b] and b not in follower_of]
        if miss:
            vals = h_out[miss]
            if out_dtype is not None:
                vals = round_to_storage(vals, out_dtype)
            slots, n_evicted = bank.insert(q[miss], qinv[miss], vals, tick)
        if follower_of:
            slot_of = {b: j for b, j in zip(miss, slots)}
            hit = hit.copy()
            idx = idx.copy()
            for b, a in sorted(follower_of.items()):
                j = slot_of[a]
                h_out[b] = bank.value(int(bank.act_slot[j]))      # the leader's output as stored
                hit[b] = True
                idx[b] = j
                if flags & FLAG_UPDATE_LRU:
                    bank.touch([j], tick)
    return GateResult(h_out, q, qinv, idx, sim, hit, slots, n_evicted, revalidated, divergence, refreshed, follower_of)


def infer(h0: np.ndarray, banks: Sequence[Optional[Bank]], Ps: Sequence[np.ndarray],
          cs: Sequence[Optional[np.ndarray]], weights: Sequence[Dict[str, np.ndarray]], arch: int,
          n_heads: int, eps: float, gelu_kind: int, tau: float, flags: int = 0, tick: int = 0,
          out_dtype: Optional[str] = None, single_fingerprint: bool = False, reval_every: int = 0,
          drift_bound: float = 0.0) -> Tuple[np.ndarray, List[GateResult]]:
    """Algorithm 1 for a batch: h_0 through all L gated layers.

    Default: layer l fingerprints its own input h_{l-1} with P_l.  With
    ``single_fingerprint`` the fingerprint of h_0 (under P_1) is computed once
    and reused at every layer, as the algorithm is printed.  If ``out_dtype``
    is given, every layer's output is rounded to it before feeding the next
    layer (the run stores activations in that type).
    """
    h = np.asarray(h0, dtype=np.float64)
    results = []
    fp0 = None
    if single_fingerprint:
        dt = next(b.dtype for b in banks if b is not None)
        fp0 = fingerprint(h, Ps[0], cs[0], dt)
    for l, w in enumerate(weights):
        r = gated_layer(h, banks[l], Ps[l], cs[l], w, arch, n_heads, eps, gelu_kind, tau, flags, tick,
                        out_dtype, fp_override=fp0, reval_every=reval_every, drift_bound=drift_bound)
        results.append(r)
        h = r.h_out
        if out_dtype is not None:
            h = round_to_storage(h, out_dtype).astype(np.float64)
    return h, results
