"""Thin ctypes binding over libllmc.so -- argument marshalling only.

Every function has the name of the C entry point it calls (include/llmc.h) and
passes torch tensors as raw device pointers.  Nothing is computed here; if the
library is missing this module raises instead of falling back to anything.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libllmc.so")

LLMC_OK = 0
ERR_INVALID_ARG, ERR_SHAPE, ERR_DTYPE, ERR_BANK_FULL, ERR_WORKSPACE, ERR_HIP = 1, 2, 3, 4, 5, 6
F32, BF16 = 0, 1
EVICT_NONE, EVICT_LRU, EVICT_DECAYED_HITS = 0, 1, 2
INSERT_ON_MISS, UPDATE_LRU, REVALIDATE, HINT_MOSTLY_CARRIED, DEFER_COPY, DEDUP, LOOKUP_LSH = 1, 2, 4, 8, 16, 32, 64
CNT_HIT, CNT_MISS, CNT_NEAR_TAU, CNT_NEAR_TIE, CNT_INSERTED, CNT_EVICTED, CNT_DROPPED = 0, 1, 2, 3, 4, 5, 6
CNT_COMPUTED, CNT_REVALIDATED, CNT_DIVERGED, CNT_TIE_OVERFLOW, CNT_DEDUP, CNT_WORDS = 7, 8, 9, 10, 11, 12
MAX_UPDATE_ROWS = 4096

EXPORTS = [
    "llmc_bank_create", "llmc_bank_destroy", "llmc_bank_refresh", "llmc_bank_insert", "llmc_bank_evict",
    "llmc_fingerprint", "llmc_fingerprint_workspace_bytes", "llmc_inv_norm", "llmc_match",
    "llmc_match_workspace_bytes", "llmc_gather_hits", "llmc_layer_forward_gated",
    "llmc_layer_workspace_bytes", "llmc_profile_begin", "llmc_profile_report", "llmc_profile_end",
    "llmc_last_error", "llmc_version", "llmc_fingerprint_bits", "llmc_match_bits",
    "llmc_match_bits_workspace_bytes", "llmc_max_hamming", "llmc_bank_pool_values",
    "llmc_lsh_index_bytes", "llmc_lsh_build", "llmc_match_bits_lsh", "llmc_materialize", "llmc_match_noalloc",
    "llmc_fingerprint_prefix", "llmc_fingerprint_prefix_workspace_bytes",
]
MATCH_STATIC_SCRATCH_BYTES = 5 << 20


class BankDesc(C.Structure):
    _fields_ = [("n_slots", C.c_int32), ("k", C.c_int32), ("S", C.c_int32), ("d", C.c_int32),
                ("n_act_slots", C.c_int32), ("dtype", C.c_int32), ("policy", C.c_int32),
                ("d_fp", C.c_void_p), ("d_act", C.c_void_p), ("d_inv_norm", C.c_void_p),
                ("d_act_slot", C.c_void_p), ("d_last_used", C.c_void_p), ("d_hits", C.c_void_p),
                ("d_valid", C.c_void_p), ("half_life", C.c_int32), ("reval_every", C.c_int32),
                ("drift_bound", C.c_float), ("rank", C.c_int32), ("d_basis", C.c_void_p),
                ("d_act_pool", C.c_void_p), ("d_next_proj", C.c_void_p), ("d_next_bias", C.c_void_p),
                ("next_k", C.c_int32), ("d_next_fp", C.c_void_p), ("d_next_inv", C.c_void_p),
                ("key_bits", C.c_int32), ("d_lsh_index", C.c_void_p), ("lsh_index_bytes", C.c_size_t)]


class LayerDesc(C.Structure):
    _fields_ = [("arch", C.c_int32), ("d", C.c_int32), ("n_heads", C.c_int32), ("d_ff", C.c_int32),
                ("gelu", C.c_int32), ("ln_eps", C.c_float), ("dtype", C.c_int32),
                ("d_wqkv", C.c_void_p), ("d_bqkv", C.c_void_p), ("d_wo", C.c_void_p), ("d_bo", C.c_void_p),
                ("d_w1", C.c_void_p), ("d_b1", C.c_void_p), ("d_w2", C.c_void_p), ("d_b2", C.c_void_p),
                ("d_ln1_g", C.c_void_p), ("d_ln1_b", C.c_void_p), ("d_ln2_g", C.c_void_p), ("d_ln2_b", C.c_void_p)]


class FpDesc(C.Structure):
    _fields_ = [("d_proj", C.c_void_p), ("d_bias", C.c_void_p), ("k", C.c_int32),
                ("d_pooled_in", C.c_void_p), ("d_pooled_in_valid", C.c_void_p), ("d_key_in", C.c_void_p),
                ("d_key_inv_in", C.c_void_p), ("prev_bank", C.c_void_p), ("d_ref_in", C.c_void_p)]


class GateOut(C.Structure):
    _fields_ = [("d_idx", C.c_void_p), ("d_sim", C.c_void_p), ("d_hit", C.c_void_p),
                ("d_counters", C.c_void_p), ("d_slots", C.c_void_p), ("d_pooled_out", C.c_void_p),
                ("d_pooled_out_valid", C.c_void_p), ("d_key_out", C.c_void_p), ("d_key_inv_out", C.c_void_p),
                ("d_ref_out", C.c_void_p), ("d_fp_used", C.c_void_p), ("d_inv_norm_used", C.c_void_p)]


class LlmcError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__("llmc status %d: %s" % (status, msg))
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """Load libllmc.so (built in-tree by build.py); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libllmc.so is not built: run `python -m paper_2512_16843_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, u32, u64, f32, sz, i64 = C.c_void_p, C.c_int32, C.c_uint32, C.c_uint64, C.c_float, C.c_size_t, C.c_int64
        L.llmc_last_error.restype = C.c_char_p
        L.llmc_version.restype = C.c_char_p
        L.llmc_bank_create.argtypes = [C.POINTER(BankDesc), C.POINTER(vp)]
        L.llmc_bank_destroy.argtypes = [vp]
        L.llmc_bank_refresh.argtypes = [vp, vp]
        L.llmc_bank_insert.argtypes = [vp, vp, vp, vp, vp, vp, i32, u64, vp, vp, vp]
        L.llmc_bank_evict.argtypes = [vp, vp, i32, vp, vp]
        L.llmc_bank_pool_values.argtypes = [vp, vp]
        L.llmc_materialize.argtypes = [vp, vp, i32, vp, vp]
        L.llmc_fingerprint.argtypes = [vp, i32, i32, i32, i32, vp, vp, i32, vp, vp, vp, sz, vp]
        L.llmc_fingerprint_workspace_bytes.argtypes = [i32, i32, i32]
        L.llmc_fingerprint_workspace_bytes.restype = sz
        L.llmc_inv_norm.argtypes = [vp, i64, i32, i32, vp, vp]
        L.llmc_match.argtypes = [vp, vp, vp, i32, f32, vp, vp, vp, vp, vp, sz, vp]
        L.llmc_match_noalloc.argtypes = [vp, vp, vp, i32, f32, vp, vp, vp, vp, vp]
        L.llmc_match_workspace_bytes.argtypes = [vp, i32]
        L.llmc_match_workspace_bytes.restype = sz
        L.llmc_gather_hits.argtypes = [vp, vp, vp, vp, i32, vp, vp]
        L.llmc_layer_forward_gated.argtypes = [C.POINTER(LayerDesc), vp, C.POINTER(FpDesc), vp, vp, i32, i32, f32,
                                               u32, u64, vp, vp, C.POINTER(GateOut), vp, sz, vp]
        L.llmc_layer_workspace_bytes.argtypes = [C.POINTER(LayerDesc), i32, i32, i32]
        L.llmc_layer_workspace_bytes.restype = sz
        L.llmc_fingerprint_prefix.argtypes = [vp, vp, i32, i32, i32, vp, vp, i32, vp, vp, vp, sz, vp]
        L.llmc_fingerprint_prefix_workspace_bytes.argtypes = [vp, i32, i32, i32]
        L.llmc_fingerprint_prefix_workspace_bytes.restype = sz
        L.llmc_fingerprint_bits.argtypes = [vp, i32, i32, i32, i32, vp, vp, i32, vp, vp, sz, vp]
        L.llmc_match_bits.argtypes = [vp, vp, i32, i32, vp, i32, i32, vp, vp, vp, vp, sz, vp]
        L.llmc_match_bits_workspace_bytes.argtypes = [i32, i32, i32]
        L.llmc_match_bits_workspace_bytes.restype = sz
        L.llmc_max_hamming.argtypes = [f32, i32]
        L.llmc_lsh_index_bytes.argtypes = [i32, i32]
        L.llmc_lsh_index_bytes.restype = sz
        L.llmc_lsh_build.argtypes = [vp, vp, i32, i32, vp, sz, vp]
        L.llmc_match_bits_lsh.argtypes = [vp, i32, i32, vp, sz, vp, i32, i32, vp, vp, vp, vp, vp]
        L.llmc_max_hamming.restype = i32
        L.llmc_profile_begin.argtypes = [i32]
        L.llmc_profile_report.argtypes = [C.c_char_p, sz]
        L.llmc_profile_report.restype = i32
        L.llmc_profile_end.argtypes = []
        for name in EXPORTS:
            fn = getattr(L, name)
            if fn.restype is C.c_int:
                fn.restype = C.c_int
        _lib = L
    return _lib


def _check(st: int) -> None:
    if st != LLMC_OK:
        raise LlmcError(st, lib().llmc_last_error().decode())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_contiguous(), "llmc takes contiguous tensors"
    return t.data_ptr()


def _stream(stream: Optional[torch.cuda.Stream]) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return F32
    if dt == torch.bfloat16:
        return BF16
    raise LlmcError(ERR_DTYPE, "unsupported torch dtype %s" % dt)


# ---------------------------------------------------------------------------
# bank
# ---------------------------------------------------------------------------

class Bank:
    """Device arrays of one layer's bank plus the library handle wrapping them."""

    def __init__(self, n_slots: int, k: int, S: int, d: int, dtype: torch.dtype, device="cuda",
                 n_act_slots: Optional[int] = None, policy: int = EVICT_LRU,
                 act_slot: Optional[torch.Tensor] = None, half_life: int = 0, reval_every: int = 0,
                 drift_bound: float = 0.0, basis: Optional[torch.Tensor] = None, keep_means: bool = False,
                 next_proj: Optional[torch.Tensor] = None, next_bias: Optional[torch.Tensor] = None,
                 key_bits: bool = False, lsh: bool = False):
        A = n_slots if n_act_slots is None else n_act_slots
        self.n_slots, self.k, self.S, self.d, self.n_act_slots = n_slots, k, S, d, A
        self.dtype = dtype
        self.key_bits = key_bits          # keys are sign bits: int32 words [n_slots, k / 32]
        self.fp = torch.zeros((n_slots, k // 32), dtype=torch.int32, device=device) if key_bits else \
            torch.zeros((n_slots, k), dtype=dtype, device=device)
        self.inv_norm = torch.zeros((n_slots,), dtype=torch.float32, device=device)
        self.basis = basis          # [rank, d]: cached values are stored as coefficients on it
        self.rank = 0 if basis is None else int(basis.shape[0])
        self.act = torch.zeros((A, S, d if basis is None else self.rank), dtype=dtype, device=device)
        self.act_slot = act_slot
        # token mean of every cached output (the next layer's pooled input of a hit)
        self.act_pool = torch.zeros((A, d), dtype=torch.float32, device=device) if keep_means else None
        # the key of every cached output under the NEXT layer's fingerprint map (needs keep_means)
        self.next_proj, self.next_bias = next_proj, next_bias
        self.next_k = 0 if next_proj is None else int(next_proj.shape[1])
        self.next_fp = torch.zeros((A, self.next_k), dtype=dtype, device=device) if next_proj is not None else None
        self.next_inv = torch.zeros((A,), dtype=torch.float32, device=device) if next_proj is not None else None
        self.last_used = torch.zeros((n_slots,), dtype=torch.int64, device=device)   # uint64 bit pattern
        self.hits = torch.zeros((n_slots,), dtype=torch.int32, device=device)        # uint32 bit pattern
        self.valid = torch.zeros((n_slots,), dtype=torch.uint8, device=device)
        self.policy = policy
        self.half_life = half_life
        self.reval_every, self.drift_bound = reval_every, drift_bound
        # bucket index of sign-bit keys (kept current by the library)
        self.lsh_index = torch.zeros((lib().llmc_lsh_index_bytes(n_slots, k),), dtype=torch.uint8, device=device) \
            if (lsh and key_bits) else None
        self.handle = None
        self.create()

    def desc(self) -> BankDesc:
        return BankDesc(self.n_slots, self.k, self.S, self.d, self.n_act_slots, dtype_code(self.dtype), self.policy,
                        _ptr(self.fp), _ptr(self.act), _ptr(self.inv_norm), _ptr(self.act_slot),
                        _ptr(self.last_used), _ptr(self.hits), _ptr(self.valid), self.half_life, self.reval_every,
                        self.drift_bound, self.rank, _ptr(self.basis), _ptr(self.act_pool), _ptr(self.next_proj),
                        _ptr(self.next_bias), self.next_k, _ptr(self.next_fp), _ptr(self.next_inv), 1 if self.key_bits else 0,
                        _ptr(self.lsh_index), 0 if self.lsh_index is None else self.lsh_index.numel())

    def create(self) -> None:
        torch.cuda.synchronize()
        self.handle = llmc_bank_create(self.desc())

    def refresh(self, stream=None) -> None:
        llmc_bank_refresh(self.handle, stream)

    def close(self) -> None:
        if self.handle is not None:
            llmc_bank_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def llmc_bank_create(desc: BankDesc) -> int:
    out = C.c_void_p()
    _check(lib().llmc_bank_create(C.byref(desc), C.byref(out)))
    return out.value


def llmc_bank_destroy(handle: int) -> None:
    _check(lib().llmc_bank_destroy(handle))


def llmc_bank_refresh(handle: int, stream=None) -> None:
    _check(lib().llmc_bank_refresh(handle, _stream(stream)))


def llmc_bank_insert(bank: Bank, fp: torch.Tensor, inv_norm: torch.Tensor, act: torch.Tensor,
                     rows: Optional[torch.Tensor], m: Optional[torch.Tensor], m_max: int, tick: int,
                     slots_out: torch.Tensor, counters: Optional[torch.Tensor] = None, stream=None) -> None:
    _check(lib().llmc_bank_insert(bank.handle, _ptr(fp), _ptr(inv_norm), _ptr(act), _ptr(rows), _ptr(m), m_max, tick,
                                  _ptr(slots_out), _ptr(counters), _stream(stream)))


def llmc_bank_pool_values(bank: Bank, stream=None) -> None:
    _check(lib().llmc_bank_pool_values(bank.handle, _stream(stream)))


def llmc_bank_evict(bank: Bank, m: Optional[torch.Tensor], m_max: int, victims_out: torch.Tensor, stream=None) -> None:
    _check(lib().llmc_bank_evict(bank.handle, _ptr(m), m_max, _ptr(victims_out), _stream(stream)))


# ---------------------------------------------------------------------------
# fingerprint / match / gather
# ---------------------------------------------------------------------------

def llmc_fingerprint_workspace_bytes(B: int, S: int, d: int) -> int:
    return lib().llmc_fingerprint_workspace_bytes(B, S, d)


def llmc_fingerprint(h: torch.Tensor, proj: torch.Tensor, bias: Optional[torch.Tensor], fp_out: torch.Tensor,
                     inv_norm_out: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    B, S, d = h.shape
    _check(lib().llmc_fingerprint(_ptr(h), B, S, d, dtype_code(h.dtype), _ptr(proj), _ptr(bias), proj.shape[1],
                                  _ptr(fp_out), _ptr(inv_norm_out), _ptr(workspace), workspace.numel(),
                                  _stream(stream)))


def llmc_fingerprint_prefix_workspace_bytes(layer: "LayerDesc", B: int, S: int, n_prefix: int) -> int:
    return lib().llmc_fingerprint_prefix_workspace_bytes(C.byref(layer), B, S, n_prefix)


def llmc_fingerprint_prefix(layer: "LayerDesc", h: torch.Tensor, n_prefix: int, proj2: torch.Tensor,
                            bias: Optional[torch.Tensor], fp_out: torch.Tensor, inv_norm_out: torch.Tensor,
                            workspace: torch.Tensor, stream=None) -> None:
    """Keys from the token average and the prefix attention mean together; proj2 is [2 d, k]."""
    B, S, d = h.shape
    _check(lib().llmc_fingerprint_prefix(C.byref(layer), _ptr(h), B, S, n_prefix, _ptr(proj2), _ptr(bias),
                                         proj2.shape[1], _ptr(fp_out), _ptr(inv_norm_out), _ptr(workspace),
                                         workspace.numel(), _stream(stream)))


def llmc_inv_norm(fp: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    n, k = fp.shape
    _check(lib().llmc_inv_norm(_ptr(fp), n, k, dtype_code(fp.dtype), _ptr(out), _stream(stream)))


def llmc_match_workspace_bytes(bank: Bank, B: int) -> int:
    return lib().llmc_match_workspace_bytes(bank.handle, B)


def llmc_match(bank: Bank, fp: torch.Tensor, inv_norm: torch.Tensor, tau: float, idx: torch.Tensor,
               sim: Optional[torch.Tensor], hit: Optional[torch.Tensor], near_tie: Optional[torch.Tensor],
               workspace: torch.Tensor, stream=None) -> None:
    _check(lib().llmc_match(bank.handle, _ptr(fp), _ptr(inv_norm), fp.shape[0], tau, _ptr(idx), _ptr(sim), _ptr(hit),
                            _ptr(near_tie), _ptr(workspace), workspace.numel(), _stream(stream)))


def llmc_match_noalloc(bank: Bank, fp: torch.Tensor, inv_norm: torch.Tensor, tau: float, idx: torch.Tensor,
                       sim: Optional[torch.Tensor], hit: Optional[torch.Tensor], near_tie: Optional[torch.Tensor],
                       stream=None) -> None:
    _check(lib().llmc_match_noalloc(bank.handle, _ptr(fp), _ptr(inv_norm), fp.shape[0], tau, _ptr(idx), _ptr(sim),
                                    _ptr(hit), _ptr(near_tie), _stream(stream)))


def llmc_fingerprint_bits(h: torch.Tensor, proj: torch.Tensor, bias: Optional[torch.Tensor], bits_out: torch.Tensor,
                          workspace: torch.Tensor, stream=None) -> None:
    """Sign-bit keys: bits_out [B, k / 32] int32 (the words' bit patterns)."""
    B, S, d = h.shape
    assert bits_out.dtype == torch.int32 and tuple(bits_out.shape) == (B, proj.shape[1] // 32)
    _check(lib().llmc_fingerprint_bits(_ptr(h), B, S, d, dtype_code(h.dtype), _ptr(proj), _ptr(bias), proj.shape[1],
                                       _ptr(bits_out), _ptr(workspace), workspace.numel(), _stream(stream)))


def llmc_match_bits_workspace_bytes(N: int, k: int, B: int) -> int:
    return lib().llmc_match_bits_workspace_bytes(N, k, B)


def llmc_max_hamming(tau: float, k: int) -> int:
    return lib().llmc_max_hamming(tau, k)


def llmc_match_bits(bank_bits: torch.Tensor, valid: torch.Tensor, query_bits: torch.Tensor, max_hamming: int,
                    idx: torch.Tensor, dist: Optional[torch.Tensor], hit: Optional[torch.Tensor],
                    workspace: torch.Tensor, stream=None) -> None:
    N, W = bank_bits.shape
    assert bank_bits.dtype == torch.int32 and query_bits.dtype == torch.int32 and query_bits.shape[1] == W
    _check(lib().llmc_match_bits(_ptr(bank_bits), _ptr(valid), N, W * 32, _ptr(query_bits), query_bits.shape[0],
                                 max_hamming, _ptr(idx), _ptr(dist), _ptr(hit), _ptr(workspace), workspace.numel(),
                                 _stream(stream)))


def llmc_lsh_index_bytes(N: int, k: int) -> int:
    return lib().llmc_lsh_index_bytes(N, k)


def llmc_lsh_build(bank_bits: torch.Tensor, valid: torch.Tensor, index: torch.Tensor, stream=None) -> None:
    N, W = bank_bits.shape
    _check(lib().llmc_lsh_build(_ptr(bank_bits), _ptr(valid), N, W * 32, _ptr(index), index.numel(), _stream(stream)))


def llmc_match_bits_lsh(bank_bits: torch.Tensor, index: torch.Tensor, query_bits: torch.Tensor, max_hamming: int,
                        idx: torch.Tensor, dist: Optional[torch.Tensor], hit: Optional[torch.Tensor],
                        compared: Optional[torch.Tensor] = None, stream=None) -> None:
    N, W = bank_bits.shape
    _check(lib().llmc_match_bits_lsh(_ptr(bank_bits), N, W * 32, _ptr(index), index.numel(), _ptr(query_bits),
                                     query_bits.shape[0], max_hamming, _ptr(idx), _ptr(dist), _ptr(hit), _ptr(compared),
                                     _stream(stream)))


def llmc_materialize(bank: Bank, ref: torch.Tensor, h: torch.Tensor, stream=None) -> None:
    _check(lib().llmc_materialize(bank.handle, _ptr(ref), h.shape[0], _ptr(h), _stream(stream)))


def llmc_gather_hits(bank: Bank, idx: torch.Tensor, rows: Optional[torch.Tensor], n: Optional[torch.Tensor],
                     n_max: int, h_out: torch.Tensor, stream=None) -> None:
    _check(lib().llmc_gather_hits(bank.handle, _ptr(idx), _ptr(rows), _ptr(n), n_max, _ptr(h_out), _stream(stream)))


# ---------------------------------------------------------------------------
# the gated layer
# ---------------------------------------------------------------------------

@dataclass
class Layer:
    """Device weights of one block and its descriptor."""
    arch: int
    d: int
    n_heads: int
    d_ff: int
    gelu: int
    ln_eps: float
    dtype: torch.dtype
    w: Dict[str, torch.Tensor]

    def desc(self) -> LayerDesc:
        w = self.w
        return LayerDesc(self.arch, self.d, self.n_heads, self.d_ff, self.gelu, self.ln_eps, dtype_code(self.dtype),
                         _ptr(w["wqkv"]), _ptr(w["bqkv"]), _ptr(w["wo"]), _ptr(w["bo"]), _ptr(w["w1"]), _ptr(w["b1"]),
                         _ptr(w["w2"]), _ptr(w["b2"]), _ptr(w["ln1_g"]), _ptr(w["ln1_b"]), _ptr(w["ln2_g"]),
                         _ptr(w["ln2_b"]))


def llmc_layer_workspace_bytes(layer: Layer, B: int, S: int, k: int) -> int:
    d = layer.desc()
    return lib().llmc_layer_workspace_bytes(C.byref(d), B, S, k)


class GateBuffers:
    """Optional per-row outputs of the gate, allocated once per (B)."""

    def __init__(self, B: int, device="cuda", d: int = 0, next_k: int = 0, dtype: torch.dtype = torch.bfloat16,
                 counters: Optional[torch.Tensor] = None, k_used: int = 0, key_bits: bool = False):
        # d > 0: also the buffers that carry the token means of reused rows to the next layer;
        # next_k > 0: and their finished keys under the next layer's fingerprint map
        self.pooled = torch.zeros((B, d), dtype=torch.float32, device=device) if d > 0 else None
        self.pooled_valid = torch.zeros((B,), dtype=torch.uint8, device=device) if d > 0 else None
        self.key = torch.zeros((B, next_k), dtype=dtype, device=device) if next_k > 0 else None
        self.key_inv = torch.zeros((B,), dtype=torch.float32, device=device) if next_k > 0 else None
        # deferred copies: value row of the entry that answered a row, -1 where the row was written
        self.ref = torch.full((B,), -1, dtype=torch.int32, device=device)
        self.idx = torch.empty((B,), dtype=torch.int32, device=device)
        self.sim = torch.empty((B,), dtype=torch.float32, device=device)
        self.hit = torch.empty((B,), dtype=torch.uint8, device=device)
        # the counters may be a row of a caller's [layers, CNT_WORDS] block, so that one copy fetches all layers
        self.counters = torch.zeros((CNT_WORDS,), dtype=torch.int32, device=device) if counters is None else counters
        self.slots = torch.empty((B,), dtype=torch.int32, device=device)
        # k_used > 0: the keys the rows were matched with (and their inverse norms) are written here
        self.fp_used = None if k_used <= 0 else (
            torch.zeros((B, k_used // 32), dtype=torch.int32, device=device) if key_bits else
            torch.zeros((B, k_used), dtype=dtype, device=device))
        self.inv_used = torch.zeros((B,), dtype=torch.float32, device=device) if k_used > 0 else None

    def struct(self) -> GateOut:
        return GateOut(_ptr(self.idx), _ptr(self.sim), _ptr(self.hit), _ptr(self.counters), _ptr(self.slots),
                       _ptr(self.pooled), _ptr(self.pooled_valid), _ptr(self.key), _ptr(self.key_inv), _ptr(self.ref),
                       _ptr(self.fp_used), _ptr(self.inv_used))


def llmc_layer_forward_gated(layer: Layer, bank: Optional[Bank], proj: Optional[torch.Tensor],
                             bias: Optional[torch.Tensor], h_in: torch.Tensor, h_out: torch.Tensor, tau: float,
                             flags: int, tick: int, workspace: torch.Tensor, out: Optional[GateBuffers] = None,
                             fp_given: Optional[torch.Tensor] = None, inv_norm_given: Optional[torch.Tensor] = None,
                             stream=None, carry: Optional["GateBuffers"] = None,
                             prev_bank: Optional[Bank] = None) -> None:
    """``carry``: the GateBuffers of the call that produced ``h_in`` (its pooled / pooled_valid are taken as the
    token means of the rows it answered from its bank).  ``prev_bank``: that call was made with DEFER_COPY on this
    bank; carry.ref then says which rows of ``h_in`` are references to its value rows."""
    B, S, _ = h_in.shape
    ld = layer.desc()
    fpd = FpDesc(_ptr(proj), _ptr(bias), proj.shape[1] if proj is not None else 0,
                 _ptr(carry.pooled) if carry is not None else None,
                 _ptr(carry.pooled_valid) if carry is not None else None,
                 _ptr(carry.key) if carry is not None else None,
                 _ptr(carry.key_inv) if carry is not None else None,
                 prev_bank.handle if prev_bank is not None else None,
                 _ptr(carry.ref) if (prev_bank is not None and carry is not None) else None)
    go = out.struct() if out is not None else None
    _check(lib().llmc_layer_forward_gated(
        C.byref(ld), bank.handle if bank is not None else None, C.byref(fpd), _ptr(h_in), _ptr(h_out), B, S, tau,
        flags, tick, _ptr(fp_given), _ptr(inv_norm_given), C.byref(go) if go is not None else None,
        _ptr(workspace), workspace.numel(), _stream(stream)))


def llmc_profile_begin(max_records: int) -> None:
    _check(lib().llmc_profile_begin(max_records))


def llmc_profile_report() -> Dict[str, tuple]:
    """{kernel name: (launch count, total milliseconds)} since the last report."""
    buf = C.create_string_buffer(1 << 16)
    lib().llmc_profile_report(buf, len(buf))
    out = {}
    for line in buf.value.decode().splitlines():
        name, cnt, ms = line.split()
        out[name] = (int(cnt), float(ms))
    return out


def llmc_profile_end() -> None:
    _check(lib().llmc_profile_end())


def layer_from_weights(cfg, w: Dict[str, torch.Tensor], device="cuda") -> Layer:
    """Move one layer's weight dict (see workloads.make_layer_weights) to the device."""
    return Layer(cfg.arch, cfg.d, cfg.n_heads, cfg.d_ff, cfg.gelu, cfg.ln_eps, cfg.torch_dtype,
                 {k: v.to(device).contiguous() for k, v in w.items()})
