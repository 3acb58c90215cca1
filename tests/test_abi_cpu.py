"""Host-only checks of the C ABI: the library loads, exports every declared entry point,
and rejects bad arguments before touching the GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2512_16843_amd import llmc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "llmc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(llmc_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(llmc.LIB_PATH):
        from paper_2512_16843_amd.build import build_library
        build_library()
    return llmc.lib()


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(llmc.EXPORTS)
    assert b"gfx950" in lib.llmc_version()


def test_null_and_shape_errors_come_before_any_gpu_call(lib):
    assert lib.llmc_fingerprint(None, 1, 1, 64, 0, None, None, 32, None, None, None, 0, None) == llmc.ERR_INVALID_ARG
    assert b"NULL" in lib.llmc_last_error()
    fake = C.c_void_p(4096)      # never dereferenced: validation fails first
    assert lib.llmc_fingerprint(fake, 1, 1, 64, 7, fake, None, 32, fake, fake, fake, 1 << 20, None) == llmc.ERR_DTYPE
    assert lib.llmc_fingerprint(fake, 1, 1, 65, 0, fake, None, 32, fake, fake, fake, 1 << 20, None) == llmc.ERR_SHAPE
    assert lib.llmc_fingerprint(fake, 1, 1, 64, 0, fake, None, 33, fake, fake, fake, 1 << 20, None) == llmc.ERR_SHAPE
    assert lib.llmc_fingerprint(fake, 0, 1, 64, 0, fake, None, 32, fake, fake, fake, 1 << 20, None) == llmc.ERR_INVALID_ARG
    assert lib.llmc_fingerprint(fake, 1, 1, 64, 0, fake, None, 32, fake, fake, fake, 8, None) == llmc.ERR_WORKSPACE
    misaligned = C.c_void_p(4100)
    assert lib.llmc_fingerprint(misaligned, 1, 1, 64, 0, fake, None, 32, fake, fake, fake, 1 << 20, None) == llmc.ERR_SHAPE
    assert lib.llmc_match(None, fake, fake, 4, 0.5, fake, None, None, None, fake, 1 << 20, None) == llmc.ERR_INVALID_ARG
    assert lib.llmc_bank_insert(None, fake, fake, fake, None, None, 4, 1, fake, None, None) == llmc.ERR_INVALID_ARG
    assert lib.llmc_bank_evict(None, None, 4, fake, None) == llmc.ERR_INVALID_ARG
    assert lib.llmc_gather_hits(None, fake, None, None, 4, fake, None) == llmc.ERR_INVALID_ARG
    assert lib.llmc_bank_destroy(None) == llmc.LLMC_OK


def test_bank_create_validation(lib):
    out = C.c_void_p()
    assert lib.llmc_bank_create(None, C.byref(out)) == llmc.ERR_INVALID_ARG
    p = 4096

    def desc(**kw):
        base = dict(n_slots=16, k=32, S=4, d=64, n_act_slots=16, dtype=llmc.BF16, policy=llmc.EVICT_LRU,
                    d_fp=p, d_act=p, d_inv_norm=p, d_act_slot=None, d_last_used=p, d_hits=p, d_valid=p, half_life=0, reval_every=0, drift_bound=0.0, rank=0, d_basis=None, d_act_pool=None, d_next_proj=None, d_next_bias=None, next_k=0, d_next_fp=None,
                    d_next_inv=None, key_bits=0, d_lsh_index=None, lsh_index_bytes=0)
        base.update(kw)
        return llmc.BankDesc(**base)

    assert lib.llmc_bank_create(C.byref(desc(dtype=9)), C.byref(out)) == llmc.ERR_DTYPE
    assert lib.llmc_bank_create(C.byref(desc(k=48)), C.byref(out)) == llmc.ERR_SHAPE
    assert lib.llmc_bank_create(C.byref(desc(d=100)), C.byref(out)) == llmc.ERR_SHAPE
    assert lib.llmc_bank_create(C.byref(desc(n_slots=0)), C.byref(out)) == llmc.ERR_SHAPE
    assert lib.llmc_bank_create(C.byref(desc(n_act_slots=8)), C.byref(out)) == llmc.ERR_SHAPE      # identity map
    assert lib.llmc_bank_create(C.byref(desc(n_act_slots=32)), C.byref(out)) == llmc.ERR_SHAPE
    assert lib.llmc_bank_create(C.byref(desc(d_valid=None)), C.byref(out)) == llmc.ERR_INVALID_ARG
    assert lib.llmc_bank_create(C.byref(desc(policy=5)), C.byref(out)) == llmc.ERR_INVALID_ARG
    assert lib.llmc_bank_create(C.byref(desc(d_next_proj=p, d_next_fp=p, d_next_inv=p, next_k=32)), C.byref(out)) == llmc.ERR_INVALID_ARG   # no means
    assert lib.llmc_bank_create(C.byref(desc(d_act_pool=p, d_next_proj=p, d_next_fp=p, d_next_inv=p, next_k=40)), C.byref(out)) == llmc.ERR_SHAPE
    assert lib.llmc_bank_create(C.byref(desc(key_bits=2)), C.byref(out)) == llmc.ERR_INVALID_ARG
    # a bucket index: sign-bit keys only, k of 64 / 128 / 256 / 512, 256-byte aligned, large enough
    need = lib.llmc_lsh_index_bytes(16, 64)
    aligned = C.c_void_p(1 << 20)
    assert lib.llmc_bank_create(C.byref(desc(k=64, d_lsh_index=aligned, lsh_index_bytes=need)), C.byref(out)) == llmc.ERR_INVALID_ARG
    assert lib.llmc_bank_create(C.byref(desc(key_bits=1, d_lsh_index=aligned, lsh_index_bytes=1 << 30)), C.byref(out)) == llmc.ERR_SHAPE
    assert lib.llmc_bank_create(C.byref(desc(k=64, key_bits=1, d_lsh_index=C.c_void_p((1 << 20) + 16), lsh_index_bytes=need)),
                                C.byref(out)) == llmc.ERR_SHAPE
    assert lib.llmc_bank_create(C.byref(desc(k=64, key_bits=1, d_lsh_index=aligned, lsh_index_bytes=need - 1)),
                                C.byref(out)) == llmc.ERR_WORKSPACE
    assert lib.llmc_bank_create(C.byref(desc(d_inv_norm=None)), C.byref(out)) == llmc.ERR_INVALID_ARG
    assert lib.llmc_bank_create(C.byref(desc(rank=32, d_basis=p)), C.byref(out)) == llmc.ERR_SHAPE
    assert lib.llmc_bank_create(C.byref(desc(rank=128, d_basis=p)), C.byref(out)) == llmc.ERR_SHAPE            # above d = 64
    assert lib.llmc_bank_create(C.byref(desc(rank=64, d_basis=None)), C.byref(out)) == llmc.ERR_INVALID_ARG
    assert lib.llmc_bank_create(C.byref(desc(rank=64, d_basis=p, policy=llmc.EVICT_NONE)), C.byref(out)) == llmc.ERR_INVALID_ARG
    assert lib.llmc_bank_create(C.byref(desc(policy=llmc.EVICT_DECAYED_HITS, half_life=-1)), C.byref(out)) == llmc.ERR_INVALID_ARG
    assert lib.llmc_bank_create(C.byref(desc(policy=llmc.EVICT_DECAYED_HITS, n_slots=(1 << 24) + 1,
                                             n_act_slots=(1 << 24) + 1)), C.byref(out)) == llmc.ERR_SHAPE
    assert out.value is None


def test_gated_layer_validation(lib):
    p = 4096
    ptrs = {n: p for n in ("d_wqkv", "d_bqkv", "d_wo", "d_bo", "d_w1", "d_b1", "d_w2", "d_b2",
                           "d_ln1_g", "d_ln1_b", "d_ln2_g", "d_ln2_b")}

    def layer(**kw):
        base = dict(arch=0, d=128, n_heads=2, d_ff=512, gelu=0, ln_eps=1e-5, dtype=llmc.F32, **ptrs)
        base.update(kw)
        return llmc.LayerDesc(**base)

    def call(ld, B=2, S=4, tau=0.9, flags=0, tick=1, h_in=p, h_out=2 * p, ws=p, ws_bytes=1 << 30):
        return lib.llmc_layer_forward_gated(C.byref(ld) if ld is not None else None, None, None, h_in, h_out, B, S,
                                            tau, flags, tick, None, None, None, ws, ws_bytes, None)

    assert call(None) == llmc.ERR_INVALID_ARG
    assert call(layer(n_heads=4)) == llmc.ERR_SHAPE              # head size 32
    assert call(layer(dtype=3)) == llmc.ERR_DTYPE
    assert call(layer(arch=2)) == llmc.ERR_INVALID_ARG
    assert call(layer(d_w1=None)) == llmc.ERR_INVALID_ARG
    assert call(layer(), h_out=p) == llmc.ERR_INVALID_ARG        # in-place is refused
    assert call(layer(), tau=float("nan")) == llmc.ERR_INVALID_ARG
    assert call(layer(), flags=128) == llmc.ERR_INVALID_ARG       # unknown flag bit
    assert call(layer(), tick=1 << 40) == llmc.ERR_INVALID_ARG
    assert call(layer(), B=0) == llmc.ERR_INVALID_ARG
    assert call(layer(), ws_bytes=16) == llmc.ERR_WORKSPACE
    ld = layer()
    need = lib.llmc_layer_workspace_bytes(C.byref(ld), 2, 4, 0)
    assert need > 2 * 4 * (3 * 128 + 3 * 128 + 512) * 4


def test_bit_key_entry_points_validate_and_max_hamming_matches_the_oracle(lib):
    from oracle import llmc_oracle as O
    fake = C.c_void_p(4096)
    assert lib.llmc_match_bits(None, fake, 4, 64, fake, 2, 3, fake, None, None, fake, 1 << 20, None) == llmc.ERR_INVALID_ARG
    assert lib.llmc_match_bits(fake, fake, 4, 48, fake, 2, 3, fake, None, None, fake, 1 << 20, None) == llmc.ERR_SHAPE
    assert lib.llmc_match_bits(fake, fake, 4, 2048, fake, 2, 3, fake, None, None, fake, 1 << 20, None) == llmc.ERR_SHAPE
    assert lib.llmc_match_bits(fake, fake, 0, 64, fake, 2, 3, fake, None, None, fake, 1 << 20, None) == llmc.ERR_INVALID_ARG
    assert lib.llmc_match_bits(fake, fake, 4, 64, fake, 2, 3, fake, None, None, fake, 8, None) == llmc.ERR_WORKSPACE
    assert lib.llmc_match_bits_workspace_bytes(4, 48, 2) == 0
    assert lib.llmc_match_bits_workspace_bytes(1 << 20, 256, 4096) >= (1 << 20) * 4
    assert lib.llmc_fingerprint_bits(None, 1, 1, 64, 0, fake, None, 32, fake, fake, 1 << 20, None) == llmc.ERR_INVALID_ARG
    assert lib.llmc_fingerprint_bits(fake, 1, 1, 64, 0, fake, None, 40, fake, fake, 1 << 20, None) == llmc.ERR_SHAPE
    assert lib.llmc_fingerprint_bits(fake, 1, 1, 64, 0, fake, None, 32, fake, fake, 8, None) == llmc.ERR_WORKSPACE
    import numpy as np
    for k in (32, 64, 256, 1024):
        for tau in (-1.0, -0.5, 0.0, 0.3, 0.82, 0.9, 0.95, 0.98, 0.999, 0.99999, 1.0, 2.0):
            assert lib.llmc_max_hamming(tau, k) == O.max_hamming(float(np.float32(tau)), k), (tau, k)
    assert lib.llmc_max_hamming(0.5, 0) == -1


def test_fingerprint_prefix_rejects_bad_arguments(lib):
    fake = C.c_void_p(1 << 20)
    w = {n: fake for n in ("d_wqkv", "d_bqkv", "d_wo", "d_bo", "d_w1", "d_b1", "d_w2", "d_b2", "d_ln1_g", "d_ln1_b",
                           "d_ln2_g", "d_ln2_b")}
    layer = llmc.LayerDesc(arch=0, d=128, n_heads=2, d_ff=512, gelu=0, ln_eps=1e-5, dtype=llmc.BF16, **w)
    need = lib.llmc_fingerprint_prefix_workspace_bytes(C.byref(layer), 4, 32, 8)
    assert need > 4 * 2 * 128 * 4
    assert lib.llmc_fingerprint_prefix_workspace_bytes(C.byref(layer), 4, 32, 33) == 0          # prefix longer than S

    def call(n_prefix=8, k=64, ws=need, h=fake, B=4, S=32):
        return lib.llmc_fingerprint_prefix(C.byref(layer), h, B, S, n_prefix, fake, None, k, fake, fake, fake, ws, None)

    assert call(n_prefix=0) == llmc.ERR_INVALID_ARG
    assert call(n_prefix=33) == llmc.ERR_INVALID_ARG
    assert call(h=None) == llmc.ERR_INVALID_ARG
    assert call(k=40) == llmc.ERR_SHAPE
    assert call(ws=need - 1) == llmc.ERR_WORKSPACE
    assert call(h=C.c_void_p((1 << 20) + 2)) == llmc.ERR_SHAPE
