"""Pins of the oracle's sign-bit keys (SimHash bits, Hamming match) against things other than itself:
hand-made words, Python's own bit counting, closed forms of the projection's sign, the angle law of
random hyperplanes, brute-force loops, and agreement with the cosine match on separated clusters.
"""
import math

import numpy as np
import pytest

from oracle import llmc_oracle as O


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def test_bit_order_is_least_significant_first_word_by_word():
    bits = np.zeros((1, 64), dtype=bool)
    bits[0, [0, 31, 33, 63]] = True
    w = O.pack_bits(bits)
    assert w.dtype == np.uint32 and w.shape == (1, 2)
    assert int(w[0, 0]) == 0x80000001 and int(w[0, 1]) == 0x80000002
    assert np.array_equal(O.unpack_bits(w, 64), bits)
    g = rng(1)
    b = g.random((5, 3, 96)) > 0.5
    assert np.array_equal(O.unpack_bits(O.pack_bits(b), 96), b)


def test_hamming_against_python_bit_count():
    g = rng(2)
    k = 160
    q = g.integers(0, 2 ** 32, size=(7, k // 32), dtype=np.uint64).astype(np.uint32)
    b = g.integers(0, 2 ** 32, size=(11, k // 32), dtype=np.uint64).astype(np.uint32)
    H = O.hamming(q, b, k)
    for i in range(7):
        for j in range(11):
            want = sum(bin(int(q[i, w]) ^ int(b[j, w])).count("1") for w in range(k // 32))
            assert H[i, j] == want
    assert np.all(O.hamming(q, q, k).diagonal() == 0)
    assert np.all(O.hamming(q, ~q, k).diagonal() == k)


def test_sign_bits_closed_forms():
    g = rng(3)
    d = 64
    x = g.standard_normal((4, 1, d))
    x[0, 0, 5] = 0.0                                  # zero counts as non-negative
    P = np.eye(d)
    w = O.fingerprint_bits(x, P, None)
    assert np.array_equal(O.unpack_bits(w, d), x[:, 0, :] >= 0)
    c = g.standard_normal(d)
    assert np.array_equal(O.unpack_bits(O.fingerprint_bits(x, P, c), d), (x[:, 0, :] + c) >= 0)
    # mean over tokens, [d, k] orientation with d != k: explicit loops
    h = g.standard_normal((3, 5, 8))
    P2 = g.standard_normal((8, 32))
    want = np.zeros((3, 32), dtype=bool)
    for b in range(3):
        for j in range(32):
            acc = 0.0
            for i in range(8):
                acc += (sum(h[b, t, i] for t in range(5)) / 5.0) * P2[i, j]
            want[b, j] = acc >= 0
    assert np.array_equal(O.unpack_bits(O.fingerprint_bits(h, P2, None), 32), want)
    # positive scaling leaves the key alone, negation complements it (no exact zeros here)
    assert np.array_equal(O.fingerprint_bits(3.5 * h, P2, None), O.fingerprint_bits(h, P2, None))
    assert np.array_equal(O.fingerprint_bits(-h, P2, None), ~O.fingerprint_bits(h, P2, None))


def test_random_hyperplanes_separate_with_probability_angle_over_pi():
    g = rng(4)
    d, k = 48, 4096
    P = g.standard_normal((d, k))
    a = g.standard_normal(d)
    r = g.standard_normal(d)
    r -= a * (a @ r) / (a @ a)
    a /= np.linalg.norm(a)
    r /= np.linalg.norm(r)
    for theta in (0.1, 0.5, 1.0, 2.0, 3.0):
        b = math.cos(theta) * a + math.sin(theta) * r
        wa = O.fingerprint_bits(a[None, None, :], P, None)
        wb = O.fingerprint_bits(b[None, None, :], P, None)
        H = int(O.hamming(wa, wb, k)[0, 0])
        p = theta / math.pi
        assert abs(H / k - p) < 4.5 * math.sqrt(p * (1 - p) / k) + 1e-9, (theta, H)
        assert abs(O.cosine_estimate(np.array([H]), k)[0] - math.cos(theta)) < 0.08


def test_match_bits_brute_force_ties_holes_and_empty_bank():
    g = rng(5)
    k, N, B = 64, 40, 9
    bank = g.integers(0, 2 ** 32, size=(N, 2), dtype=np.uint64).astype(np.uint32)
    q = g.integers(0, 2 ** 32, size=(B, 2), dtype=np.uint64).astype(np.uint32)
    bank[17] = bank[4]                                 # duplicates: the lower slot must win
    q[0] = bank[17]
    q[1] = bank[30] ^ np.array([1, 0], dtype=np.uint32)   # one bit off slot 30
    valid = (g.random(N) > 0.2).astype(np.uint8)
    valid[[4, 17, 30]] = 1
    idx, dist = O.match_bits(q, bank, valid, k)
    for b in range(B):
        best, bj = None, -1
        for j in range(N):
            if not valid[j]:
                continue
            h = sum(bin(int(q[b, w]) ^ int(bank[j, w])).count("1") for w in range(2))
            if best is None or h < best:
                best, bj = h, j
        assert idx[b] == bj and dist[b] == best
    assert idx[0] == 4 and dist[0] == 0 and idx[1] == 30 and dist[1] == 1
    valid[4] = 0
    assert O.match_bits(q[:1], bank, valid, k)[0][0] == 17
    idx, dist = O.match_bits(q, bank, np.zeros(N, np.uint8), k)
    assert np.all(idx == -1) and np.all(dist == O.NO_MATCH_DIST)


def test_max_hamming_is_the_threshold_on_the_cosine_estimate():
    k = 256
    prev = k
    for tau in (-1.0, -0.3, 0.2, 0.5, 0.9, 0.95, 0.98, 0.999, 0.99999, 1.0, 1.5):
        m = O.max_hamming(tau, k)
        assert m <= prev
        prev = m
        for H in range(0, k + 1):
            assert (math.cos(math.pi * H / k) > tau) == (H <= m)
    assert O.max_hamming(math.cos(math.pi * 10.5 / k), k) == 10
    assert O.max_hamming(1.0, k) == -1 and O.max_hamming(0.99999, k) == 0
    idx = np.array([3, -1, 5, 7])
    dist = np.array([10, 0, 11, 0])
    assert O.threshold_bits(idx, dist, 10).tolist() == [True, False, False, True]
    assert not O.threshold_bits(idx, dist, -1).any()


def test_bit_match_finds_the_cosine_neighbour_on_separated_clusters():
    g = rng(6)
    d, k, n_cl = 96, 512, 24
    centres = g.standard_normal((n_cl, d))
    P = g.standard_normal((d, k)) / math.sqrt(k)
    bank_h = centres[:, None, :]                        # one token per sequence
    queries = centres[g.integers(0, n_cl, size=40)] + 0.15 * g.standard_normal((40, d))
    bits_bank = O.fingerprint_bits(bank_h, P, None)
    bits_q = O.fingerprint_bits(queries[:, None, :], P, None)
    idx_b, dist = O.match_bits(bits_q, bits_bank, np.ones(n_cl, np.uint8), k)
    fb, ib = O.fingerprint(bank_h, P, None, "f32")
    fq, iq = O.fingerprint(queries[:, None, :], P, None, "f32")
    idx_c, sim = O.match(fq, iq, fb, ib, np.ones(n_cl, np.uint8))
    assert np.array_equal(idx_b, idx_c)
    assert np.max(np.abs(O.cosine_estimate(dist, k) - sim)) < 0.15


def test_gated_layer_with_sign_bit_bank():
    """A bank of sign-bit keys in the gate: resubmitted inputs hit at distance 0 and return the stored values,
    tau >= 1 computes everything, inserted keys are the inputs' sign bits."""
    g = rng(8)
    S, d, k, N, B = 4, 32, 64, 10, 6
    w = {"wqkv": g.standard_normal((3 * d, d)) * 0.05, "bqkv": np.zeros(3 * d), "wo": g.standard_normal((d, d)) * 0.05,
         "bo": np.zeros(d), "w1": g.standard_normal((2 * d, d)) * 0.05, "b1": np.zeros(2 * d),
         "w2": g.standard_normal((d, 2 * d)) * 0.05, "b2": np.zeros(d), "ln1_g": np.ones(d), "ln1_b": np.zeros(d),
         "ln2_g": np.ones(d), "ln2_b": np.zeros(d)}
    P = g.standard_normal((d, k)) / np.sqrt(k)
    h = g.standard_normal((B, S, d))
    bank = O.Bank(N, k, S, d, "f32", key_bits=True)
    assert bank.fp.shape == (N, 2) and bank.fp.dtype == np.uint32
    r1 = O.gated_layer(h, bank, P, None, w, O.ENCODER_POST_LN, 2, 1e-5, O.GELU_ERF, 0.95, flags=O.FLAG_INSERT_ON_MISS, tick=1)
    assert not r1.hit.any() and r1.slots == list(range(B))
    assert np.array_equal(bank.fp[:B], O.fingerprint_bits(h, P, None))
    r2 = O.gated_layer(h, bank, P, None, w, O.ENCODER_POST_LN, 2, 1e-5, O.GELU_ERF, 0.95)
    assert r2.hit.all() and np.array_equal(r2.idx, np.arange(B)) and np.allclose(r2.sim, 1.0)
    np.testing.assert_allclose(r2.h_out, r1.h_out, atol=1e-6)
    r3 = O.gated_layer(h, bank, P, None, w, O.ENCODER_POST_LN, 2, 1e-5, O.GELU_ERF, 1.0)
    assert not r3.hit.any()
    np.testing.assert_allclose(r3.h_out, r1.h_out, atol=1e-12)
    # against a bank holding only entry 0, the negated input has every sign flipped: distance k, cosine estimate -1
    bank.valid[1:] = 0
    r4 = O.gated_layer(-h[:1], bank, P, None, w, O.ENCODER_POST_LN, 2, 1e-5, O.GELU_ERF, -0.5)
    assert not r4.hit.any() and r4.idx[0] == 0 and np.allclose(r4.sim, -1.0)


def test_lsh_buckets_candidates_by_explicit_loops_and_agreement_with_the_full_match():
    g = rng(9)
    k, N, B = 64, 300, 20
    bank = g.integers(0, 2 ** 32, size=(N, 2), dtype=np.uint64).astype(np.uint32)
    q = g.integers(0, 2 ** 32, size=(B, 2), dtype=np.uint64).astype(np.uint32)
    valid = (g.random(N) > 0.1).astype(np.uint8)
    for b in range(0, B, 2):                      # near-duplicates: a few flipped bits leave most bands intact
        j = int(g.integers(0, N))
        q[b] = bank[j]
        for _ in range(3):
            i = int(g.integers(0, k))
            q[b, i // 32] ^= np.uint32(1 << (i % 32))
    cand = O.lsh_candidates(q, bank, valid, k)
    bits_q, bits_b = O.unpack_bits(q, k), O.unpack_bits(bank, k)
    for b in range(B):
        for j in range(N):
            share = any(np.array_equal(bits_q[b, 16 * t:16 * t + 16], bits_b[j, 16 * t:16 * t + 16]) for t in range(k // 16))
            assert cand[b, j] == (share and bool(valid[j]))
    idx, dist, n = O.match_bits_lsh(q, bank, valid, k)
    fidx, fdist = O.match_bits(q, bank, valid, k)
    assert np.array_equal(n, cand.sum(axis=1))
    for b in range(B):
        if n[b] == 0:
            assert idx[b] == -1 and dist[b] == O.NO_MATCH_DIST
        else:
            js = np.nonzero(cand[b])[0]
            hs = [int(O.hamming(q[b:b + 1], bank[j:j + 1], k)[0, 0]) for j in js]
            assert dist[b] == min(hs) and idx[b] == js[int(np.argmin(hs))]
        if fidx[b] >= 0 and cand[b, fidx[b]]:     # the true nearest shares a band: the bucketed lookup finds it
            assert idx[b] == fidx[b] and dist[b] == fdist[b]
    near = np.arange(0, B, 2)
    ok = valid[fidx[near]] == 1
    assert np.array_equal(idx[near][fdist[near] <= 3], fidx[near][fdist[near] <= 3])


def test_gate_with_bucketed_lookup_sees_only_entries_that_share_a_band():
    """FLAG_LOOKUP_LSH in the gated layer: the bank is consulted through the band buckets.  Hand-made keys: the query
    differs from entry 0 by ONE bit in EVERY 16-bit band (distance k / 16, well under the threshold's bound, so the
    full comparison hits) and from entry 1 by 40 bits that all sit in the first three bands (the other band is intact).
    The bucketed lookup cannot see entry 0 and answers with entry 1, which is too far: a miss; the full comparison
    answers with entry 0: a hit."""
    g = rng(11)
    S, d, k, N = 4, 32, 64, 6
    w = {"wqkv": g.standard_normal((3 * d, d)) * 0.05, "bqkv": np.zeros(3 * d), "wo": g.standard_normal((d, d)) * 0.05,
         "bo": np.zeros(d), "w1": g.standard_normal((2 * d, d)) * 0.05, "b1": np.zeros(2 * d),
         "w2": g.standard_normal((d, 2 * d)) * 0.05, "b2": np.zeros(d), "ln1_g": np.ones(d), "ln1_b": np.zeros(d),
         "ln2_g": np.ones(d), "ln2_b": np.zeros(d)}
    h = g.standard_normal((1, S, d))
    qbits = g.integers(0, 2, (1, k)).astype(bool)
    e0 = qbits.copy()
    e0[0, [3, 16 + 5, 32 + 9, 48 + 1]] ^= True                      # one bit in each of the four bands
    e1 = qbits.copy()
    e1[0, np.r_[0:16, 16:32, 32:40]] ^= True                        # 40 bits, band 3 untouched
    bank = O.Bank(N, k, S, d, "f32", key_bits=True)
    bank.fp[0], bank.fp[1] = O.pack_bits(e0)[0], O.pack_bits(e1)[0]
    bank.valid[:2] = 1
    bank.act[0], bank.act[1] = 1.0, 2.0
    q = O.pack_bits(qbits)
    tau = np.float32(0.9)
    assert O.max_hamming(tau, k) >= 4 and O.max_hamming(tau, k) < 40
    full = O.gated_layer(h, bank, None, None, w, O.ENCODER_POST_LN, 2, 1e-5, O.GELU_ERF, tau,
                         fp_override=(q, np.zeros(1, np.float32)))
    assert full.hit[0] and full.idx[0] == 0 and np.all(full.h_out[0] == 1.0)
    lsh = O.gated_layer(h, bank, None, None, w, O.ENCODER_POST_LN, 2, 1e-5, O.GELU_ERF, tau,
                        flags=O.FLAG_LOOKUP_LSH, fp_override=(q, np.zeros(1, np.float32)))
    assert not lsh.hit[0] and lsh.idx[0] == 1
    np.testing.assert_allclose(lsh.sim[0], np.cos(np.pi * 40 / k), atol=1e-12)
    np.testing.assert_allclose(lsh.h_out[0], O.layer_forward(h[0], w, O.ENCODER_POST_LN, 2, 1e-5, O.GELU_ERF), atol=0)
    # an entry equal to the query in one band and nowhere else is seen; an invalid one is not
    bank.valid[1] = 0
    none = O.gated_layer(h, bank, None, None, w, O.ENCODER_POST_LN, 2, 1e-5, O.GELU_ERF, tau,
                         flags=O.FLAG_LOOKUP_LSH, fp_override=(q, np.zeros(1, np.float32)))
    assert not none.hit[0] and none.idx[0] == -1 and none.sim[0] == -np.inf
    # the resubmitted key itself shares every band: both lookups agree on it
    bank.fp[2] = q[0]
    bank.valid[2] = 1
    bank.act[2] = 3.0
    same = O.gated_layer(h, bank, None, None, w, O.ENCODER_POST_LN, 2, 1e-5, O.GELU_ERF, tau,
                         flags=O.FLAG_LOOKUP_LSH, fp_override=(q, np.zeros(1, np.float32)))
    assert same.hit[0] and same.idx[0] == 2 and same.sim[0] == 1.0 and np.all(same.h_out[0] == 3.0)
