"""Pins for the oracle's fingerprint, match and threshold steps (CPU only).

The paper prints no worked example, so these pin the oracle to what the
definitions fix: closed forms, brute force on tiny inputs, invariants.
"""
import math

import numpy as np
import pytest

from oracle import llmc_oracle as O


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ---- bf16 rounding ----------------------------------------------------------

def test_round_to_bf16_matches_torch_and_ties_to_even():
    import torch
    x = rng(0).standard_normal(20000).astype(np.float32) * np.float32(3.0)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(O.round_to_bf16(x), want)
    # exact halfway cases: 1 + 2^-8 lies between 1 and 1 + 2^-7 -> even mantissa (1.0)
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == np.float32(1.0)
    # 1 + 3*2^-8 lies between 1+2^-7 (odd) and 1+2^-6 (even) -> 1 + 2^-6
    assert O.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == np.float32(1.0 + 2.0 ** -6)
    assert O.round_to_bf16(np.array([0.0, -0.0, 1.0, -2.5]))[3] == np.float32(-2.5)


# ---- pooling + projection: closed forms (Section IV-B) -----------------------

def test_fingerprint_single_token_is_that_token():
    r = rng(1)
    h = r.standard_normal((3, 1, 16))
    q, qinv = O.fingerprint(h, np.eye(16), None, "f32")
    want = h[:, 0, :] / np.linalg.norm(h[:, 0, :], axis=1, keepdims=True)
    np.testing.assert_allclose(q, want, rtol=0, atol=1e-7)
    np.testing.assert_allclose(qinv, 1.0, atol=1e-6)


def test_fingerprint_identity_projection_is_normalised_mean():
    r = rng(2)
    h = r.standard_normal((4, 7, 12))
    q, _ = O.fingerprint(h, np.eye(12), None, "f32")
    for b in range(4):
        m = np.zeros(12)
        for t in range(7):          # explicit token loop: a dropped or doubled token shows here
            m += h[b, t]
        m /= 7.0
        np.testing.assert_allclose(q[b], m / math.sqrt(float(m @ m)), atol=1e-7)


def test_fingerprint_constant_rows_and_scale_invariance():
    r = rng(3)
    P = r.standard_normal((10, 6))
    row = r.standard_normal(10)
    h = np.broadcast_to(row, (2, 5, 10)).copy()
    q, _ = O.fingerprint(h, P, None, "f32")
    v = row @ P
    np.testing.assert_allclose(q[0], v / np.linalg.norm(v), atol=1e-7)
    h2 = r.standard_normal((3, 9, 10))
    q1, _ = O.fingerprint(h2, P, None, "f32")
    q2, _ = O.fingerprint(4.0 * h2, P, None, "f32")     # power of two: exact in fp
    np.testing.assert_allclose(q1, q2, atol=1e-7)


def test_fingerprint_projection_orientation_and_bias():
    # P is [d, k]: v_j = sum_i p_i P[i, j].  A transposed operand fails (d != k).
    r = rng(4)
    d, k = 5, 3
    h = r.standard_normal((2, 4, d))
    P = r.standard_normal((d, k))
    c = r.standard_normal(k)
    q, _ = O.fingerprint(h, P, c, "f32")
    for b in range(2):
        p = h[b].mean(axis=0)
        v = np.array([sum(p[i] * P[i, j] for i in range(d)) + c[j] for j in range(k)])
        np.testing.assert_allclose(q[b], v / np.linalg.norm(v), atol=1e-7)
    # centring bias c = -P^T mu removes the common component mu exactly
    mu = r.standard_normal(d)
    q_c, _ = O.fingerprint(h, P, -(mu @ P), "f32")
    q_s, _ = O.fingerprint(h - mu, P, None, "f32")
    np.testing.assert_allclose(q_c, q_s, atol=1e-6)


def test_fingerprint_zero_vector_and_bf16_inverse_norm_of_rounded_key():
    h = np.zeros((1, 3, 8))
    q, qinv = O.fingerprint(h, np.eye(8), None, "bf16")
    assert np.all(q == 0) and qinv[0] == 0
    r = rng(5)
    h = r.standard_normal((6, 5, 32))
    P = r.standard_normal((32, 16))
    q, qinv = O.fingerprint(h, P, None, "bf16")
    # keys are bf16-representable, and qinv is the norm of the rounded key, not of the exact one
    assert np.array_equal(q, O.round_to_bf16(q))
    for b in range(6):
        n = math.sqrt(sum(float(x) ** 2 for x in q[b]))
        assert abs(float(qinv[b]) - 1.0 / n) < 1e-7
        assert abs(n - 1.0) < 2.0 ** -8


# ---- match: brute force, permutation, self-hit (Section III-C) ---------------

def brute_force_match(q, qinv, bank, binv, valid):
    B, k = q.shape
    idx = np.full(B, -1, dtype=np.int32)
    sim = np.full(B, -np.inf)
    for b in range(B):
        for j in range(bank.shape[0]):
            if not valid[j]:
                continue
            dot = 0.0
            for t in range(k):
                dot += float(q[b, t]) * float(bank[j, t])
            s = dot * float(qinv[b]) * float(binv[j])
            if s > sim[b]:
                sim[b], idx[b] = s, j
    return idx, sim


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_match_equals_brute_force(seed):
    r = rng(10 + seed)
    N, B, k = 48, 9, 8
    bank = O.round_to_bf16(r.standard_normal((N, k)))
    q = O.round_to_bf16(r.standard_normal((B, k)))
    valid = (r.random(N) > 0.2).astype(np.uint8)
    binv, qinv = O.inv_norm(bank), O.inv_norm(q)
    idx, sim = O.match(q, qinv, bank, binv, valid)
    bidx, bsim = brute_force_match(q, qinv, bank, binv, valid)
    assert np.array_equal(idx, bidx)
    np.testing.assert_allclose(sim, bsim, rtol=0, atol=1e-12)
    assert np.all(valid[idx] == 1)


def test_match_uses_bank_norms_before_argmax():
    # entry 0 has the larger dot product, entry 1 the larger cosine
    bank = np.array([[3.0, 3.0], [1.0, 0.0]], dtype=np.float32)
    q = np.array([[1.0, 0.0]], dtype=np.float32)
    idx, sim = O.match(q, O.inv_norm(q), bank, O.inv_norm(bank), np.ones(2, np.uint8))
    assert idx[0] == 1 and abs(sim[0] - 1.0) < 1e-7


def test_match_permutation_ties_self_and_empty():
    r = rng(20)
    N, B, k = 40, 6, 16
    bank = O.round_to_bf16(r.standard_normal((N, k)))
    q = O.round_to_bf16(r.standard_normal((B, k)))
    valid = np.ones(N, np.uint8)
    binv, qinv = O.inv_norm(bank), O.inv_norm(q)
    idx, sim = O.match(q, qinv, bank, binv, valid)
    perm = r.permutation(N)
    idx_p, sim_p = O.match(q, qinv, bank[perm], binv[perm], valid)
    assert np.array_equal(perm[idx_p], idx)
    np.testing.assert_allclose(sim_p, sim, atol=1e-15)
    # scale invariance of the cosine: scaling a key (and its stored inverse norm) changes nothing
    bank2 = bank.copy()
    bank2[3] *= 2.0
    idx2, sim2 = O.match(q, qinv, bank2, O.inv_norm(bank2), valid)
    assert np.array_equal(idx2, idx)
    np.testing.assert_allclose(sim2, sim, atol=1e-7)
    # duplicates: lowest slot wins
    bank3 = bank.copy()
    bank3[17] = bank3[5]
    bank3[30] = bank3[5]
    qq = bank3[[30]]
    i3, s3 = O.match(qq, O.inv_norm(qq), bank3, O.inv_norm(bank3), valid)
    assert i3[0] == 5 and abs(s3[0] - 1.0) < 1e-6
    # the query itself in the bank: similarity 1
    i4, s4 = O.match(bank[[11]], binv[[11]], bank, binv, valid)
    assert i4[0] == 11 and abs(s4[0] - 1.0) < 1e-6
    # invalid slots are never returned; empty bank -> -1, -inf
    v = valid.copy()
    v[11] = 0
    i5, _ = O.match(bank[[11]], binv[[11]], bank, binv, v)
    assert i5[0] != 11
    i6, s6 = O.match(q, qinv, bank, binv, np.zeros(N, np.uint8))
    assert np.all(i6 == -1) and np.all(np.isneginf(s6))


# ---- threshold (Section IV-A) -------------------------------------------------

def test_threshold_strict_and_monotone():
    sim = np.array([0.5, 0.95, 0.9500001, 1.0, -np.inf])
    assert O.threshold(sim, 0.95).tolist() == [False, False, True, True, False]
    assert not O.threshold(sim, 1.0 + 1e-3).any()
    assert O.threshold(sim[:4], -2.0).all()
    prev = None
    for tau in [0.0, 0.5, 0.9, 0.95, 0.99, 1.0]:
        h = set(np.nonzero(O.threshold(sim, tau))[0].tolist())
        if prev is not None:
            assert h <= prev
        prev = h


# ---- near-tie sets: the slots a parity test may accept besides the oracle's own index ---------

def plane_keys(cosines):
    """Unit keys (cos t, sin t, 0, 0) in fp64, so that the similarity to the query (1, 0, 0, 0) is cos t."""
    c = np.asarray(cosines, dtype=np.float64)
    return np.stack([c, np.sqrt(1.0 - c * c), np.zeros_like(c), np.zeros_like(c)], axis=1)


def test_near_tie_sets_on_a_hand_made_bank():
    # slot:      0 best      1 best - 1e-6   2 invalid, above all   3 best - 1e-5   4 far      5 = slot 0 again
    cosines = [0.9,          0.9 - 1e-6,     0.99,                  0.9 - 1e-5,     0.1,       0.9]
    bank = plane_keys(cosines)
    valid = np.array([1, 1, 0, 1, 1, 1], np.uint8)
    q = np.array([[1.0, 0.0, 0.0, 0.0]])
    one = np.ones(1, np.float32)
    binv = np.ones(6, np.float32)
    # default gap 2e-6: the two slots 1e-6 apart and the exact duplicate, not the one 1e-5 below, never the invalid one
    assert O.near_tie_sets(q, one, bank, binv, valid)[0].tolist() == [0, 1, 5]
    # a wider gap takes the slot 1e-5 below in; the best is still defined by VALID slots only
    assert O.near_tie_sets(q, one, bank, binv, valid, gap=2e-5)[0].tolist() == [0, 1, 3, 5]
    # gap 0 keeps exact ties only (the boundary is inclusive)
    assert O.near_tie_sets(q, one, bank, binv, valid, gap=0.0)[0].tolist() == [0, 5]
    # just below / just above a distance: 1e-6 apart is outside a gap of 0.9e-6 and inside one of 1.1e-6
    assert O.near_tie_sets(q, one, bank, binv, valid, gap=0.9e-6)[0].tolist() == [0, 5]
    assert O.near_tie_sets(q, one, bank, binv, valid, gap=1.1e-6)[0].tolist() == [0, 1, 5]
    # with slot 2 valid it is the best and stands alone
    valid2 = np.ones(6, np.uint8)
    assert O.near_tie_sets(q, one, bank, binv, valid2)[0].tolist() == [2]
    # the oracle's own match index is always a member, and is the lowest member on exact ties
    idx, _ = O.match(q, one, bank, binv, valid)
    assert idx[0] == 0


@pytest.mark.parametrize("seed", [0, 1])
def test_near_tie_sets_equal_brute_force(seed):
    r = rng(40 + seed)
    N, B, k = 60, 7, 8
    bank = O.round_to_bf16(r.standard_normal((N, k)))
    bank[20] = bank[3]                           # an exact duplicate
    q = O.round_to_bf16(bank[[3, 11, 40]] + 1e-3 * r.standard_normal((3, k)))
    q = np.concatenate([q, O.round_to_bf16(r.standard_normal((B - 3, k)))])
    valid = (r.random(N) > 0.15).astype(np.uint8)
    valid[[3, 20]] = 1
    binv, qinv = O.inv_norm(bank), O.inv_norm(q)
    for gap in (2e-6, 1e-2, 0.3):
        sets = O.near_tie_sets(q, qinv, bank, binv, valid, gap=gap)
        for b in range(B):
            sims = {}
            for j in range(N):
                if valid[j]:
                    dot = math.fsum(float(q[b, t]) * float(bank[j, t]) for t in range(k))
                    sims[j] = dot * float(qinv[b]) * float(binv[j])
            best = max(sims.values())
            want = sorted(j for j, s in sims.items() if s >= best - gap)
            # rows whose distance to the boundary is below the rounding noise of the two summation orders are not
            # decidable this way; none occur with these seeds
            assert all(abs((best - s) - gap) > 1e-12 for s in sims.values())
            assert sets[b].tolist() == want, (gap, b)
    assert len(O.near_tie_sets(q, qinv, bank, binv, valid, gap=0.3)[0]) >= 2      # slot 3 and its duplicate at least
    assert any(len(s_) > 2 for s_ in O.near_tie_sets(q, qinv, bank, binv, valid, gap=0.3))


# ---- fingerprint with prefix attention statistics (Section IV-B, second feature) ---------------------------

def _toy_block(g, d, scale=0.3):
    return {"wqkv": g.standard_normal((3 * d, d)) * scale, "bqkv": g.standard_normal(3 * d) * 0.1,
            "wo": g.standard_normal((d, d)) * scale, "bo": g.standard_normal(d) * 0.1,
            "w1": g.standard_normal((2 * d, d)) * scale, "b1": np.zeros(2 * d),
            "w2": g.standard_normal((d, 2 * d)) * scale, "b2": np.zeros(d),
            "ln1_g": 1.0 + 0.1 * g.standard_normal(d), "ln1_b": 0.1 * g.standard_normal(d),
            "ln2_g": np.ones(d), "ln2_b": np.zeros(d)}


@pytest.mark.parametrize("arch", [O.ENCODER_POST_LN, O.DECODER_PRE_LN])
def test_prefix_attention_mean_against_the_library_attention(arch):
    """The prefix feature against torch.nn.functional.multi_head_attention_forward (float64) run on the prefix
    tokens alone, and -- for the causal block -- against the first rows of the attention over the WHOLE sequence,
    which a causal mask makes independent of the later tokens."""
    import torch
    import torch.nn.functional as F
    g = rng(21)
    B, S, d, H, n_p, eps = 3, 12, 16, 2, 5, 1e-5
    w = _toy_block(g, d)
    h = g.standard_normal((B, S, d))
    got = O.prefix_attention_mean(h, w, arch, H, eps, n_p)
    t = {k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in w.items()}
    for b in range(B):
        x = torch.from_numpy(h[b, :n_p])
        mask = None
        if arch == O.DECODER_PRE_LN:
            x = F.layer_norm(x, (d,), t["ln1_g"], t["ln1_b"], eps)
            mask = torch.triu(torch.full((n_p, n_p), float("-inf"), dtype=torch.float64), diagonal=1)
        out, _ = F.multi_head_attention_forward(x.unsqueeze(1), x.unsqueeze(1), x.unsqueeze(1), d, H, t["wqkv"], t["bqkv"],
                                                None, None, False, 0.0, t["wo"], t["bo"], training=False,
                                                need_weights=False, attn_mask=mask)
        np.testing.assert_allclose(got[b], out.squeeze(1).mean(dim=0).numpy(), rtol=0, atol=1e-12)
    if arch == O.DECODER_PRE_LN:
        for b in range(B):
            xl = O.layer_norm(h[b], w["ln1_g"], w["ln1_b"], eps)
            full = O.attention(xl, w["wqkv"], w["bqkv"], w["wo"], w["bo"], H, causal=True)
            np.testing.assert_allclose(got[b], full[:n_p].mean(axis=0), rtol=0, atol=1e-12)
        # ... and so tokens after the prefix do not move the feature at all
        h2 = h.copy()
        h2[:, n_p:] = g.standard_normal((B, S - n_p, d))
        assert np.array_equal(O.prefix_attention_mean(h2, w, arch, H, eps, n_p), got)
    else:
        # the bidirectional block: with the whole sequence as prefix the feature is the mean of the block's attention
        full = O.attention(h[0], w["wqkv"], w["bqkv"], w["wo"], w["bo"], H, causal=False)
        np.testing.assert_allclose(O.prefix_attention_mean(h[:1], w, arch, H, eps, S)[0], full.mean(axis=0), atol=1e-12)


def test_fingerprint_prefix_reduces_to_the_plain_fingerprint_and_to_a_hand_computation():
    g = rng(22)
    B, S, d, k, H, n_p = 4, 9, 16, 32, 2, 4
    w = _toy_block(g, d)
    h = g.standard_normal((B, S, d))
    P = g.standard_normal((d, k)) / np.sqrt(k)
    Pa = g.standard_normal((d, k)) / np.sqrt(k)
    c = g.standard_normal(k) * 0.05
    # a zero map for the attention feature: the plain fingerprint, bit for bit
    q0, i0 = O.fingerprint_prefix(h, np.concatenate([P, np.zeros((d, k))]), c, "f32", w, O.ENCODER_POST_LN, H, 1e-5, n_p)
    q1, i1 = O.fingerprint(h, P, c, "f32")
    assert np.array_equal(q0, q1) and np.array_equal(i0, i1)
    # both features: written out by hand
    a = O.prefix_attention_mean(h, w, O.ENCODER_POST_LN, H, 1e-5, n_p)
    v = h.mean(axis=1) @ P + a @ Pa + c
    u = v / np.linalg.norm(v, axis=1, keepdims=True)
    q2, i2 = O.fingerprint_prefix(h, np.concatenate([P, Pa]), c, "f32", w, O.ENCODER_POST_LN, H, 1e-5, n_p)
    np.testing.assert_allclose(q2, u.astype(np.float32), rtol=0, atol=1e-7)
    np.testing.assert_allclose(i2, 1.0 / np.linalg.norm(q2.astype(np.float64), axis=1), rtol=1e-6)
    # a dropped or swapped feature would show: the key moves when only the attention map changes
    q3, _ = O.fingerprint_prefix(h, np.concatenate([P, -Pa]), c, "f32", w, O.ENCODER_POST_LN, H, 1e-5, n_p)
    assert np.abs(q3 - q2).max() > 1e-3
    # bf16 storage: the rounded key of the same vector
    q4, _ = O.fingerprint_prefix(h, np.concatenate([P, Pa]), c, "bf16", w, O.ENCODER_POST_LN, H, 1e-5, n_p)
    assert np.array_equal(q4, O.round_to_bf16(u))


def test_prefix_feature_is_shared_by_inputs_with_a_common_prefix():
    """What the feature is for: two inputs of a causal model that share their first tokens have the same prefix
    attention mean whatever follows, while their token averages differ; the key with the attention feature is
    therefore closer for them than the key without it when the maps weigh the two features alike."""
    g = rng(23)
    S, d, k, H, n_p = 16, 16, 64, 2, 6
    w = _toy_block(g, d)
    a_in = g.standard_normal((1, S, d))
    b_in = a_in.copy()
    b_in[:, n_p:] = g.standard_normal((1, S - n_p, d))
    fa = O.prefix_attention_mean(a_in, w, O.DECODER_PRE_LN, H, 1e-5, n_p)
    fb = O.prefix_attention_mean(b_in, w, O.DECODER_PRE_LN, H, 1e-5, n_p)
    assert np.array_equal(fa, fb)
    P = g.standard_normal((d, k)) / np.sqrt(k)
    Pa = 4.0 * g.standard_normal((d, k)) / np.sqrt(k)
    def cos(x, y):
        return float((x.astype(np.float64) @ y.astype(np.float64).T)[0, 0] / np.linalg.norm(x) / np.linalg.norm(y))
    plain = cos(O.fingerprint(a_in, P, None, "f32")[0], O.fingerprint(b_in, P, None, "f32")[0])
    both = cos(O.fingerprint_prefix(a_in, np.concatenate([P, Pa]), None, "f32", w, O.DECODER_PRE_LN, H, 1e-5, n_p)[0],
               O.fingerprint_prefix(b_in, np.concatenate([P, Pa]), None, "f32", w, O.DECODER_PRE_LN, H, 1e-5, n_p)[0])
    assert both > plain
