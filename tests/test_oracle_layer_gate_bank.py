"""Pins for the oracle's transformer blocks, gated layer and bank (CPU only)."""
import math
from collections import OrderedDict

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import llmc_oracle as O
from paper_2512_16843_amd import workloads as W


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def np_weights(w):
    return {k: v.float().numpy() for k, v in w.items()}


# ---- f_l against library routines in float64 ---------------------------------

def torch_block(x, w, arch, n_heads, eps, gelu_kind):
    """The same block assembled from torch.nn.functional primitives (float64)."""
    t = {k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in w.items()}
    x = torch.from_numpy(np.asarray(x, dtype=np.float64))
    S, d = x.shape
    approx = "none" if gelu_kind == O.GELU_ERF else "tanh"

    def mha(inp, causal):
        mask = None
        if causal:
            mask = torch.triu(torch.full((S, S), float("-inf"), dtype=torch.float64), diagonal=1)
        out, _ = F.multi_head_attention_forward(
            inp.unsqueeze(1), inp.unsqueeze(1), inp.unsqueeze(1), d, n_heads,
            t["wqkv"], t["bqkv"], None, None, False, 0.0, t["wo"], t["bo"],
            training=False, need_weights=False, attn_mask=mask)
        return out.squeeze(1)

    if arch == O.ENCODER_POST_LN:
        x1 = F.layer_norm(x + mha(x, False), (d,), t["ln1_g"], t["ln1_b"], eps)
        ff = F.linear(F.gelu(F.linear(x1, t["w1"], t["b1"]), approximate=approx), t["w2"], t["b2"])
        return F.layer_norm(x1 + ff, (d,), t["ln2_g"], t["ln2_b"], eps).numpy()
    x1 = x + mha(F.layer_norm(x, (d,), t["ln1_g"], t["ln1_b"], eps), True)
    ff = F.linear(F.gelu(F.linear(F.layer_norm(x1, (d,), t["ln2_g"], t["ln2_b"], eps), t["w1"], t["b1"]),
                         approximate=approx), t["w2"], t["b2"])
    return (x1 + ff).numpy()


@pytest.mark.parametrize("arch,gelu_kind,eps", [(O.ENCODER_POST_LN, O.GELU_ERF, 1e-12),
                                                (O.DECODER_PRE_LN, O.GELU_TANH, 1e-5),
                                                (O.ENCODER_POST_LN, O.GELU_TANH, 1e-5)])
def test_layer_matches_torch_functional(arch, gelu_kind, eps):
    cfg = W.scaled(W.TINY_ENCODER, d=48, n_heads=3, d_ff=80, S=11, n_layers=1)
    w = np_weights(W.make_layer_weights(cfg, seed=3)[0])
    # larger weights so that softmax and GELU are exercised away from their linear regime
    for k in ("wqkv", "wo", "w1", "w2"):
        w[k] = w[k] * 12.0
    x = rng(1).standard_normal((cfg.S, cfg.d))
    got = O.layer_forward(x, w, arch, cfg.n_heads, eps, gelu_kind)
    want = torch_block(x, w, arch, cfg.n_heads, eps, gelu_kind)
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-10)


def test_gelu_layernorm_softmax_basics():
    xs = np.array([-3.0, -1.0, 0.0, 0.5, 2.0])
    for x, g in zip(xs, O.gelu(xs, O.GELU_ERF)):
        assert abs(g - 0.5 * x * (1.0 + math.erf(x / math.sqrt(2.0)))) < 1e-15
    assert O.gelu(np.array([0.0]), O.GELU_TANH)[0] == 0.0
    assert abs(O.gelu(np.array([10.0]), O.GELU_TANH)[0] - 10.0) < 1e-12
    # the tanh form differs from the erf form (by < 1e-3) -- they must not be confused
    dlt = np.abs(O.gelu(xs, O.GELU_TANH) - O.gelu(xs, O.GELU_ERF))
    assert 1e-5 < dlt.max() < 1e-3
    x = rng(0).standard_normal((5, 64)) * 3 + 1
    y = O.layer_norm(x, np.ones(64), np.zeros(64), 1e-12)
    np.testing.assert_allclose(y.mean(axis=1), 0, atol=1e-12)
    np.testing.assert_allclose(y.var(axis=1), 1, atol=1e-9)


def test_decoder_is_causal_and_encoder_is_not():
    cfg = W.scaled(W.TINY_ENCODER, d=32, n_heads=2, d_ff=64, S=10, n_layers=1)
    w = np_weights(W.make_layer_weights(cfg, seed=5)[0])
    for k in ("wqkv", "wo"):
        w[k] = w[k] * 10.0
    x = rng(2).standard_normal((cfg.S, cfg.d))
    x2 = x.copy()
    x2[6:] = rng(3).standard_normal((4, cfg.d))
    yd = O.decoder_layer_pre_ln(x, w, 2, 1e-5)
    yd2 = O.decoder_layer_pre_ln(x2, w, 2, 1e-5)
    np.testing.assert_allclose(yd[:6], yd2[:6], atol=1e-13)
    assert np.abs(yd[6:] - yd2[6:]).max() > 1e-3
    ye = O.encoder_layer_post_ln(x, w, 2, 1e-12)
    ye2 = O.encoder_layer_post_ln(x2, w, 2, 1e-12)
    assert np.abs(ye[:6] - ye2[:6]).max() > 1e-6


# ---- bank: LRU against a list-based simulation (Section IV-D) ----------------

class ListLRU:
    """Textbook LRU over a fixed number of slots: free slots first (lowest index),
    then the least recently used entry; ties in recency broken by slot."""

    def __init__(self, n):
        self.n = n
        self.entries = {}        # slot -> (last_used, payload)

    def take(self):
        for j in range(self.n):
            if j not in self.entries:
                return j
        return min(self.entries, key=lambda j: (self.entries[j][0], j))


def test_lru_scripted_trace():
    bank = O.Bank(4, 2, 1, 1, "f32")
    sim = ListLRU(4)
    r = rng(7)
    payload = 0
    for tick in range(1, 40):
        # a few hits on random valid entries, then 1-3 insertions, all at this tick
        live = [j for j in range(4) if bank.valid[j]]
        hit_slots = [int(r.choice(live)) for _ in range(int(r.integers(0, 3)))] if live else []
        bank.touch(hit_slots, tick)
        for j in hit_slots:
            sim.entries[j] = (tick, sim.entries[j][1])
        m = int(r.integers(1, 4))
        # batch semantics: the m slots are chosen on the pre-insert state
        want = []
        snapshot = dict(sim.entries)
        for i in range(m):
            j = sim.take()
            want.append(j)
            sim.entries[j] = (math.inf, None)      # reserved: not chosen twice in a batch
        sim.entries = snapshot
        q = np.full((m, 2), 1.0, dtype=np.float32)
        acts = np.arange(payload, payload + m, dtype=np.float32).reshape(m, 1, 1)
        got, _ = bank.insert(q, O.inv_norm(q), acts, tick)
        assert got == want
        assert len(set(got)) == m
        for i, j in enumerate(want):
            sim.entries[j] = (tick, payload + i)
        payload += m
        for j, (lu, p) in sim.entries.items():
            assert int(bank.last_used[j]) == lu and bank.act[j, 0, 0] == p and bank.valid[j]
        assert bank.valid.sum() <= 4


def test_lru_victims_are_m_smallest_and_evict_invalidates():
    bank = O.Bank(6, 2, 1, 1, "f32")
    q = np.ones((6, 2), np.float32)
    bank.insert(q, O.inv_norm(q), np.zeros((6, 1, 1), np.float32), tick=1)
    bank.touch([0, 3], 5)
    bank.touch([4], 3)
    assert bank.lru_victims(3) == [1, 2, 5]
    assert bank.lru_victims(5) == [1, 2, 5, 4, 0]
    assert bank.evict(2) == [1, 2]
    assert bank.valid.tolist() == [1, 0, 0, 1, 1, 1]
    assert bank.select_slots(3) == [1, 2, 5]       # free slots first, then oldest
    assert int(bank.hits[0]) == 1 and int(bank.hits[4]) == 1
    full = O.Bank(2, 2, 1, 1, "f32", lru=False)
    full.insert(q[:2], O.inv_norm(q[:2]), np.zeros((2, 1, 1), np.float32), 1)
    with pytest.raises(RuntimeError):
        full.insert(q[:1], O.inv_norm(q[:1]), np.zeros((1, 1, 1), np.float32), 2)


def test_decayed_hits_policy_against_an_event_log_simulation():
    """Staleness-aware replacement: an entry's standing is the number of its hits, each hit weighing 1/2 per
    epoch gone by (floored at every epoch boundary).  The check keeps, per entry, the raw LOG of hit ticks and
    recomputes the standing from the log at the moment of each choice, instead of keeping running counters."""
    half_life = 5
    N = 6
    bank = O.Bank(N, 2, 1, 1, "f32", decayed_hits=True, half_life=half_life)
    r = rng(11)
    log = {}                                   # slot -> dict(ins=tick, hits=[ticks])

    def standing(slot, now):
        e_now = now // half_life
        # replay: a counter that gains 1 per hit and is halved (floor) at every epoch boundary since insertion
        c, e = 0, log[slot]["ins"] // half_life
        events = sorted(log[slot]["hits"])
        for t in events + [None]:
            target = e_now if t is None else t // half_life
            while e < target:
                c //= 2
                e += 1
            if t is not None:
                c += 1
        last = max([log[slot]["ins"]] + events)
        return (min(c, 65535), last, slot)

    payload = 0
    for tick in range(1, 60):
        live = sorted(log)
        hit_slots = [int(r.choice(live)) for _ in range(int(r.integers(0, 4)))] if live else []
        bank.touch(hit_slots, tick)
        for j in hit_slots:
            log[j]["hits"].append(tick)
        if tick % 3 == 0:
            m = int(r.integers(1, 3))
            free = [j for j in range(N) if j not in log]
            order = free + sorted(log, key=lambda j: standing(j, tick))
            want = order[:m]
            q = np.ones((m, 2), np.float32)
            got, n_ev = bank.insert(q, O.inv_norm(q), np.full((m, 1, 1), payload, np.float32), tick)
            assert got == want, (tick, got, want)
            assert n_ev == sum(1 for j in want if j in log)
            for j in want:
                log[j] = dict(ins=tick, hits=[])
            payload += 1
        for j in log:
            assert int(bank.hits[j]) == standing(j, tick)[0]
    # with half_life 0 the counts never decay: plain least-frequently-used
    lfu = O.Bank(3, 2, 1, 1, "f32", decayed_hits=True, half_life=0)
    q = np.ones((3, 2), np.float32)
    lfu.insert(q, O.inv_norm(q), np.zeros((3, 1, 1), np.float32), 1)
    lfu.touch([0, 0, 2], 1000)
    assert lfu.lru_victims(3) == [1, 2, 0] and int(lfu.hits[0]) == 2


# ---- gated layer invariants (Section IV-A, Algorithm 1) ----------------------

def tiny_setup(arch=O.ENCODER_POST_LN, n_src=12, dtype="f32"):
    cfg = W.scaled(W.TINY_ENCODER, d=32, n_heads=2, d_ff=64, S=6, n_layers=2, B=5, n_bank=16, k=8,
                   vocab=50, arch=arch, gelu=O.GELU_ERF if arch == 0 else O.GELU_TANH,
                   ln_eps=1e-12 if arch == 0 else 1e-5)
    ws = [np_weights(w) for w in W.make_layer_weights(cfg, seed=0)]
    tok, pos = W.make_embeddings(cfg, seed=0)
    Ps = [p.float().numpy() for p in W.make_projection(cfg.d, cfg.k, torch.float32, seed=3, n_layers=2)]
    src = W.make_sources(cfg, n_src, seed=1)
    h_src = W.embed(torch.from_numpy(src), tok, pos, torch.float32).numpy()
    return cfg, ws, tok, pos, Ps, src, h_src


def build_banks(cfg, ws, Ps, h_src, dtype="f32"):
    banks = [O.Bank(cfg.n_bank, cfg.k, cfg.S, cfg.d, dtype) for _ in range(cfg.n_layers)]
    h, res = O.infer(h_src, banks, Ps, [None] * cfg.n_layers, ws, cfg.arch, cfg.n_heads, cfg.ln_eps,
                     cfg.gelu, tau=2.0, flags=O.FLAG_INSERT_ON_MISS, tick=1)
    return banks, h, res


@pytest.mark.parametrize("arch", [O.ENCODER_POST_LN, O.DECODER_PRE_LN])
def test_tau_above_one_is_plain_forward(arch):
    cfg, ws, tok, pos, Ps, src, h_src = tiny_setup(arch)
    banks, _, _ = build_banks(cfg, ws, Ps, h_src)
    ids, _ = W.make_substitution_queries(cfg, src, n_dup=3, n_subst=1, seed=2)
    h0 = W.embed(torch.from_numpy(ids), tok, pos, torch.float32).numpy()
    out, res = O.infer(h0, banks, Ps, [None, None], ws, cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu,
                       tau=1.0 + 1e-3)
    assert all(not r.hit.any() for r in res)
    plain = h0.astype(np.float64)
    for w in ws:
        plain = np.stack([O.layer_forward(plain[b], w, cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu)
                          for b in range(cfg.B)])
    assert np.array_equal(out, plain)


def test_resubmitted_sources_hit_at_similarity_one_with_stored_values():
    cfg, ws, tok, pos, Ps, src, h_src = tiny_setup()
    banks, h_built, res_b = build_banks(cfg, ws, Ps, h_src)
    # insertion took free slots in ascending order, one per source row
    assert res_b[0].slots == list(range(len(src))) and res_b[0].n_evicted == 0
    out, res = O.infer(h_src[:5], banks, Ps, [None, None], ws, cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu,
                       tau=0.95)
    for l, r in enumerate(res):
        assert r.hit.all()
        assert r.idx.tolist() == [0, 1, 2, 3, 4]
        np.testing.assert_allclose(r.sim, 1.0, atol=1e-6)
        assert np.array_equal(r.h_out, banks[l].act[:5].astype(np.float64))
    assert np.array_equal(out, banks[-1].act[:5].astype(np.float64))


def test_gate_mixes_hits_and_misses_and_updates_lru():
    cfg, ws, tok, pos, Ps, src, h_src = tiny_setup()
    banks, _, _ = build_banks(cfg, ws, Ps, h_src)
    ids, srcmap = W.make_dial_queries(cfg, src, rho=0.6, seed=4)
    h0 = W.embed(torch.from_numpy(ids), tok, pos, torch.float32).numpy()
    bank = banks[0]
    r = O.gated_layer(h0, bank, Ps[0], None, ws[0], cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu, tau=0.999,
                      flags=O.FLAG_INSERT_ON_MISS | O.FLAG_UPDATE_LRU, tick=9)
    for b in range(cfg.B):
        if srcmap[b] >= 0:
            assert r.hit[b] and r.idx[b] == srcmap[b]
            assert np.array_equal(r.h_out[b], bank.act[srcmap[b]].astype(np.float64))
            assert int(bank.last_used[srcmap[b]]) == 9
        else:
            assert not r.hit[b]
            np.testing.assert_array_equal(
                r.h_out[b], O.layer_forward(h0[b], ws[0], cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu))
    n_miss = int((~r.hit).sum())
    assert r.slots == list(range(len(src), len(src) + n_miss))
    # hit set shrinks as tau grows
    prev = None
    for tau in (0.0, 0.5, 0.9, 0.999, 1.001):
        rr = O.gated_layer(h0, bank, Ps[0], None, ws[0], cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu, tau)
        s = set(np.nonzero(rr.hit)[0].tolist())
        assert prev is None or s <= prev
        prev = s
    # an uncached layer is the plain forward
    r0 = O.gated_layer(h0, None, None, None, ws[0], cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu, tau=0.0)
    np.testing.assert_array_equal(
        r0.h_out[0], O.layer_forward(h0[0], ws[0], cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu))


def test_divergence_monitor_recomputes_sampled_hits_and_refreshes_drifted_entries():
    cfg, ws, tok, pos, Ps, src, h_src = tiny_setup()
    banks, _, _ = build_banks(cfg, ws, Ps, h_src)
    bank = banks[0]
    h = h_src[:cfg.B]                               # resubmitted sources: every row hits at similarity 1
    plain = np.stack([O.layer_forward(h[b].astype(np.float64), ws[0], cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu)
                      for b in range(cfg.B)])
    before = bank.act.copy()
    # no drift: sampled rows (tick + b) % 2 == 0 are recomputed, equal to the cache, nothing is replaced
    r = O.gated_layer(h, bank, Ps[0], None, ws[0], cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu, 0.95,
                      flags=O.FLAG_REVALIDATE, tick=3, reval_every=2, drift_bound=1e-5)
    assert r.hit.all() and r.revalidated == [b for b in range(cfg.B) if (3 + b) % 2 == 0]
    assert max(r.divergence) < 1e-6 and r.refreshed == [] and np.array_equal(bank.act, before)   # fp32 storage
    np.testing.assert_allclose(r.h_out, plain, atol=1e-12)
    # drift two cached values by hand: one sampled (replaced by the fresh output), one not sampled (left alone)
    s_sampled, s_other = int(r.idx[1]), int(r.idx[2])
    bank.act[s_sampled] += 0.5
    bank.act[s_other] += 0.5
    drifted = bank.act.copy()
    r = O.gated_layer(h, bank, Ps[0], None, ws[0], cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu, 0.95,
                      flags=O.FLAG_REVALIDATE, tick=3, reval_every=2, drift_bound=0.05)
    assert r.refreshed == [s_sampled]
    i = r.revalidated.index(1)
    want = np.abs(plain[1] - drifted[s_sampled]).max() / np.abs(drifted[s_sampled]).max()
    assert abs(r.divergence[i] - want) < 1e-12 and want > 0.05
    np.testing.assert_allclose(bank.act[s_sampled], plain[1], atol=1e-6)
    assert np.array_equal(bank.act[s_other], drifted[s_other])
    np.testing.assert_allclose(r.h_out[1], plain[1], atol=1e-12)          # the sampled row returns the fresh output
    assert np.array_equal(r.h_out[2], drifted[s_other])                   # the other one still returns its cache
    # without the flag, or with reval_every 0, nothing is recomputed; sampled rows are not inserted again
    r = O.gated_layer(h, bank, Ps[0], None, ws[0], cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu, 0.95,
                      flags=O.FLAG_INSERT_ON_MISS, tick=4, reval_every=2, drift_bound=0.05)
    assert r.revalidated == [] and r.slots == []
    n_valid = int(bank.valid.sum())
    r = O.gated_layer(h, bank, Ps[0], None, ws[0], cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu, 0.95,
                      flags=O.FLAG_INSERT_ON_MISS | O.FLAG_REVALIDATE, tick=4, reval_every=1, drift_bound=0.05)
    assert r.revalidated == list(range(cfg.B)) and r.slots == [] and int(bank.valid.sum()) == n_valid


def test_compressed_values_are_projections_on_the_basis():
    g = rng(21)
    S, d, r = 5, 16, 4
    U, _ = np.linalg.qr(g.standard_normal((d, r)))
    U = U.T                                              # [r, d], orthonormal rows
    bank = O.Bank(3, 2, S, d, "f32", basis=U)
    assert bank.act.shape == (3, S, r)
    inside = g.standard_normal((S, r)) @ U               # lies in the span: reconstructed exactly (to fp32 storage)
    outside = g.standard_normal((S, d))
    q = np.ones((2, 2), np.float32)
    bank.insert(q, O.inv_norm(q), np.stack([inside, outside]), tick=1)
    np.testing.assert_allclose(bank.value(0), inside, atol=1e-6)
    # the reconstruction of a general output is its orthogonal projection: explicit loops
    want = np.zeros((S, d))
    for t in range(S):
        for i in range(r):
            c = sum(outside[t, j] * U[i, j] for j in range(d))
            for j in range(d):
                want[t, j] += c * U[i, j]
    np.testing.assert_allclose(bank.value(1), want, atol=1e-6)
    resid = outside - bank.value(1)
    assert np.abs(resid @ U.T).max() < 1e-6               # what is lost is orthogonal to the basis
    # a full-rank basis loses nothing; a hit of the gated layer returns the reconstruction
    full = O.Bank(2, 2, S, d, "f32", basis=np.eye(d))
    full.insert(q[:1], O.inv_norm(q[:1]), outside[None], tick=1)
    np.testing.assert_allclose(full.value(0), outside, atol=1e-6)
    cfg, ws, tok, pos, Ps, src, h_src = tiny_setup()
    Ub, _ = np.linalg.qr(rng(22).standard_normal((cfg.d, 8)))
    cb = O.Bank(cfg.n_bank, cfg.k, cfg.S, cfg.d, "f32", basis=Ub.T)
    r1 = O.gated_layer(h_src[:cfg.B], cb, Ps[0], None, ws[0], cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu, 2.0,
                       flags=O.FLAG_INSERT_ON_MISS, tick=1)
    r2 = O.gated_layer(h_src[:cfg.B], cb, Ps[0], None, ws[0], cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu, 0.95)
    assert r2.hit.all()
    np.testing.assert_allclose(r2.h_out, (r1.h_out @ Ub) @ Ub.T, atol=1e-5)


def test_single_fingerprint_mode_reuses_layer_one_key():
    cfg, ws, tok, pos, Ps, src, h_src = tiny_setup()
    banks = [O.Bank(cfg.n_bank, cfg.k, cfg.S, cfg.d, "f32") for _ in range(2)]
    _, res = O.infer(h_src, banks, Ps, [None, None], ws, cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu, tau=2.0,
                     flags=O.FLAG_INSERT_ON_MISS, tick=1, single_fingerprint=True)
    assert np.array_equal(banks[0].fp, banks[1].fp)
    assert np.array_equal(res[0].q, res[1].q)
    _, res2 = O.infer(h_src[:3], banks, Ps, [None, None], ws, cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu,
                      tau=0.99, single_fingerprint=True)
    assert all(r.hit.all() for r in res2)


def test_workload_generators_are_deterministic_and_shaped():
    cfg = W.scaled(W.BERT_BASE, B=10, S=40, n_layers=1)
    a = W.make_sources(cfg, 5, seed=1)
    b = W.make_sources(cfg, 5, seed=1)
    assert np.array_equal(a, b) and a.shape == (5, 40) and a.max() < cfg.vocab
    ids, s = W.make_substitution_queries(cfg, a, n_dup=6, n_subst=2, seed=2)
    for r_ in range(10):
        if s[r_] >= 0:
            assert (ids[r_] != a[s[r_]]).sum() <= 2
    assert (s >= 0).sum() == 6
    dcfg = W.scaled(W.GPT2_SMALL, B=4, S=64, n_layers=1)
    srcs = W.make_sources(dcfg, 3, seed=1)
    ids, s, plen = W.make_prefix_queries(dcfg, srcs, seed=2)
    for r_ in range(4):
        assert np.array_equal(ids[r_, :plen[r_]], srcs[s[r_], :plen[r_]]) and 16 <= plen[r_] <= 48
    cl = W.make_clustered_bank(8, 4, 32, 0.05, 10, seed=5)
    assert cl["bank"].shape == (32, 32) and cl["queries"].shape == (10, 32)
    n = cl["bank"].float().norm(dim=1)
    assert torch.all((n - 1).abs() < 1e-2)
    st = W.StemStream(W.scaled(W.BERT_LARGE, B=8, S=20, n_layers=1), group=4, stem_len=12, n_stems=5)
    ids, sid = st.next_batch()
    assert np.array_equal(ids[0, :12], ids[3, :12]) and not np.array_equal(ids[0, 12:], ids[1, 12:])


# ---- within-batch reuse: Algorithm 1 applied to the rows of a batch one after the other ----------

def test_dedup_equals_algorithm_1_row_by_row():
    """FLAG_DEDUP against the literal sequential algorithm: the same rows fed one at a time (each miss stored before
    the next row is looked up).  Keys are hand-made unit vectors in a plane, so every similarity is a known cosine:
    bank entries at 0 and 90 degrees; batch rows at
        0 (hits the bank), 200 (fresh: leader), 200 again (exact duplicate: follows), 230 (cos 30 = 0.866 < tau: a
        second leader), 220 (cos 20 = 0.94 to the first leader, cos 10 = 0.985 to the second: follows the SECOND),
        90 (hits the bank), 300 (fresh: leader), 205 (follows the first leader)."""
    cfg, ws, _tok, _pos, Ps, _src, h_src = tiny_setup(n_src=10)
    wnp = ws[0]
    tau = 0.9
    k = cfg.k
    def key(deg):
        v = np.zeros((k,), np.float32)
        v[0], v[1] = math.cos(math.radians(deg)), math.sin(math.radians(deg))
        return v
    angles = [0, 200, 200, 230, 220, 90, 300, 205]
    B = len(angles)
    q = np.stack([key(a) for a in angles])
    qinv = O.inv_norm(q)
    h = rng(5).standard_normal((B, cfg.S, cfg.d))
    flags = O.FLAG_INSERT_ON_MISS | O.FLAG_UPDATE_LRU

    def fresh_bank():
        bank = O.Bank(8, k, cfg.S, cfg.d, "f32")
        seed_keys = np.stack([key(0), key(90)])
        vals = rng(6).standard_normal((2, cfg.S, cfg.d)).astype(np.float32)
        bank.insert(seed_keys, O.inv_norm(seed_keys), vals, tick=1)
        return bank

    # the batch at once, with within-batch reuse
    bank_b = fresh_bank()
    r = O.gated_layer(h, bank_b, None, None, wnp, cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu, tau,
                      flags=flags | O.FLAG_DEDUP, tick=2, out_dtype="f32", fp_override=(q, qinv))
    assert r.follower_of == {2: 1, 4: 3, 7: 1}
    assert r.hit.tolist() == [True, False, True, False, True, True, False, True]
    # row by row: Algorithm 1 as printed
    bank_s = fresh_bank()
    seq_hit, seq_idx, seq_out = [], [], []
    for b in range(B):
        rb = O.gated_layer(h[b:b + 1], bank_s, None, None, wnp, cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu, tau,
                           flags=flags, tick=2, out_dtype="f32", fp_override=(q[b:b + 1], qinv[b:b + 1]))
        seq_hit.append(bool(rb.hit[0]))
        seq_idx.append(int(rb.idx[0]) if rb.hit[0] else rb.slots[0])
        seq_out.append(rb.h_out[0])
    assert r.hit.tolist()[0] and seq_hit == [True, False, True, False, True, True, False, True]
    # the entry a row ends up associated with: the slot it hit, or the slot it was stored in
    slot_of_leader = {b: s for b, s in zip([b for b in range(B) if not r.hit[b]], r.slots)}
    got_idx = [int(r.idx[b]) if r.hit[b] else slot_of_leader[b] for b in range(B)]
    assert got_idx == seq_idx
    for b in range(B):
        want = seq_out[b]
        if r.hit[b]:
            want = np.asarray(want, dtype=np.float32)        # reused rows return the value as stored
        np.testing.assert_allclose(r.h_out[b], want, rtol=0, atol=1e-6)
    # and the banks end up identical: keys, validity, recency, hit counts, values
    assert np.array_equal(bank_b.valid, bank_s.valid) and np.array_equal(bank_b.fp, bank_s.fp)
    assert np.array_equal(bank_b.last_used, bank_s.last_used) and np.array_equal(bank_b.hits, bank_s.hits)
    assert np.array_equal(bank_b.act, bank_s.act)
    assert bank_b.hits[:2].tolist() == [1, 1] and int(bank_b.valid.sum()) == 5
    # similarities reported for followers are those to the leader's key
    np.testing.assert_allclose([r.sim[2], r.sim[4], r.sim[7]],
                               [1.0, math.cos(math.radians(10)), math.cos(math.radians(5))], atol=1e-6)
    # without the flag the same batch stores every miss (five rows, the snapshot semantics)
    bank_n = fresh_bank()
    rn = O.gated_layer(h, bank_n, None, None, wnp, cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu, tau,
                       flags=flags, tick=2, out_dtype="f32", fp_override=(q, qinv))
    assert int((~rn.hit).sum()) == 6 and len(rn.slots) == 6 and rn.follower_of == {}
