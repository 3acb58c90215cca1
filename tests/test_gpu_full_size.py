"""GPU parity at the full sizes of the workload configs, in the launch configuration the
benchmark times.  The oracle cannot run whole batches at these sizes, so it is applied to
sampled rows (teacher-forced with the GPU's own layer inputs and bank arrays), and the rest
is covered by properties that hold at any size.
"""
import copy
import sys

import numpy as np
import pytest
import torch

from oracle import llmc_oracle as O
from paper_2512_16843_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2


def say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def L():
    from paper_2512_16843_amd import llmc
    assert torch.cuda.is_available()
    llmc.lib()
    return llmc


def npf(t):
    return t.detach().float().cpu().numpy()


def f32(x):
    return float(np.float32(x))


def rel_err_rows(got, want):
    got = np.asarray(got, dtype=np.float64).reshape(got.shape[0], -1)
    want = np.asarray(want, dtype=np.float64).reshape(want.shape[0], -1)
    return np.abs(got - want).max(axis=1) / np.maximum(np.abs(want).max(axis=1), 1e-30)


class LazyAct:
    """Cached outputs stay on the device; a row comes to the host when the oracle reads it."""

    def __init__(self, t):
        self.t = t

    def __getitem__(self, j):
        return npf(self.t[int(j)])


def oracle_view(bank, dtype="bf16"):
    ob = O.Bank(1, bank.k, 1, 1, dtype)
    ob.N, ob.S, ob.d, ob.A = bank.n_slots, bank.S, bank.d, bank.n_act_slots
    ob.fp, ob.inv_norm, ob.valid = npf(bank.fp), npf(bank.inv_norm), bank.valid.cpu().numpy()
    ob.act_slot = (np.arange(bank.n_slots, dtype=np.int32) if bank.act_slot is None
                   else bank.act_slot.cpu().numpy())
    ob.last_used = bank.last_used.cpu().numpy().astype(np.uint64)
    ob.hits = bank.hits.cpu().numpy().astype(np.uint32)
    ob.act = LazyAct(bank.act)
    return ob


def build_banks(L, st, cfg, src, tok, pos):
    src_t = torch.from_numpy(src).cuda()
    for s in range(0, src.shape[0], cfg.B):
        h = W.embed(src_t[s:s + cfg.B], tok, pos, cfg.torch_dtype)
        st.forward(h, tau=2.0, flags=L.INSERT_ON_MISS, tick=1)
    torch.cuda.synchronize()


def sampled_teacher_forced(L, st, cfg, ws, Ps, h0, tau, rows, layers):
    """Oracle on `rows` of the batch at `layers`, fed the GPU's own h_{l-1} and bank arrays."""
    outs = st.forward(h0, tau=tau, keep_all=True)
    torch.cuda.synchronize()
    report = []
    for l in layers:
        h_prev = h0 if l == 0 else outs[l - 1]
        ob = oracle_view(st.banks[l])
        wnp = {k: npf(v) for k, v in ws[l].items()}
        r = O.gated_layer(npf(h_prev[rows]), ob, npf(Ps[l]), None, wnp, cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu,
                          f32(tau))
        g = st.gate[l]
        hit = g.hit.cpu().numpy().astype(bool)[rows]
        idx = g.idx.cpu().numpy()[rows]
        sim = npf(g.sim)[rows]
        near = np.abs(r.sim - f32(tau)) < 1e-3
        ties = O.near_tie_sets(r.q, r.qinv, ob.fp, ob.inv_norm, ob.valid)
        multi = np.array([len(t) > 1 for t in ties])
        assert np.array_equal(hit[~near], r.hit[~near]), (l, hit, r.hit, r.sim)
        ok = ~near & ~multi
        assert np.array_equal(idx[ok], r.idx[ok]), (l, idx, r.idx)
        for i in np.nonzero(multi)[0]:
            assert idx[i] in ties[i]
        np.testing.assert_allclose(sim, r.sim, atol=2e-4)
        got = npf(outs[l][rows])
        err = 0.0
        for i in range(len(rows)):
            if hit[i]:
                assert np.array_equal(got[i], npf(st.banks[l].act[int(idx[i])]))
            elif not r.hit[i]:
                err = max(err, float(rel_err_rows(got[i:i + 1], r.h_out[i:i + 1])[0]))
        assert err < TOL_BF16, (l, err)
        report.append((l, int(hit.sum()), int(near.sum()), int(multi.sum()), err))
    # properties over the whole batch, every layer
    for l in range(cfg.n_layers):
        g = st.gate[l]
        hit = g.hit.bool()
        cnt = g.counters.cpu()
        assert int(cnt[L.CNT_HIT]) == int(hit.sum()) and int(cnt[L.CNT_HIT]) + int(cnt[L.CNT_MISS]) == cfg.B
        if hit.any():
            rows_h = torch.nonzero(hit).flatten()
            assert torch.all(st.banks[l].valid[g.idx[rows_h].long()] == 1)
            pick = rows_h[:: max(1, len(rows_h) // 4)][:4]
            for b in pick.tolist():
                assert torch.equal(outs[l][b], st.banks[l].act[int(g.idx[b])])
        assert torch.isfinite(outs[l].float()).all()
    return report


def test_bert_base_full_config_sampled(L):
    from paper_2512_16843_amd.engine import GatedStack
    cfg = W.BERT_BASE
    say(f"{cfg.name}: L={cfg.n_layers} B={cfg.B} S={cfg.S} bank {cfg.n_bank}: build + sampled teacher-forced parity")
    ws = W.make_layer_weights(cfg, seed=0)
    tok, pos = W.make_embeddings(cfg, seed=0)
    tok, pos = tok.cuda(), pos.cuda()
    Ps = W.make_projection(cfg.d, cfg.k, cfg.torch_dtype, seed=3, n_layers=cfg.n_layers)
    src = W.make_sources(cfg, cfg.n_bank, seed=1)
    st = GatedStack(cfg, ws, Ps)
    build_banks(L, st, cfg, src, tok, pos)
    for b in st.banks:
        assert int(b.valid.sum()) == cfg.n_bank
    ids, srcmap = W.make_substitution_queries(cfg, src, n_dup=38, n_subst=12, seed=2)
    h0 = W.embed(torch.from_numpy(ids).cuda(), tok, pos, cfg.torch_dtype)
    dup = np.nonzero(srcmap >= 0)[0][:2].tolist()
    fresh = np.nonzero(srcmap < 0)[0][:2].tolist()
    rows = dup + fresh
    for tau in (0.98, 2.0):
        rep = sampled_teacher_forced(L, st, cfg, ws, Ps, h0, tau, rows, layers=[0, 5, 11])
        for r in rep:
            say("  tau=%s layer %d: sampled hits %d, near-threshold %d, near-tie %d, max miss-row err %.2e"
                % ((tau,) + r))
        hits = st.hit_counts()[:, L.CNT_HIT].numpy()
        say("  tau=%s hits per layer %s" % (tau, hits.tolist()))
        if tau < 1:
            # a row that hit source j at layer l presents source j's next input: hits never decrease
            assert np.all(np.diff(hits) >= 0)
            g0 = st.gate[0]
            hit0 = g0.hit.cpu().numpy().astype(bool)
            assert np.array_equal(g0.idx.cpu().numpy()[hit0 & (srcmap >= 0)], srcmap[hit0 & (srcmap >= 0)])
    st.close()
    del st
    torch.cuda.empty_cache()


def test_gpt2_small_full_config_sampled(L):
    from paper_2512_16843_amd.engine import GatedStack
    cfg = W.GPT2_SMALL
    say(f"{cfg.name}: L={cfg.n_layers} B={cfg.B} S={cfg.S} bank {cfg.n_bank}: build + sampled teacher-forced parity")
    ws = W.make_layer_weights(cfg, seed=0)
    tok, pos = W.make_embeddings(cfg, seed=0)
    tok, pos = tok.cuda(), pos.cuda()
    Ps = W.make_projection(cfg.d, cfg.k, cfg.torch_dtype, seed=3, n_layers=cfg.n_layers)
    src = W.make_sources(cfg, cfg.n_bank, seed=1)
    st = GatedStack(cfg, ws, Ps)
    build_banks(L, st, cfg, src, tok, pos)
    ids, srcmap, plen = W.make_prefix_queries(cfg, src, seed=2)
    h0 = W.embed(torch.from_numpy(ids).cuda(), tok, pos, cfg.torch_dtype)
    for tau in (0.95, 2.0):
        rep = sampled_teacher_forced(L, st, cfg, ws, Ps, h0, tau, rows=[0, 9], layers=[0, 11])
        for r in rep:
            say("  tau=%s layer %d: sampled hits %d, near-threshold %d, near-tie %d, max miss-row err %.2e"
                % ((tau,) + r))
        say("  tau=%s hits per layer %s" % (tau, st.hit_counts()[:, L.CNT_HIT].tolist()))
    st.close()
    del st
    torch.cuda.empty_cache()


def test_match_stress_full_size(L):
    say("bank-match stress: 1,048,576 keys x 256, 4,096 queries, threshold 0.95, gather of 384 x 768 outputs")
    data = W.make_clustered_bank(4096, 256, 256, 0.05, 4096, seed=5)
    N, k, S, d, A = 1048576, 256, 384, 768, 4096
    act_slot = data["cluster"].cuda()
    bank = L.Bank(N, k, S, d, torch.bfloat16, "cuda", n_act_slots=A, act_slot=act_slot)
    bank.fp.copy_(data["bank"])
    L.llmc_inv_norm(bank.fp, bank.inv_norm)
    bank.valid.fill_(1)
    g = torch.Generator(device="cuda").manual_seed(11)
    bank.act.copy_(torch.randn((A, S, d), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16))
    bank.refresh()
    q = data["queries"].cuda()
    B = q.shape[0]
    qinv = torch.empty((B,), dtype=torch.float32, device="cuda")
    L.llmc_inv_norm(q, qinv)
    idx = torch.empty((B,), dtype=torch.int32, device="cuda")
    sim = torch.empty((B,), dtype=torch.float32, device="cuda")
    hit = torch.empty((B,), dtype=torch.uint8, device="cuda")
    tie = torch.empty((B,), dtype=torch.uint8, device="cuda")
    ws = torch.empty((L.llmc_match_workspace_bytes(bank, B),), dtype=torch.uint8, device="cuda")
    tau = 0.95
    L.llmc_match(bank, q, qinv, tau, idx, sim, hit, tie, ws)
    torch.cuda.synchronize()
    idx2 = torch.empty_like(idx)
    L.llmc_match(bank, q, qinv, tau, idx2, sim, hit, tie, ws)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2)                       # run-to-run determinism
    # properties over all queries
    qc = data["q_cluster"].numpy()
    inside = qc >= 0
    idx_h, hit_h, sim_h = idx.cpu().numpy(), hit.cpu().numpy().astype(bool), npf(sim)
    assert idx_h.min() >= 0 and idx_h.max() < N
    assert np.array_equal(idx_h[inside] // 256, qc[inside])
    assert hit_h[inside].all() and not hit_h[~inside].any()
    say("  hit rate %.3f, near-tie rows %d" % (hit_h.mean(), int(tie.sum())))
    # oracle on sampled queries, one at a time
    bank_np = npf(bank.fp)
    binv_np = npf(bank.inv_norm)
    valid_np = np.ones(N, np.uint8)
    sample = list(range(0, B, 128))[:24] + [B - 1]
    qs, qis = npf(q[sample]), npf(qinv[sample])
    oidx, osim = O.match(qs, qis, bank_np, binv_np, valid_np)
    ties = O.near_tie_sets(qs, qis, bank_np, binv_np, valid_np)
    n_multi = 0
    for i, b in enumerate(sample):
        if len(ties[i]) > 1:
            n_multi += 1
            assert idx_h[b] in ties[i]
        else:
            assert idx_h[b] == oidx[i], (b, idx_h[b], oidx[i])
        assert abs(sim_h[b] - osim[i]) < 1e-5
        if abs(osim[i] - f32(tau)) >= 1e-3:
            assert hit_h[b] == (osim[i] > f32(tau))
    say("  %d sampled queries agree with the oracle (%d of them with oracle near-ties)" % (len(sample), n_multi))
    # gather of the hit rows: exact copies of the cluster's value row
    rows = torch.nonzero(hit).flatten().int()
    n = torch.tensor([rows.numel()], dtype=torch.int32, device="cuda")
    out = torch.zeros((B, S, d), dtype=torch.bfloat16, device="cuda")
    L.llmc_gather_hits(bank, idx, rows.contiguous(), n, B, out)
    torch.cuda.synchronize()
    for b in rows[:: max(1, rows.numel() // 16)].tolist():
        assert torch.equal(out[b], bank.act[int(idx_h[b]) // 256])
    miss_rows = torch.nonzero(hit == 0).flatten()
    assert torch.all(out[miss_rows[:8]] == 0)
    bank.close()
    del bank, out
    torch.cuda.empty_cache()


def test_bert_large_dynamic_bank_scaled_teacher_forced(L):
    """Insertion + LRU eviction across successive batches of stem-sharing candidates, on a
    scaled copy (2 layers, 96-entry banks, batch 32) that the oracle can follow batch by batch."""
    from paper_2512_16843_amd.engine import GatedStack
    cfg = W.scaled(W.BERT_LARGE, n_layers=2, B=32, n_bank=96)
    say(f"{cfg.name} scaled: L=2 B=32 S={cfg.S} bank 96, 6 batches with INSERT_ON_MISS | UPDATE_LRU")
    ws = W.make_layer_weights(cfg, seed=0)
    tok, pos = W.make_embeddings(cfg, seed=0)
    tok, pos = tok.cuda(), pos.cuda()
    Ps = W.make_projection(cfg.d, cfg.k, cfg.torch_dtype, seed=3, n_layers=cfg.n_layers)
    st = GatedStack(cfg, ws, Ps)
    stream = W.StemStream(cfg, group=4, stem_len=80, n_stems=6, seed=4)
    flags = L.INSERT_ON_MISS | L.UPDATE_LRU
    tau = 0.95
    wnp = [{k: npf(v) for k, v in w.items()} for w in ws]
    evicted_total = 0
    for tick in range(1, 7):
        ids, _ = stream.next_batch()
        h0 = W.embed(torch.from_numpy(ids).cuda(), tok, pos, cfg.torch_dtype)
        pre = []
        for b in st.banks:
            ob = O.Bank(b.n_slots, b.k, b.S, b.d, "bf16")
            ob.fp, ob.inv_norm, ob.act = npf(b.fp), npf(b.inv_norm), npf(b.act)
            ob.valid = b.valid.cpu().numpy().copy()
            ob.last_used = b.last_used.cpu().numpy().astype(np.uint64)
            ob.hits = b.hits.cpu().numpy().astype(np.uint32)
            pre.append(ob)
        outs = st.forward(h0, tau=tau, flags=flags, tick=tick, keep_all=True)
        torch.cuda.synchronize()
        for l in range(cfg.n_layers):
            h_prev = h0 if l == 0 else outs[l - 1]
            ob = pre[l]
            before = copy.deepcopy(ob)
            r = O.gated_layer(npf(h_prev), ob, npf(Ps[l]), None, wnp[l], cfg.arch, cfg.n_heads, cfg.ln_eps, cfg.gelu,
                              f32(tau), flags=O.FLAG_INSERT_ON_MISS | O.FLAG_UPDATE_LRU, tick=tick, out_dtype="bf16")
            g = st.gate[l]
            hit = g.hit.cpu().numpy().astype(bool)
            near = np.abs(r.sim - f32(tau)) < 1e-3
            assert np.array_equal(hit[~near], r.hit[~near])
            if not np.array_equal(hit, r.hit):
                say("  batch %d layer %d: a row within 1e-3 of the threshold was decided differently; "
                    "slot-level comparison skipped for this layer" % (tick, l))
                continue
            ties = O.near_tie_sets(r.q, r.qinv, before.fp, before.inv_norm, before.valid)
            gi = g.idx.cpu().numpy()
            for b in range(cfg.B):
                assert gi[b] == r.idx[b] or (gi[b] in ties[b])
            n_miss = int((~hit).sum())
            assert g.slots.cpu().tolist()[:n_miss] == r.slots
            cnt = g.counters.cpu()
            assert int(cnt[L.CNT_INSERTED]) == n_miss and int(cnt[L.CNT_EVICTED]) == r.n_evicted
            evicted_total += r.n_evicted
            bk = st.banks[l]
            assert np.array_equal(bk.valid.cpu().numpy(), ob.valid)
            v = ob.valid.astype(bool)
            assert np.array_equal(bk.last_used.cpu().numpy().astype(np.uint64)[v], ob.last_used[v])
            assert np.array_equal(bk.hits.cpu().numpy().astype(np.uint32)[v], ob.hits[v])
            miss = ~hit
            if miss.any():
                assert rel_err_rows(npf(outs[l])[miss], r.h_out[miss]).max() < TOL_BF16
            # stored values are the GPU's own outputs of the miss rows, bit for bit
            for i, b in enumerate(np.nonzero(miss)[0]):
                assert torch.equal(bk.act[r.slots[i]], outs[l][int(b)])
        say("  batch %d: hits per layer %s" % (tick, [int(st.gate[l].hit.sum()) for l in range(cfg.n_layers)]))
    assert evicted_total > 0
    st.close()
    del st
    torch.cuda.empty_cache()


def test_bert_large_full_config_dynamic_properties(L):
    """The full 24-layer, 32,768-entry-bank configuration with insertion and eviction active:
    banks pre-filled to capacity, then batches of stem-sharing candidates; checked by invariants."""
    from paper_2512_16843_amd.engine import GatedStack
    cfg = W.BERT_LARGE
    free, total = torch.cuda.mem_get_info()
    need = cfg.n_layers * cfg.n_bank * cfg.S * cfg.d * 2 + (8 << 30)
    if free < need:
        pytest.skip("needs %.0f GB of free HBM" % (need / 2 ** 30))
    say(f"{cfg.name}: L={cfg.n_layers} B={cfg.B} S={cfg.S} bank {cfg.n_bank}: pre-fill, then 6 batches with eviction")
    ws = W.make_layer_weights(cfg, seed=0)
    tok, pos = W.make_embeddings(cfg, seed=0)
    tok, pos = tok.cuda(), pos.cuda()
    Ps = W.make_projection(cfg.d, cfg.k, cfg.torch_dtype, seed=3, n_layers=cfg.n_layers)
    st = GatedStack(cfg, ws, Ps)
    stream = W.StemStream(cfg, group=4, stem_len=80, n_stems=512, seed=4)
    flags = L.INSERT_ON_MISS | L.UPDATE_LRU
    tick = 0
    for _ in range(cfg.n_bank // cfg.B):           # warm-up stream fills every bank
        tick += 1
        ids, _ = stream.next_batch()
        st.forward(W.embed(torch.from_numpy(ids).cuda(), tok, pos, cfg.torch_dtype), tau=2.0, flags=flags, tick=tick)
    torch.cuda.synchronize()
    for b in st.banks:
        assert int(b.valid.sum()) == cfg.n_bank
    tau = 0.95
    for step in range(6):
        tick += 1
        ids, _ = stream.next_batch()
        h0 = W.embed(torch.from_numpy(ids).cuda(), tok, pos, cfg.torch_dtype)
        lu_before = st.banks[3].last_used.clone()
        out = st.forward(h0, tau=tau, flags=flags, tick=tick)
        torch.cuda.synchronize()
        cnt = st.hit_counts()
        assert torch.all(cnt[:, L.CNT_HIT] + cnt[:, L.CNT_MISS] == cfg.B)
        assert torch.all(cnt[:, L.CNT_INSERTED] == cnt[:, L.CNT_MISS])
        assert torch.all(cnt[:, L.CNT_EVICTED] == cnt[:, L.CNT_INSERTED])       # banks are full: every insert evicts
        assert torch.all(cnt[:, L.CNT_DROPPED] == 0)
        for b in st.banks:
            assert int(b.valid.sum()) == cfg.n_bank
        # layer 3: the slots taken are exactly the least recently used ones (hits of this batch count as used now)
        g = st.gate[3]
        n_miss = int(cnt[3, L.CNT_MISS])
        if n_miss:
            slots = g.slots[:n_miss].long()
            assert len(torch.unique(slots)) == n_miss
            lu = lu_before.clone()
            hit_rows = torch.nonzero(g.hit).flatten()
            lu[g.idx[hit_rows].long()] = tick
            key = lu * cfg.n_bank + torch.arange(cfg.n_bank, device="cuda")
            want = torch.argsort(key)[:n_miss]
            assert torch.equal(slots, want)
            assert torch.all(st.banks[3].last_used[slots] == tick) and torch.all(st.banks[3].hits[slots] == 0)
        assert torch.isfinite(out.float()).all()
        say("  batch %d: hit rate %.3f, inserted %d, evicted %d" % (
            step, float(cnt[:, L.CNT_HIT].sum()) / (cfg.B * cfg.n_layers), int(cnt[:, L.CNT_INSERTED].sum()),
            int(cnt[:, L.CNT_EVICTED].sum())))
    st.close()
    del st
    torch.cuda.empty_cache()
