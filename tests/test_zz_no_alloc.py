"""llmc_match_noalloc, the bank match for callers that cannot allocate: its results against llmc_match's on the
same inputs, on two calls in a row that share the library's fixed scratch (the second smaller than the first),
and its refusal of sizes beyond that scratch."""
import sys

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def unit_rows(g, n, k):
    x = g.standard_normal((n, k))
    return x / np.linalg.norm(x, axis=1, keepdims=True)


def make_bank(L, N, k, seed, holes=True):
    g = np.random.Generator(np.random.PCG64(seed))
    bank = L.Bank(N, k, 1, 64, torch.bfloat16, "cuda")
    bank.fp.copy_(torch.from_numpy(unit_rows(g, N, k).astype(np.float32)).to(torch.bfloat16))
    L.llmc_inv_norm(bank.fp, bank.inv_norm)
    valid = np.ones(N, np.uint8)
    if holes:
        valid[g.random(N) < 0.1] = 0
    bank.valid.copy_(torch.from_numpy(valid))
    bank.refresh()
    return bank, g


def both(L, bank, q, tau):
    B = q.shape[0]
    qinv = torch.empty((B,), dtype=torch.float32, device="cuda")
    L.llmc_inv_norm(q, qinv)
    res = []
    for variant in ("workspace", "noalloc"):
        idx = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        sim = torch.full((B,), -7.0, dtype=torch.float32, device="cuda")
        hit = torch.full((B,), 9, dtype=torch.uint8, device="cuda")
        tie = torch.full((B,), 9, dtype=torch.uint8, device="cuda")
        if variant == "workspace":
            ws = torch.empty((L.llmc_match_workspace_bytes(bank, B),), dtype=torch.uint8, device="cuda")
            L.llmc_match(bank, q, qinv, tau, idx, sim, hit, tie, ws)
        else:
            L.llmc_match_noalloc(bank, q, qinv, tau, idx, sim, hit, tie)
        torch.cuda.synchronize()
        res.append((idx, sim, hit, tie))
    return res


def test_match_noalloc_equals_match_on_two_calls_in_a_row():
    from paper_2512_16843_amd import llmc as L
    assert torch.cuda.is_available()
    L.lib()
    # first call: 300 queries (the many-query kernel) against 20,000 slots; second, smaller: 37 queries against 1,000
    # slots of another bank, whose candidates land on scratch that still holds the first call's
    for N, B, k, seed in ((20000, 300, 256, 1), (1000, 37, 64, 2)):
        say(f"llmc_match_noalloc vs llmc_match: N={N} B={B} k={k}")
        bank, g = make_bank(L, N, k, seed)
        near = np.nonzero(bank.valid.cpu().numpy())[0][:B // 2]
        qn = np.concatenate([bank.fp[torch.from_numpy(near).cuda()].float().cpu().numpy()
                             + 0.02 * g.standard_normal((len(near), k)), unit_rows(g, B - len(near), k)])
        q = torch.from_numpy(qn.astype(np.float32)).to(torch.bfloat16).cuda()
        (i0, s0, h0, t0), (i1, s1, h1, t1) = both(L, bank, q, 0.9)
        assert torch.equal(i0, i1) and torch.equal(s0, s1) and torch.equal(h0, h1) and torch.equal(t0, t1)
        assert int(h0.sum()) > 0 and int((h0 == 0).sum()) > 0 and int(i0.min()) >= 0
        bank.close()


def test_match_noalloc_rejects_what_does_not_fit():
    from paper_2512_16843_amd import llmc as L
    L.lib()
    bank, g = make_bank(L, 16384, 256, 3, holes=False)
    B = 4096
    assert L.llmc_match_workspace_bytes(bank, B) > L.MATCH_STATIC_SCRATCH_BYTES
    q = torch.from_numpy(unit_rows(g, B, 256).astype(np.float32)).to(torch.bfloat16).cuda()
    qinv = torch.ones((B,), dtype=torch.float32, device="cuda")
    idx = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    with pytest.raises(L.LlmcError) as e:
        L.llmc_match_noalloc(bank, q, qinv, 0.9, idx, None, None, None)
    assert e.value.status == L.ERR_WORKSPACE and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert torch.all(idx == -7)                 # nothing was enqueued
    bank.close()
