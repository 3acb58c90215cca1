"""Seeded synthetic inputs for the cache-gated transformer layer.

This module only *draws inputs*: token ids, embedding tables, layer weights,
projection matrices, fingerprint clusters.  It holds none of the method's
arithmetic (no pooling, no similarity, no layer math), so both the CPU oracle's
tests and the HIP path's tests can take their inputs from it without sharing
any of the code under test.

All randomness comes from ``numpy.random.Generator(PCG64(seed))``.  Arrays are
returned as CPU torch tensors already rounded to the run dtype (fp32 or bf16),
so that both sides read exactly the same stored values.

The workloads stand in, by shape and token statistics only, for the corpora the
paper evaluates on (Section V-A): fixed-length encoder inputs, long causal
contexts, and groups of candidate sequences sharing a stem.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np
import torch

ENCODER_POST_LN = 0
DECODER_PRE_LN = 1

GELU_ERF = 0
GELU_TANH = 1


@dataclass(frozen=True)
class ModelConfig:
    """Shape of one transformer stack f_1..f_L (Section IV-A)."""

    name: str
    arch: int            # ENCODER_POST_LN or DECODER_PRE_LN
    n_layers: int
    d: int
    n_heads: int
    d_ff: int
    gelu: int            # GELU_ERF or GELU_TANH
    ln_eps: float
    dtype: str           # "f32" or "bf16"
    vocab: int
    B: int               # sequences per batch
    S: int               # tokens per sequence
    n_bank: int          # N, bank entries per layer
    k: int               # fingerprint dimension
    zipf_a: Optional[float] = None   # None = uniform token ids

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


TINY_ENCODER = ModelConfig(
    name="tiny-encoder", arch=ENCODER_POST_LN, n_layers=2, d=128, n_heads=2, d_ff=512,
    gelu=GELU_ERF, ln_eps=1e-12, dtype="f32", vocab=1000, B=8, S=32, n_bank=256, k=64)

BERT_BASE = ModelConfig(
    name="bert-base-shaped", arch=ENCODER_POST_LN, n_layers=12, d=768, n_heads=12, d_ff=3072,
    gelu=GELU_ERF, ln_eps=1e-12, dtype="bf16", vocab=30522, B=64, S=384, n_bank=16384, k=256,
    zipf_a=1.1)

GPT2_SMALL = ModelConfig(
    name="gpt2-small-shaped", arch=DECODER_PRE_LN, n_layers=12, d=768, n_heads=12, d_ff=3072,
    gelu=GELU_TANH, ln_eps=1e-5, dtype="bf16", vocab=50257, B=16, S=1024, n_bank=4096, k=256,
    zipf_a=1.05)

BERT_LARGE = ModelConfig(
    name="bert-large-shaped", arch=ENCODER_POST_LN, n_layers=24, d=1024, n_heads=16, d_ff=4096,
    gelu=GELU_ERF, ln_eps=1e-12, dtype="bf16", vocab=30522, B=256, S=128, n_bank=32768, k=256,
    zipf_a=1.1)


def scaled(cfg: ModelConfig, **kw) -> ModelConfig:
    """Copy of ``cfg`` with some fields replaced (smaller test-sized variants)."""
    d = dict(cfg.__dict__)
    d.update(kw)
    return ModelConfig(**d)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def _store(a: np.ndarray, dtype: torch.dtype) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dtype)


# ----------------------------------------------------------------------------
# weights and embeddings
# ----------------------------------------------------------------------------

LAYER_TENSORS = ("wqkv", "bqkv", "wo", "bo", "w1", "b1", "w2", "b2",
                 "ln1_g", "ln1_b", "ln2_g", "ln2_b")


def make_layer_weights(cfg: ModelConfig, seed: int = 0) -> List[Dict[str, torch.Tensor]]:
    """Random-init weights for every layer, stored in the run dtype.

    Linear weights are [out_features, in_features] (the contraction index is
    contiguous): ``wqkv [3d, d]`` (rows 0..d-1 = Q, d..2d-1 = K, 2d..3d-1 = V,
    head h owning features h*dh..(h+1)*dh-1 of each), ``wo [d, d]``,
    ``w1 [d_ff, d]``, ``w2 [d, d_ff]``.  Weights ~ N(0, 0.02^2).  Biases and
    the LayerNorm affine parameters are drawn non-trivially (b ~ N(0, 0.02^2),
    gamma ~ 1 + N(0, 0.05^2), beta ~ N(0, 0.05^2)) so that a dropped bias or
    affine term shows up in parity tests.
    """
    rng = _rng(seed)
    d, f = cfg.d, cfg.d_ff
    dt = cfg.torch_dtype
    layers = []
    for _ in range(cfg.n_layers):
        w = {
            "wqkv": _store(rng.normal(0.0, 0.02, (3 * d, d)), dt),
            "bqkv": _store(rng.normal(0.0, 0.02, (3 * d,)), dt),
            "wo": _store(rng.normal(0.0, 0.02, (d, d)), dt),
            "bo": _store(rng.normal(0.0, 0.02, (d,)), dt),
            "w1": _store(rng.normal(0.0, 0.02, (f, d)), dt),
            "b1": _store(rng.normal(0.0, 0.02, (f,)), dt),
            "w2": _store(rng.normal(0.0, 0.02, (d, f)), dt),
            "b2": _store(rng.normal(0.0, 0.02, (d,)), dt),
            "ln1_g": _store(1.0 + rng.normal(0.0, 0.05, (d,)), dt),
            "ln1_b": _store(rng.normal(0.0, 0.05, (d,)), dt),
            "ln2_g": _store(1.0 + rng.normal(0.0, 0.05, (d,)), dt),
            "ln2_b": _store(rng.normal(0.0, 0.05, (d,)), dt),
        }
        layers.append(w)
    return layers


def make_embeddings(cfg: ModelConfig, seed: int = 0) -> Tuple[torch.Tensor, torch.Tensor]:
    """Token table [vocab, d] and position table [S, d], N(0, 1), fp32.

    Unit-variance tables keep h_0 at the scale LayerNorm outputs have, so the
    first layer sees inputs of the same magnitude as the later ones.
    """
    rng = _rng(seed + 7919)
    tok = rng.standard_normal((cfg.vocab, cfg.d), dtype=np.float32)
    pos = rng.standard_normal((cfg.S, cfg.d), dtype=np.float32) * np.float32(0.1)
    return torch.from_numpy(tok), torch.from_numpy(pos)


def embed(ids: torch.Tensor, tok: torch.Tensor, pos: torch.Tensor, dtype: torch.dtype) -> torch.Tensor:
    """h_0 = E(X): table lookup plus position table, rounded to the run dtype.

    This is the model's input boundary (Section IV-A), not a step of the
    cache-gated layer; it is plain indexing done by the harness.
    """
    S = ids.shape[-1]
    h = tok[ids.long()] + pos[:S].unsqueeze(0)
    return h.to(dtype).contiguous()


def make_projection(d: int, k: int, dtype: torch.dtype, seed: int = 3,
                    n_layers: int = 1) -> List[torch.Tensor]:
    """Per-layer random projection P_l [d, k] ~ N(0, 1/k), stored in the run dtype."""
    rng = _rng(seed)
    return [_store(rng.normal(0.0, 1.0 / np.sqrt(k), (d, k)), dtype) for _ in range(n_layers)]


# ----------------------------------------------------------------------------
# token streams
# ----------------------------------------------------------------------------

class TokenLaw:
    """Token-id distribution: uniform, or rank r with p ~ r^-a mapped to ids by a seeded permutation."""

    def __init__(self, vocab: int, zipf_a: Optional[float], seed: int):
        self.vocab = vocab
        if zipf_a is None:
            self.cdf = None
            self.perm = None
        else:
            r = np.arange(1, vocab + 1, dtype=np.float64)
            p = r ** (-zipf_a)
            p /= p.sum()
            self.cdf = np.cumsum(p)
            self.cdf[-1] = 1.0
            self.perm = _rng(seed + 104729).permutation(vocab)

    def draw(self, rng: np.random.Generator, shape) -> np.ndarray:
        if self.cdf is None:
            return rng.integers(0, self.vocab, size=shape, dtype=np.int64)
        u = rng.random(size=shape)
        ranks = np.searchsorted(self.cdf, u, side="left")
        ranks = np.minimum(ranks, self.vocab - 1)
        return self.perm[ranks].astype(np.int64)


def make_sources(cfg: ModelConfig, n: int, seed: int = 1) -> np.ndarray:
    """``n`` seeded base sequences [n, S] from the config's token law."""
    law = TokenLaw(cfg.vocab, cfg.zipf_a, seed)
    return law.draw(_rng(seed), (n, cfg.S))


def make_substitution_queries(cfg: ModelConfig, sources: np.ndarray, n_dup: int, n_subst,
                              seed: int = 2) -> Tuple[np.ndarray, np.ndarray]:
    """Encoder-style queries: ``n_dup`` rows are copies of a random source with
    some positions resampled, the remaining ``B - n_dup`` rows are fresh.

    ``n_subst`` is an int (exactly that many distinct positions are resampled)
    or a pair (lo, hi) (a per-row count drawn uniformly from lo..hi).
    Returns (ids [B, S], src [B]) with src = source row or -1 for a fresh row.
    """
    rng = _rng(seed)
    law = TokenLaw(cfg.vocab, cfg.zipf_a, 1)
    B, S = cfg.B, cfg.S
    ids = law.draw(rng, (B, S))
    src = np.full((B,), -1, dtype=np.int64)
    rows = rng.permutation(B)[:n_dup]
    for b in rows:
        j = int(rng.integers(0, sources.shape[0]))
        src[b] = j
        row = sources[j].copy()
        ns = n_subst if isinstance(n_subst, int) else int(rng.integers(n_subst[0], n_subst[1] + 1))
        pos = rng.permutation(S)[:ns]
        row[pos] = law.draw(rng, (ns,))
        ids[b] = row
    return ids, src


def make_prefix_queries(cfg: ModelConfig, sources: np.ndarray, lo_frac: float = 0.25,
                        hi_frac: float = 0.75, seed: int = 2) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Decoder-style queries: each row shares a random-length prefix with a
    random source and continues with fresh tokens.  Returns (ids, src, prefix_len)."""
    rng = _rng(seed)
    law = TokenLaw(cfg.vocab, cfg.zipf_a, 1)
    B, S = cfg.B, cfg.S
    ids = law.draw(rng, (B, S))
    src = rng.integers(0, sources.shape[0], size=(B,))
    plen = rng.integers(int(lo_frac * S), int(hi_frac * S) + 1, size=(B,))
    for b in range(B):
        ids[b, :plen[b]] = sources[src[b], :plen[b]]
    return ids, src.astype(np.int64), plen.astype(np.int64)


def make_dial_queries(cfg: ModelConfig, sources: np.ndarray, rho: float, seed: int = 2
                      ) -> Tuple[np.ndarray, np.ndarray]:
    """Hit-rate dial: a fraction ``rho`` of rows are exact copies of bank
    sources, the rest are fresh draws.  Returns (ids, src)."""
    rng = _rng(seed)
    law = TokenLaw(cfg.vocab, cfg.zipf_a, 1)
    B = cfg.B
    ids = law.draw(rng, (B, cfg.S))
    src = np.full((B,), -1, dtype=np.int64)
    n_copy = int(round(rho * B))
    rows = rng.permutation(B)[:n_copy]
    for b in rows:
        j = int(rng.integers(0, sources.shape[0]))
        ids[b] = sources[j]
        src[b] = j
    return ids, src


class StemStream:
    """Stream of batches made of groups of candidates that share a stem.

    Each batch has ``B / group`` groups; a group is one ``stem_len``-token stem
    followed by ``group`` different fresh tails.  Stems recur: they are drawn
    from a pool of ``n_stems`` with Zipf(1.0) popularity, so later batches meet
    stems whose earlier completions were inserted into the banks.
    """

    def __init__(self, cfg: ModelConfig, group: int = 4, stem_len: int = 80, n_stems: int = 512,
                 seed: int = 4):
        assert cfg.B % group == 0 and stem_len < cfg.S
        self.cfg, self.group, self.stem_len = cfg, group, stem_len
        self.law = TokenLaw(cfg.vocab, cfg.zipf_a, 1)
        self.rng = _rng(seed)
        self.stems = self.law.draw(self.rng, (n_stems, stem_len))
        pop = 1.0 / np.arange(1, n_stems + 1, dtype=np.float64)
        self.pop_cdf = np.cumsum(pop / pop.sum())
        self.pop_cdf[-1] = 1.0

    def next_batch(self) -> Tuple[np.ndarray, np.ndarray]:
        cfg = self.cfg
        n_groups = cfg.B // self.group
        u = self.rng.random(n_groups)
        stem_id = np.minimum(np.searchsorted(self.pop_cdf, u), len(self.pop_cdf) - 1)
        ids = self.law.draw(self.rng, (cfg.B, cfg.S))
        for g in range(n_groups):
            ids[g * self.group:(g + 1) * self.group, :self.stem_len] = self.stems[stem_id[g]]
        return ids, np.repeat(stem_id, self.group)


# ----------------------------------------------------------------------------
# bank-match stress inputs (clustered unit fingerprints)
# ----------------------------------------------------------------------------

def make_clustered_bank(n_clusters: int, per_cluster: int, k: int, sigma: float, n_queries: int,
                        frac_within: float = 0.5, seed: int = 5, chunk: int = 65536
                        ) -> Dict[str, torch.Tensor]:
    """Unit-norm Gaussian fingerprints in ``n_clusters`` clusters, bf16.

    Entry j belongs to cluster j // per_cluster and equals
    ``unit(c + sigma * g / sqrt(k))``, g ~ N(0, I): ``sigma`` is the expected
    norm of the perturbation.  Queries: a fraction ``frac_within`` are further
    draws from a random cluster, the rest are uniform on the sphere.
    Returns bf16 tensors ``bank [N, k]``, ``queries [Q, k]`` plus ``cluster [N]``
    (int32) and ``q_cluster [Q]`` (int64, -1 = uniform query).  The inverse norms of
    the *stored* vectors are not computed here: that is part of the method.
    """
    rng = _rng(seed)
    centres = rng.standard_normal((n_clusters, k))
    centres /= np.linalg.norm(centres, axis=1, keepdims=True)
    N = n_clusters * per_cluster
    bank = torch.empty((N, k), dtype=torch.bfloat16)
    scale = sigma / np.sqrt(k)
    for s in range(0, N, chunk):
        e = min(N, s + chunk)
        cl = np.arange(s, e) // per_cluster
        v = centres[cl] + scale * rng.standard_normal((e - s, k))
        v /= np.linalg.norm(v, axis=1, keepdims=True)
        bank[s:e] = torch.from_numpy(v.astype(np.float32)).to(torch.bfloat16)
    n_in = int(round(frac_within * n_queries))
    q_cluster = np.full((n_queries,), -1, dtype=np.int64)
    rows = rng.permutation(n_queries)[:n_in]
    q = rng.standard_normal((n_queries, k))
    for b in rows:
        c = int(rng.integers(0, n_clusters))
        q_cluster[b] = c
        q[b] = centres[c] + scale * rng.standard_normal(k)
    q /= np.linalg.norm(q, axis=1, keepdims=True)
    return {
        "bank": bank,
        "queries": torch.from_numpy(q.astype(np.float32)).to(torch.bfloat16),
        "cluster": torch.from_numpy((np.arange(N) // per_cluster).astype(np.int32)),
        "q_cluster": torch.from_numpy(q_cluster),
    }
