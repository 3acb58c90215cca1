"""Harness around the C ABI: holds device weights, banks and buffers of an L-layer
stack and calls ``llmc_layer_forward_gated`` once per layer (Algorithm 1's loop).

Nothing is computed in Python: each layer is one library call that enqueues
kernels on the current stream; hit/miss counts stay on the device.
"""
from __future__ import annotations

from typing import List, Optional

import torch

from . import llmc
from .workloads import ModelConfig


class GatedStack:
    def __init__(self, cfg: ModelConfig, weights, projections, device="cuda", cached_layers=None,
                 biases: Optional[List[Optional[torch.Tensor]]] = None, n_bank: Optional[int] = None,
                 policy: int = llmc.EVICT_LRU, B: Optional[int] = None, half_life: int = 0, reval_every: int = 0,
                 drift_bound: float = 0.0, bases: Optional[List[Optional[torch.Tensor]]] = None,
                 keep_means: bool = False, keep_next_keys: bool = False, key_bits: bool = False,
                 expose_keys: bool = False, lsh: bool = False, prefix_tokens: int = 0,
                 proj2: Optional[List[torch.Tensor]] = None):
        self.cfg = cfg
        self.device = device
        self.B = cfg.B if B is None else B
        # prefix_tokens > 0: every cached layer is looked up under keys made of the token average AND the mean of the
        # layer's self-attention outputs over the first prefix_tokens tokens (proj2[l] is [2 d, k])
        self.prefix_tokens = prefix_tokens
        assert not (prefix_tokens and (keep_means or key_bits)), "prefix keys are computed per call, nothing is carried"
        self.proj2 = None if not prefix_tokens else [p.to(device).contiguous() for p in proj2]
        self.layers = [llmc.layer_from_weights(cfg, w, device) for w in weights]
        self.proj = [p.to(device).contiguous() for p in projections]
        self.bias = [None if b is None else b.to(device).contiguous() for b in (biases or [None] * cfg.n_layers)]
        n_bank = cfg.n_bank if n_bank is None else n_bank
        cached = range(cfg.n_layers) if cached_layers is None else cached_layers
        self.banks: List[Optional[llmc.Bank]] = [None] * cfg.n_layers
        cached = list(cached)
        # keep_next_keys (with keep_means): bank l also stores each cached output's key under layer l + 1's map
        self.keep_next_keys = keep_next_keys and keep_means and not key_bits
        for l in cached:
            nxt = l + 1 if (self.keep_next_keys and l + 1 < cfg.n_layers and (l + 1) in cached) else None
            self.banks[l] = llmc.Bank(n_bank, cfg.k, cfg.S, cfg.d, cfg.torch_dtype, device, policy=policy,
                                      half_life=half_life, reval_every=reval_every, drift_bound=drift_bound,
                                      basis=None if bases is None or bases[l] is None else
                                      bases[l].to(device).contiguous(), keep_means=keep_means,
                                      next_proj=None if nxt is None else self.proj[nxt],
                                      next_bias=None if nxt is None else self.bias[nxt], key_bits=key_bits,
                                      lsh=lsh)
        ws_bytes = llmc.llmc_layer_workspace_bytes(self.layers[0], self.B, cfg.S, cfg.k)
        self.workspace = torch.empty((ws_bytes,), dtype=torch.uint8, device=device)
        self.buf = [torch.empty((self.B, cfg.S, cfg.d), dtype=cfg.torch_dtype, device=device) for _ in range(2)]
        if prefix_tokens:
            nb = llmc.llmc_fingerprint_prefix_workspace_bytes(self.layers[0].desc(), self.B, cfg.S, prefix_tokens)
            self.pfx_ws = torch.empty((nb,), dtype=torch.uint8, device=device)
            self.pfx_fp = [torch.empty((self.B, cfg.k), dtype=cfg.torch_dtype, device=device) for _ in range(cfg.n_layers)]
            self.pfx_inv = [torch.empty((self.B,), dtype=torch.float32, device=device) for _ in range(cfg.n_layers)]
        # keep_means: banks store the token mean of every cached output and a reused row hands it to the next layer
        self.keep_means = keep_means
        self._hint = [False] * cfg.n_layers
        # post-LayerNorm blocks leave the pooled chunk sums of the rows they compute for the next call, so with stored
        # means every row of a later layer normally arrives pooled one way or the other: the pooling launch is dropped
        # there from the start (rows that do arrive unpooled are pooled inside the projection, same bits)
        self.auto_hint = keep_means and cfg.arch == 0
        self._deferred = [False] * cfg.n_layers
        self._stat_host = torch.zeros((cfg.n_layers, llmc.CNT_WORDS), dtype=torch.int32).pin_memory() if keep_means else None
        self.counters_all = torch.zeros((cfg.n_layers, llmc.CNT_WORDS), dtype=torch.int32, device=device)
        self._stat_event = None
        self.gate = [llmc.GateBuffers(self.B, device, d=cfg.d if keep_means else 0,
                                      next_k=cfg.k if (self.banks[l] is not None and self.banks[l].next_fp is not None) else 0,
                                      dtype=cfg.torch_dtype, counters=self.counters_all[l],
                                      k_used=cfg.k if expose_keys else 0, key_bits=key_bits)
                     for l in range(cfg.n_layers)]

    def _update_hints(self) -> None:
        """Launch-shape hints from the hit counts of an EARLIER forward, read without waiting: when the copy that a
        previous call started has landed, layers whose producer answered every row from its bank get
        LLMC_HINT_MOSTLY_CARRIED (a single uncarried row costs a whole one-workgroup pooling, about what the
        dropped launch saves several times over) (cost only: results do not depend on it)."""
        if self._stat_event is not None and self._stat_event.query():
            hits = self._stat_host[:, llmc.CNT_HIT].tolist()
            for l in range(1, self.cfg.n_layers):
                self._hint[l] = hits[l - 1] >= self.B
            self._stat_event = None

    def _start_stats(self) -> None:
        if self._stat_event is not None or torch.cuda.is_current_stream_capturing():
            return
        self._stat_host.copy_(self.counters_all, non_blocking=True)      # one small device-to-host copy, not waited for
        self._stat_event = torch.cuda.Event()
        self._stat_event.record()

    def forward(self, h0: torch.Tensor, tau: float, flags: int = 0, tick: int = 0, keep_all: bool = False,
                single_fingerprint: bool = False, defer: Optional[bool] = None):
        """Run all layers; returns h_L (a view of an internal buffer) or, with
        ``keep_all``, the list [h_1 .. h_L] as fresh tensors.

        ``defer`` (default: on when the banks keep next-layer keys and the call neither inserts nor revalidates):
        reused rows are handed from layer to layer as references to the bank entry that answered them and are
        copied only where a later layer has to compute them, and once at the end."""
        cfg = self.cfg
        B = h0.shape[0]
        assert B == self.B and h0.is_contiguous()
        h = h0
        outs = []
        fp_given = inv_given = None
        if single_fingerprint:
            fp_given = torch.empty((B, cfg.k), dtype=cfg.torch_dtype, device=self.device)
            inv_given = torch.empty((B,), dtype=torch.float32, device=self.device)
            llmc.llmc_fingerprint(h0, self.proj[0], self.bias[0], fp_given, inv_given, self.workspace)
        if self.keep_means:
            self._update_hints()
        can_defer = (self.keep_next_keys and not keep_all and not single_fingerprint and
                     not (flags & (llmc.INSERT_ON_MISS | llmc.REVALIDATE)))
        defer = can_defer if defer is None else (defer and can_defer)
        prev = None                      # the bank whose entries the rows of h may refer to
        self._deferred = [False] * cfg.n_layers
        for l in range(cfg.n_layers):
            out = torch.empty_like(h0) if keep_all else self.buf[l & 1]
            if out.data_ptr() == h.data_ptr():
                out = self.buf[(l & 1) ^ 1]
            carry = self.gate[l - 1] if (self.keep_means and l > 0) else None
            fl = flags | (llmc.HINT_MOSTLY_CARRIED if (carry is not None and (self._hint[l] or self.auto_hint)) else 0)
            bank = self.banks[l]
            # a row may stay a reference across this layer only if this layer's bank stores the key that the
            # next layer needs; the last layer (and a layer before an uncached one) copies as usual
            defer_here = defer and bank is not None and bank.next_fp is not None
            if prev is not None and (bank is None or bank.key_bits):
                llmc.llmc_materialize(prev, self.gate[l - 1].ref, h)          # this layer cannot take references
                prev = None
            fp_l, inv_l = fp_given, inv_given
            if self.prefix_tokens and bank is not None and not single_fingerprint:
                fp_l, inv_l = self.pfx_fp[l], self.pfx_inv[l]
                llmc.llmc_fingerprint_prefix(self.layers[l].desc(), h, self.prefix_tokens, self.proj2[l], self.bias[l],
                                             fp_l, inv_l, self.pfx_ws)
            llmc.llmc_layer_forward_gated(self.layers[l], bank, self.proj[l], self.bias[l], h, out, tau,
                                          fl | (llmc.DEFER_COPY if defer_here else 0), tick, self.workspace,
                                          self.gate[l], fp_l, inv_l, carry=carry, prev_bank=prev)
            prev = bank if defer_here else None
            self._deferred[l] = defer_here
            h = out
            if keep_all:
                outs.append(out)
        if prev is not None:
            llmc.llmc_materialize(prev, self.gate[cfg.n_layers - 1].ref, h)
        if self.keep_means:
            self._start_stats()
        return outs if keep_all else h

    def copied_rows(self):
        """(plain, just_in_time): rows of cached outputs that the last forward copied in the reuse step of layers that
        did not defer, and rows that travelled as references and were copied because a later layer had to compute
        them or because they were still outstanding at the end (one host sync)."""
        plain = jit = 0
        L = self.cfg.n_layers
        for l in range(L):
            if self.banks[l] is None:
                continue
            g = self.gate[l]
            if not self._deferred[l]:
                plain += int(g.hit.sum())
            elif l + 1 < L:
                jit += int(((g.ref >= 0) & (self.gate[l + 1].hit == 0)).sum())
            else:
                jit += int((g.ref >= 0).sum())
        return plain, jit

    def hit_counts(self) -> torch.Tensor:
        """[L, CNT_WORDS] device counters of the last forward (one host sync)."""
        return self.counters_all.cpu()

    def close(self):
        for b in self.banks:
            if b is not None:
                b.close()
