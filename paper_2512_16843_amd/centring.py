"""Input preparation for the centred fingerprint: the offsets c_l = -P_l^T mu_l.

Section IV-B names PCA beside SimHash as the dimensionality reduction; PCA subtracts the mean of the data before
projecting, and for a linear map that subtraction is one offset vector per layer, which the fingerprint call takes as
its optional ``c``.  mu_l is the mean, over the sequences the banks are built from, of the token mean of layer l's
input.  This module measures mu_l with plain torch reductions on the outputs of an UNCACHED forward (banks play no
part) and returns the offsets as fp32 arrays; they are inputs of the path, like the projections, and the same arrays
go to the CPU oracle and to the library.  Nothing here runs inside the cache-gated layer.
"""
from __future__ import annotations

from typing import Iterable, List

import torch

from .engine import GatedStack
from .workloads import ModelConfig


def centring_offsets(cfg: ModelConfig, weights, projections, batches: Iterable[torch.Tensor], device="cuda"
                     ) -> List[torch.Tensor]:
    """``batches`` yields device tensors h_0 [B, S, d] (the embedded bank sources, every batch of cfg.B rows).
    Returns one fp32 [k] tensor per layer (on the host)."""
    plain = GatedStack(cfg, weights, projections, device=device, cached_layers=[])
    sums = [torch.zeros((cfg.d,), dtype=torch.float64, device=device) for _ in range(cfg.n_layers)]
    n = 0
    for h0 in batches:
        outs = plain.forward(h0, tau=2.0, keep_all=True)
        ins = [h0] + outs[:-1]
        for l in range(cfg.n_layers):
            sums[l] += ins[l].to(torch.float64).mean(dim=1).sum(dim=0)
        n += h0.shape[0]
    plain.close()
    out = []
    for l in range(cfg.n_layers):
        mu = sums[l] / float(n)
        P = projections[l].to(device).to(torch.float64)
        out.append((-(mu @ P)).to(torch.float32).cpu().contiguous())
    return out


def prefix_feature_stats(cfg: ModelConfig, weights, proj2, batches: Iterable[torch.Tensor], n_prefix: int,
                         device="cuda"):
    """Mean and spread of the two fingerprint features (token average p, prefix attention mean a) of every layer's
    input over the sequences a bank is built from.  The features are taken from the library's own call
    (llmc_fingerprint_prefix leaves [p; a] of every row at the head of its workspace), the layer inputs from an
    uncached forward.  Returns per layer (mu [2 d] float64 on the host, E|p - mu_p|^2, E|a - mu_a|^2).
    ``proj2[l]`` [2 d, k] is only there because the call wants a map; the keys it makes are not used."""
    from . import llmc
    d = cfg.d
    plain = GatedStack(cfg, weights, [p[:d] for p in proj2], device=device, cached_layers=[])
    s1 = [torch.zeros((2 * d,), dtype=torch.float64, device=device) for _ in range(cfg.n_layers)]
    s2 = [torch.zeros((2 * d,), dtype=torch.float64, device=device) for _ in range(cfg.n_layers)]
    P2 = [p.to(device).contiguous() for p in proj2]
    ws = torch.empty((llmc.llmc_fingerprint_prefix_workspace_bytes(plain.layers[0].desc(), cfg.B, cfg.S, n_prefix),),
                     dtype=torch.uint8, device=device)
    fp = torch.empty((cfg.B, cfg.k), dtype=cfg.torch_dtype, device=device)
    inv = torch.empty((cfg.B,), dtype=torch.float32, device=device)
    n = 0
    for h0 in batches:
        outs = plain.forward(h0, tau=2.0, keep_all=True)
        ins = [h0] + outs[:-1]
        for l in range(cfg.n_layers):
            llmc.llmc_fingerprint_prefix(plain.layers[l].desc(), ins[l], n_prefix, P2[l], None, fp, inv, ws)
            feat = ws[:cfg.B * 2 * d * 4].view(torch.float32).view(cfg.B, 2 * d).to(torch.float64)
            s1[l] += feat.sum(dim=0)
            s2[l] += (feat * feat).sum(dim=0)
        n += h0.shape[0]
    plain.close()
    out = []
    for l in range(cfg.n_layers):
        mu = s1[l] / float(n)
        var = (s2[l] / float(n) - mu * mu).clamp_min(0.0)
        out.append((mu.cpu(), float(var[:d].sum()), float(var[d:].sum())))
    return out
