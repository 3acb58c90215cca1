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
