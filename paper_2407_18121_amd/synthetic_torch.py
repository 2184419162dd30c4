"""Device-side variant of the synthetic workload recipe, for shapes too large to draw on the host.

Same recipe as `synthetic.py` (N(0,1) tensors, sink key x8, 5% heavy-hitter keys x4 shared by the
heads of a batch element, image-token keys x0.5, rounding to the storage type) with the normal
draws taken from a seeded torch generator on the device.  Inputs only; no method arithmetic.
Callers that need the oracle's view of the same bits copy the tensors (or slices) to the host.
"""
from __future__ import annotations

import numpy as np
import torch

from . import synthetic as syn


def _gen(cfg, layer, tensor_id, device):
    g = torch.Generator(device=device)
    g.manual_seed(syn.BASE_SEED * 1000003 + cfg.cid * 10007 + layer * 101 + tensor_id)
    return g


def torch_dtype(cfg):
    return torch.float32 if cfg.dtype == "f32" else torch.bfloat16


def prompt_qkv_device(cfg: syn.Config, layer: int, device="cuda"):
    """Q, K, V [B,H,T,D] in cfg.dtype on `device`."""
    shape = (cfg.B, cfg.H, cfg.T, cfg.D)
    q = torch.randn(shape, generator=_gen(cfg, layer, 0, device), device=device, dtype=torch.float32)
    k = torch.randn(shape, generator=_gen(cfg, layer, 1, device), device=device, dtype=torch.float32)
    v = torch.randn(shape, generator=_gen(cfg, layer, 2, device), device=device, dtype=torch.float32)
    img = torch.from_numpy(syn.image_mask(cfg)).to(device)
    k[:, :, img, :] *= 0.5
    for b in range(cfg.B):
        hh = torch.from_numpy(syn.heavy_hitters(cfg, layer, b)).to(device)
        k[b, :, hh, :] *= 4.0
    k[:, :, 0, :] *= 8.0
    dt = torch_dtype(cfg)
    return q.to(dt), k.to(dt), v.to(dt)


def decode_stream_device(cfg: syn.Config, layer: int, device="cuda"):
    """q, k_new, v_new for every step: three tensors [steps,B,H,D] in cfg.dtype on `device`."""
    shape = (cfg.decode_steps, cfg.B, cfg.H, cfg.D)
    dt = torch_dtype(cfg)
    return tuple(torch.randn(shape, generator=_gen(cfg, layer, 4 + i, device), device=device,
                             dtype=torch.float32).to(dt) for i in range(3))
