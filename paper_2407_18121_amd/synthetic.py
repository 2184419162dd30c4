"""Seeded synthetic workloads standing in for the paper's LLaVA-shaped prompts.

This module only produces inputs (shapes, value distributions, token layout,
number formats).  It contains none of the method's arithmetic and is the one
module both the GPU tests/benchmark and the CPU oracle's callers use, so that
both sides see identical bits.

Recipe: Q, K, V and the per-step decode vectors are N(0,1) fp32 drawn from a
counter-based generator keyed by (base seed, config, layer, tensor, batch
element).  Key 0 is multiplied by 8 (attention sink); floor(0.05*T) distinct
positions in 1..T-1, drawn once per (config, layer, batch element) and shared by
all heads, are multiplied by 4 (heavy hitters); keys of image-patch tokens are
multiplied by 0.5.  bf16 configs round the result to bf16 (nearest even).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Tuple

import numpy as np

BASE_SEED = 20240718
RECENT = 25  # recent distance of the fixed-point elimination (Sec. 4.1)


@dataclass(frozen=True)
class Config:
    name: str
    cid: int
    layers: int
    H: int
    D: int
    B: int
    T: int
    dtype: str  # "f32" | "bf16"
    gamma: Tuple[int, int]  # retention ratio as a fraction
    decode_steps: int
    # (kind, length) runs; kind "i" = image-patch tokens, "t" = text tokens
    layout: Tuple[Tuple[str, int], ...] = field(default=())

    @property
    def n_anchor(self) -> int:
        p, q = self.gamma
        return (p * self.T + q - 1) // q

    @property
    def cap(self) -> int:
        """Cache rows needed for the whole run (ratio budget grows by gamma per token, +1 for the append)."""
        p, q = self.gamma
        return (p * (self.T + self.decode_steps) + q - 1) // q + 1

    @property
    def esize(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.D))


def _llava_layout(T: int):
    return (("t", 32), ("i", 576), ("t", T - 608))


CONFIGS = {
    "C1": Config("C1", 1, 1, 4, 64, 1, 256, "f32", (1, 2), 32, (("t", 256),)),
    "C2": Config("C2", 2, 32, 32, 128, 1, 1024, "bf16", (1, 2), 512, _llava_layout(1024)),
    "C3": Config("C3", 3, 32, 32, 128, 8, 2048, "bf16", (1, 4), 512, _llava_layout(2048)),
    "C4": Config("C4", 4, 40, 40, 128, 4, 1024, "bf16", (1, 2), 512, _llava_layout(1024)),
    "C5": Config("C5", 5, 32, 32, 128, 16, 8192, "bf16", (1, 10), 1024,
                 (("t", 32),) + (("i", 576), ("t", 64)) * 12 + (("t", 480),)),
    # shapes of the paper's own speed measurements (Table 2: budget 0.2, prompt + generated lengths)
    "T1": Config("T1", 11, 40, 40, 128, 8, 1024, "bf16", (1, 5), 512, _llava_layout(1024)),
    "T2": Config("T2", 12, 40, 40, 128, 16, 624, "bf16", (1, 5), 256, _llava_layout(624)),
    "T3": Config("T3", 13, 32, 32, 128, 16, 1024, "bf16", (1, 5), 512, _llava_layout(1024)),
    "T4": Config("T4", 14, 32, 32, 128, 48, 624, "bf16", (1, 5), 256, _llava_layout(624)),
}


def image_mask(cfg: Config) -> np.ndarray:
    """bool [T]: True where the token is an image patch."""
    m = np.zeros(cfg.T, dtype=bool)
    t = 0
    for kind, n in cfg.layout:
        if kind == "i":
            m[t:t + n] = True
        t += n
    assert t == cfg.T, (t, cfg.T)
    return m


# ---------------------------------------------------------------- number formats
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 array holding values exactly representable in `dtype`."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return x if dtype == "f32" else bf16_bits_to_f32(f32_to_bf16_bits(x))


# ---------------------------------------------------------------- generators
_TENSOR_ID = {"q": 0, "k": 1, "v": 2, "hh": 3, "dq": 4, "dk": 5, "dv": 6}


def _rng(cfg: Config, layer: int, tensor: str, b: int, extra: int = 0):
    return np.random.default_rng([BASE_SEED, cfg.cid, layer, _TENSOR_ID[tensor], b, extra])


def heavy_hitters(cfg: Config, layer: int, b: int) -> np.ndarray:
    n = int(0.05 * cfg.T)
    if n == 0:
        return np.zeros(0, dtype=np.int64)
    return np.sort(_rng(cfg, layer, "hh", b).choice(np.arange(1, cfg.T), size=n, replace=False))


def prompt_qkv(cfg: Config, layer: int = 0, batch=None):
    """Prompt Q, K, V as fp32 arrays [len(batch),H,T,D] holding values exact in cfg.dtype."""
    bs = list(range(cfg.B)) if batch is None else list(batch)
    shape = (cfg.H, cfg.T, cfg.D)
    img = image_mask(cfg)
    q = np.empty((len(bs),) + shape, np.float32)
    k = np.empty_like(q)
    v = np.empty_like(q)
    for j, b in enumerate(bs):
        q[j] = _rng(cfg, layer, "q", b).standard_normal(shape, dtype=np.float32)
        kb = _rng(cfg, layer, "k", b).standard_normal(shape, dtype=np.float32)
        v[j] = _rng(cfg, layer, "v", b).standard_normal(shape, dtype=np.float32)
        kb[:, img, :] *= np.float32(0.5)
        kb[:, heavy_hitters(cfg, layer, b), :] *= np.float32(4.0)
        kb[:, 0, :] *= np.float32(8.0)
        k[j] = kb
    return (round_to_dtype(q, cfg.dtype), round_to_dtype(k, cfg.dtype), round_to_dtype(v, cfg.dtype))


def decode_stream(cfg: Config, layer: int, batch=None):
    """All per-step decode vectors of one layer: q, k_new, v_new as fp32 [steps,len(batch),H,D] exact in cfg.dtype."""
    bs = list(range(cfg.B)) if batch is None else list(batch)
    shape = (cfg.decode_steps, cfg.H, cfg.D)
    out = []
    for name in ("dq", "dk", "dv"):
        a = np.empty((cfg.decode_steps, len(bs), cfg.H, cfg.D), np.float32)
        for j, b in enumerate(bs):
            a[:, j] = _rng(cfg, layer, name, b).standard_normal(shape, dtype=np.float32)
        out.append(round_to_dtype(a, cfg.dtype))
    return tuple(out)


def decode_qkv(cfg: Config, layer: int, step: int, batch=None):
    """Per-step q, k_new, v_new as fp32 arrays [len(batch),H,D] exact in cfg.dtype."""
    return tuple(a[step] for a in decode_stream(cfg, layer, batch))


def custom(name: str, *, H: int, D: int, B: int, T: int, dtype: str, gamma=(1, 2), decode_steps=8,
           layers: int = 1, image_frac: float = 0.5, cid: int = 99) -> Config:
    """A config of arbitrary shape for tests (image tokens in the middle of the prompt)."""
    n_img = int(T * image_frac)
    head = min(4, T - n_img)
    layout = (("t", head), ("i", n_img), ("t", T - head - n_img))
    return Config(name, cid, layers, H, D, B, T, dtype, tuple(gamma), decode_steps, layout)
