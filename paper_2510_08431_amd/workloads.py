"""Seeded synthetic inputs for the attention-JVP workloads.

Holds no attention arithmetic: only shapes, distributions and row sampling.
Both the test oracle and the HIP path are fed from here, so neither needs the other.

Every (config, batch, head) has its own torch CPU generator seed, so one head of a
long config can be regenerated alone (the CPU oracle evaluates heads one at a time).
Values are drawn in fp32 on the CPU and then cast to the config's dtype.
"""
from dataclasses import dataclass
import math

import numpy as np
import torch


@dataclass(frozen=True)
class AttnJvpConfig:
    idx: int
    name: str
    B: int
    H: int
    Lq: int
    Lkv: int
    d: int
    dtype: str            # "fp32" | "bf16"
    qk_gain: float        # multiplies Q and K after drawing
    rms_norm_qk: bool     # divide each Q/K row by its RMS over d (unit-gain QK-norm)
    tangent_std: float
    zero_tk_tv: bool      # cross-attention on time-independent conditioning

    @property
    def scale(self):
        return 1.0 / math.sqrt(self.d)

    @property
    def flops(self):
        """Six contractions of 2*Lq*Lkv*d flops each, per head."""
        return 12.0 * self.B * self.H * self.Lq * self.Lkv * self.d

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16


CONFIGS = {
    1: AttnJvpConfig(1, "tiny-self-fp32", 1, 2, 256, 256, 64, "fp32", 1.0, False, 1.0, False),
    2: AttnJvpConfig(2, "image-dit-self-bf16", 2, 16, 4096, 4096, 128, "bf16", 1.0, True, 0.5, False),
    3: AttnJvpConfig(3, "video-dit-self-bf16", 1, 12, 32760, 32760, 128, "bf16", 1.0, False, 0.5, False),
    4: AttnJvpConfig(4, "video-dit-cross-bf16", 1, 12, 32760, 512, 128, "bf16", 1.0, False, 0.5, True),
    # logits scale*q.k have variance d*g^4/d = g^4; std 8 needs g = 8**0.5
    5: AttnJvpConfig(5, "video-14b-720p-stress-bf16", 1, 40, 75600, 75600, 128, "bf16",
                     math.sqrt(8.0), False, 1.0, False),
    # not one of the five named configurations: the video self-attention shape at head dimension 64 with the same
    # model width (24 heads of 64 instead of 12 of 128), for measuring the d = 64 instantiation of the kernels
    6: AttnJvpConfig(6, "video-dit-self-d64-bf16", 1, 24, 32760, 32760, 64, "bf16", 1.0, False, 0.5, False),
}

_TENSORS = ("q", "k", "v", "tq", "tk", "tv")


def _seed(cfg, b, h, t):
    return ((1000 + cfg.idx) * 1_000_003 + (b * cfg.H + h) * 8 + t) & 0x7FFFFFFF


def make_head(cfg, b, h):
    """The six [L, d] CPU tensors of one (batch, head), in the config's dtype."""
    out = {}
    for t, name in enumerate(_TENSORS):
        L = cfg.Lq if name in ("q", "tq") else cfg.Lkv
        if cfg.zero_tk_tv and name in ("tk", "tv"):
            out[name] = torch.zeros(L, cfg.d, dtype=cfg.torch_dtype)
            continue
        g = torch.Generator(device="cpu")
        g.manual_seed(_seed(cfg, b, h, t))
        x = torch.randn(L, cfg.d, generator=g, dtype=torch.float32)
        if name in ("q", "k"):
            if cfg.rms_norm_qk:
                x = x / x.pow(2).mean(dim=-1, keepdim=True).sqrt()
            x = x * cfg.qk_gain
        elif name in ("tq", "tk", "tv"):
            x = x * cfg.tangent_std
        out[name] = x.to(cfg.torch_dtype)
    return out


def make_inputs(cfg, device="cpu"):
    """The six [B, H, L, d] tensors, contiguous, on `device`, built head by head."""
    out = {}
    for name in _TENSORS:
        L = cfg.Lq if name in ("q", "tq") else cfg.Lkv
        out[name] = torch.empty(cfg.B, cfg.H, L, cfg.d, dtype=cfg.torch_dtype, device=device)
    for b in range(cfg.B):
        for h in range(cfg.H):
            head = make_head(cfg, b, h)
            for name in _TENSORS:
                out[name][b, h].copy_(head[name])
    return out


def sample_rows(cfg, n_random, tile=128, seed=0):
    """Query rows to check on a long config: tile edges, the ragged tail and random rows."""
    Lq = cfg.Lq
    last_full = (Lq // tile) * tile
    fixed = [0, 1, tile - 1, tile, last_full - 1, min(last_full, Lq - 1), Lq - 2, Lq - 1]
    rng = np.random.default_rng(77_000 + 31 * cfg.idx + seed)
    rnd = rng.integers(0, Lq, size=n_random).tolist()
    rows = sorted({int(r) for r in fixed + rnd if 0 <= r < Lq})
    return np.asarray(rows, dtype=np.int64)
