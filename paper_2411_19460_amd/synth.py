"""Seeded synthetic inputs for one SSD layer (and for a stack of them).

This module holds no arithmetic of the method itself: it only draws tensors
with the shapes and value ranges of a Mamba-2 layer (the layer shapes are the
ones the paper's memory-constant table decodes to: H = 2*d_model/64 heads of
P = 64 channels, N = 128 states, one B/C group) and rounds them to the storage
dtype once.  Both the fp64 oracle and the HIP path consume the rounded values,
so input quantisation is never counted as error.

Recipe (per layer, drawn in this fixed order from one generator):
    x  ~ N(0,1)                      [B, L, H, P]
    u  ~ U(-7, -2.3); dt = log(1+exp(u))   [B, L, H]     (dt in [9.1e-4, 0.0955])
    A  = -exp(U(0, ln 16))           [H]   fp32          (A in [-16, -1])
    Bm ~ N(0,1)/sqrt(N)              [B, L, G, N]
    Cm ~ N(0,1)/sqrt(N)              [B, L, G, N]
    D  ~ N(0,1)                      [H]   fp32
    dy ~ N(0,1)                      [B, L, H, P]
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import numpy as np

BASE_SEED = 241119460


@dataclass(frozen=True)
class SSDConfig:
    name: str
    dtype: str          # "f32" or "bf16": storage type of x, dt, B, C, y and their gradients
    batch: int
    seqlen: int
    nheads: int
    headdim: int
    dstate: int
    ngroups: int
    chunk: int
    segment: int
    nlayers: int = 1
    index: int = 0      # position in the benchmark's config list (enters the seed)

    def seed(self, layer: int = 0) -> int:
        return BASE_SEED + 1000 * self.index + layer

    def scaled(self, **kw) -> "SSDConfig":
        return replace(self, **kw)


CONFIGS = [
    SSDConfig("c0_tiny_f32", "f32", 1, 512, 4, 16, 16, 1, 64, 256, index=0),
    SSDConfig("c1_130m_bf16", "bf16", 1, 8192, 24, 64, 128, 1, 256, 2048, index=1),
    SSDConfig("c2_2p7b_64k_bf16", "bf16", 1, 65536, 80, 64, 128, 1, 256, 4096, index=2),
    SSDConfig("c3_2p7b_1m_bf16", "bf16", 1, 1048576, 80, 64, 128, 1, 256, 16384, index=3),
    SSDConfig("c4_stack16_256k_bf16", "bf16", 1, 262144, 80, 64, 128, 1, 256, 8192, nlayers=16, index=4),
]


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 values that are already bf16-representable -> uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    a = a.astype(np.float32)
    return round_bf16(a) if dtype == "bf16" else a


def make_layer_inputs(cfg: SSDConfig, layer: int = 0, with_states: bool = False) -> dict:
    """Host (numpy) draw.  Every array is fp32 and already rounded to cfg.dtype."""
    rng = np.random.default_rng(cfg.seed(layer))
    Bt, L, H, P, G, N = cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.ngroups, cfg.dstate
    x = rng.standard_normal((Bt, L, H, P), dtype=np.float32)
    u = rng.uniform(-7.0, -2.3, (Bt, L, H))
    dt = np.log1p(np.exp(u))
    A = -np.exp(rng.uniform(0.0, math.log(16.0), (H,)))
    Bm = rng.standard_normal((Bt, L, G, N), dtype=np.float32) / math.sqrt(N)
    Cm = rng.standard_normal((Bt, L, G, N), dtype=np.float32) / math.sqrt(N)
    D = rng.standard_normal((H,), dtype=np.float32)
    dy = rng.standard_normal((Bt, L, H, P), dtype=np.float32)
    out = {
        "x": _store(x, cfg.dtype), "dt": _store(dt, cfg.dtype), "A": A.astype(np.float32),
        "B": _store(Bm, cfg.dtype), "C": _store(Cm, cfg.dtype), "D": D.astype(np.float32),
        "dy": _store(dy, cfg.dtype),
    }
    if with_states:
        out["init_state"] = rng.standard_normal((Bt, H, P, N), dtype=np.float32)
        out["dfinal_state"] = rng.standard_normal((Bt, H, P, N), dtype=np.float32)
    return out


def make_layer_inputs_device(cfg: SSDConfig, device, layer: int = 0, with_dy: bool = True) -> dict:
    """Device draw for shapes too large to draw on the host.  Returns torch tensors
    in the storage dtype (A, D fp32).  The stream of numbers differs from the host
    draw; whoever needs the values on the host copies back what it reads."""
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(cfg.seed(layer))
    Bt, L, H, P, G, N = cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.ngroups, cfg.dstate
    td = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32

    def normal(shape, scale=1.0):
        t = torch.empty(shape, device=device, dtype=td)
        # drawn slice by slice so the fp32 temporaries stay small next to the tensor itself
        step = max(1, (1 << 26) // max(1, int(np.prod(shape[2:]))))
        for s in range(0, shape[1], step):
            e = min(shape[1], s + step)
            tmp = torch.randn((shape[0], e - s) + tuple(shape[2:]), device=device, generator=g,
                              dtype=torch.float32)
            t[:, s:e] = (tmp * scale).to(td)
        return t

    x = normal((Bt, L, H, P))
    u = torch.rand((Bt, L, H), device=device, generator=g, dtype=torch.float32) * (7.0 - 2.3) - 7.0
    dt = torch.log1p(torch.exp(u)).to(td)
    A = -torch.exp(torch.rand((H,), device=device, generator=g, dtype=torch.float32) * math.log(16.0))
    Bm = normal((Bt, L, G, N), 1.0 / math.sqrt(N))
    Cm = normal((Bt, L, G, N), 1.0 / math.sqrt(N))
    D = torch.randn((H,), device=device, generator=g, dtype=torch.float32)
    out = {"x": x, "dt": dt, "A": A, "B": Bm, "C": Cm, "D": D}
    if with_dy:
        out["dy"] = normal((Bt, L, H, P))
    return out
