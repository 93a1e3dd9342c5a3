"""Seeded synthetic inputs for the SSD layer core.

This module serves both the GPU library's callers and the CPU oracle's tests.  It holds
none of the method's arithmetic: it only draws random tensors with the shapes and value
distributions of the five benchmark configurations and rounds them to the I/O dtype.

Recipe (one ``torch.Generator`` per (seed, layer), fixed draw order x, dt-noise, A, B, C, D):

* ``x  ~ N(0, 1)``                                   ``(batch, T, H, P)``
* ``dt = clamp(softplus(0.5 z + bias), 1e-3, 1e-1)``, ``z ~ N(0, 1)``, ``(batch, T, H)`` fp32,
  ``bias = log(expm1(1e-2))`` so the median step is 1e-2 and the clamp bites only in the
  far tails.  The softplus / clamp that a Mamba-2 block applies to its raw step-size
  projection is done here, outside the library: the library receives the final positive dt.
* ``A  = -exp(U(log 1, log 16))``                    ``(H)`` fp32, already negative
* ``B, C ~ 0.25 N(0, 1)``                            ``(batch, T, G, N)``
* ``D  ~ N(0, 1)``                                   ``(H)`` fp32

bf16 tensors are rounded once (round-to-nearest-even, ``Tensor.to(torch.bfloat16)``); both
the oracle and the GPU path consume the rounded values.  With ``device="cuda"`` the draws
come from torch's device generator (same distributions, different numbers) so that the
multi-gigabyte decode workload can be produced in place.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import torch

DT_MIN = 1e-3
DT_MAX = 1e-1
DT_BIAS = math.log(math.expm1(1e-2))
BC_SCALE = 0.25
A_MAX = 16.0


@dataclass(frozen=True)
class SSDConfig:
    name: str
    batch: int
    seqlen: int
    nheads: int
    headdim: int
    dstate: int
    ngroups: int
    chunk: int
    io_dtype: str  # "f32" or "bf16": dtype of x, B, C, y.  dt, A, D and the state are fp32.
    nlayers: int = 1
    decode_steps: int = 0

    @property
    def torch_io_dtype(self):
        return torch.float32 if self.io_dtype == "f32" else torch.bfloat16

    def with_(self, **kw) -> "SSDConfig":
        return replace(self, **kw)


# The five benchmark configurations (shapes only; the values are synthetic).
CONFIGS = {
    "c0_tiny_f32": SSDConfig("c0_tiny_f32", 1, 512, 4, 32, 16, 1, 64, "f32"),
    "c1_130m": SSDConfig("c1_130m", 1, 2048, 24, 64, 128, 1, 256, "bf16"),
    "c2_780m_b8": SSDConfig("c2_780m_b8", 8, 4096, 48, 64, 128, 1, 256, "bf16"),
    "c3_2p7b_long": SSDConfig("c3_2p7b_long", 1, 16384, 80, 64, 128, 1, 256, "bf16"),
    "c4_decode_b1": SSDConfig("c4_decode_b1", 1, 2048, 80, 64, 128, 1, 256, "bf16", nlayers=64,
                              decode_steps=1024),
    "c4_decode_b16": SSDConfig("c4_decode_b16", 16, 2048, 80, 64, 128, 1, 256, "bf16", nlayers=64,
                               decode_steps=1024),
}


def _generator(seed: int, layer: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + int(layer) * 7919 + 12345) & 0x7FFFFFFFFFFFFFFF)
    return g


def _randn(shape, g, device):
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32)


def _dt_from_noise(z: torch.Tensor) -> torch.Tensor:
    return torch.nn.functional.softplus(0.5 * z + DT_BIAS).clamp_(DT_MIN, DT_MAX)


def make_head_params(cfg: SSDConfig, g: torch.Generator, device):
    u = torch.rand((cfg.nheads,), generator=g, device=device, dtype=torch.float32)
    return -torch.exp(u * math.log(A_MAX))


def make_prefill_inputs(cfg: SSDConfig, seed: int = 0, layer: int = 0, device="cpu") -> dict:
    """Tensors for one ``ssd_prefill`` call: x, dt, A, B, C, D (see module docstring)."""
    g = _generator(seed, layer, device)
    io = cfg.torch_io_dtype
    Bt, T, H, P, N, G = cfg.batch, cfg.seqlen, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups
    x = _randn((Bt, T, H, P), g, device).to(io)
    dt = _dt_from_noise(_randn((Bt, T, H), g, device))
    A = make_head_params(cfg, g, device)
    B = (BC_SCALE * _randn((Bt, T, G, N), g, device)).to(io)
    C = (BC_SCALE * _randn((Bt, T, G, N), g, device)).to(io)
    D = _randn((H,), g, device)
    return {"x": x, "dt": dt, "A": A, "B": B, "C": C, "D": D}


def make_decode_inputs(cfg: SSDConfig, steps: int, seed: int = 0, layer: int = 0, device="cpu") -> dict:
    """Per-step tensors for ``steps`` decode steps of one layer, stacked on a leading step
    axis: x ``(steps, batch, H, P)``, dt ``(steps, batch, H)``, B, C ``(steps, batch, G, N)``.
    A and D are the layer's constants and must come from :func:`make_prefill_inputs`."""
    g = _generator(seed + 1, layer, device)
    io = cfg.torch_io_dtype
    Bt, H, P, N, G = cfg.batch, cfg.nheads, cfg.headdim, cfg.dstate, cfg.ngroups
    x = _randn((steps, Bt, H, P), g, device).to(io)
    dt = _dt_from_noise(_randn((steps, Bt, H), g, device))
    B = (BC_SCALE * _randn((steps, Bt, G, N), g, device)).to(io)
    C = (BC_SCALE * _randn((steps, Bt, G, N), g, device)).to(io)
    return {"x": x, "dt": dt, "B": B, "C": C}


def make_state(cfg: SSDConfig, seed: int = 0, layer: int = 0, device="cpu", scale: float = 1.0):
    """A random fp32 state ``(batch, H, P, N)`` for tests that start from a given h0."""
    g = _generator(seed + 2, layer, device)
    return scale * _randn((cfg.batch, cfg.nheads, cfg.headdim, cfg.dstate), g, device)
