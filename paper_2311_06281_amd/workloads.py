"""Seeded synthetic inputs for the five benchmark configurations.

This module holds *no* arithmetic of the method: it only draws random numbers with numpy, casts them
to the storage type and describes the call (layout name, flag names).  Both the GPU tests and the CPU
oracle tests take their inputs from here, so the two sides see bit-identical arrays.

The paper uses no dataset; its single experiment sweeps the length of one synthetic sequence
(Sec. 4, Fig. 1).  The shapes below are the linear-RNN / long-sequence shapes the benchmark names.

Recipe (all draws in float64 from ``numpy.random.default_rng([seed, batch_index])``, then rounded to
nearest-even float32; bf16 storage is the nearest-even rounding of that float32):

  cfg 1  B=1  D=1     n=4096   a ~ U(0.5,1)            b ~ U(0,1)       x0 = 1        positive
  cfg 2  B=8  D=1024  n=4096   a = sigmoid(N(2,1))     b ~ N(0,1)       x0 ~ N(0,1)   [B,n,D]
  cfg 3  B=1  D=1     n=2^26   a = exp(N(-1e-7,s=1e-4)) b ~ U(0,1e-3)   x0 = 1        positive
  cfg 4  B=64 D=4096  n=2048   log a = -softplus(N(0,1)) log b ~ N(-1,1) log x0 = 0   [B,D,n], bf16 logs
  cfg 5  B=16 D=2048  n=16384  a ~ U(-1,1)             b ~ N(0,1)       x0 ~ N(0,1)   [B,n,D]

The second parameter of N(., .) is a standard deviation.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Tuple

import numpy as np

BASE_SEED = 20231106


@dataclass(frozen=True)
class Config:
    index: int                  # 1-based, as in the benchmark description
    B: int
    D: int
    n: int
    layout: str                 # "BND" = [B, n, D] channel-contiguous, "BDN" = [B, D, n] sequence-contiguous
    flags: Tuple[str, ...]      # names of the library's flag bits
    signed_tolerance: bool      # which of the two parity tolerances applies
    bf16: bool = False
    log_domain: bool = False
    x0_scalar: bool = False
    name: str = ""

    @property
    def elements(self) -> int:
        return self.B * self.D * self.n

    @property
    def bytes_per_element(self) -> int:
        return 8 if self.bf16 else 12

    def shape(self):
        return (self.B, self.n, self.D) if self.layout == "BND" else (self.B, self.D, self.n)

    def scaled(self, B=None, D=None, n=None) -> "Config":
        """Same distributions and flags at another size (parity tests at oracle-friendly sizes)."""
        return Config(self.index, B or self.B, D or self.D, n or self.n, self.layout, self.flags,
                      self.signed_tolerance, self.bf16, self.log_domain, self.x0_scalar, self.name)


CONFIGS = {
    1: Config(1, 1, 1, 4096, "BDN", ("POSITIVE", "X0_SCALAR"), False, x0_scalar=True,
              name="single sequence n=4096"),
    2: Config(2, 8, 1024, 4096, "BND", (), True, name="linear-RNN batch [8,4096,1024]"),
    3: Config(3, 1, 1, 1 << 26, "BDN", ("POSITIVE", "X0_SCALAR"), False, x0_scalar=True,
              name="one long sequence n=2^26"),
    4: Config(4, 64, 4096, 2048, "BDN", ("LOG_INPUTS", "LOG_OUTPUT", "IN_BF16"), False, bf16=True,
              log_domain=True, name="log-space bf16 inputs [64,4096,2048]"),
    5: Config(5, 16, 2048, 16384, "BND", (), True, name="mixed-sign stress [16,16384,2048]"),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Batch:
    """Inputs for ``nb`` consecutive batch items of a configuration.

    a, b: float32 arrays of shape [nb, n, D] or [nb, D, n] (exactly the stored values; for bf16
          configurations they are the widened bf16 values and a_bits / b_bits hold the uint16 storage).
    x0:   float32 [nb*D] (or [1] when the configuration broadcasts one x0)."""
    a: np.ndarray
    b: np.ndarray
    x0: np.ndarray
    a_bits: np.ndarray = field(default=None)
    b_bits: np.ndarray = field(default=None)


def _draw_one(cfg: Config, rng: np.random.Generator):
    shp = (cfg.n, cfg.D) if cfg.layout == "BND" else (cfg.D, cfg.n)
    i = cfg.index
    if i == 1:
        a = rng.uniform(0.5, 1.0, shp)
        b = rng.uniform(0.0, 1.0, shp)
        x0 = np.ones(cfg.D)
    elif i == 2:
        z = rng.normal(2.0, 1.0, shp)
        a = 1.0 / (1.0 + np.exp(-z))
        b = rng.normal(0.0, 1.0, shp)
        x0 = rng.normal(0.0, 1.0, cfg.D)
    elif i == 3:
        a = np.exp(rng.normal(-1e-7, 1e-4, shp))
        b = rng.uniform(0.0, 1e-3, shp)
        x0 = np.ones(cfg.D)
    elif i == 4:
        z = rng.normal(0.0, 1.0, shp)
        a = -np.logaddexp(0.0, z)          # log a_t = -softplus(z)
        b = rng.normal(-1.0, 1.0, shp)     # log b_t
        x0 = np.zeros(cfg.D)               # log x_0
    elif i == 5:
        a = rng.uniform(-1.0, 1.0, shp)
        b = rng.normal(0.0, 1.0, shp)
        x0 = rng.normal(0.0, 1.0, cfg.D)
    else:
        raise ValueError(f"unknown config {i}")
    return a.astype(np.float32), b.astype(np.float32), x0.astype(np.float32)


def generate(cfg: Config, b_start: int = 0, nb: int | None = None, seed: int | None = None) -> Batch:
    """Inputs for batch items [b_start, b_start+nb) of ``cfg`` (default: all of them).

    Each batch item has its own generator seeded with (seed, item index), so slices of the full
    workload can be produced, uploaded and checked independently."""
    if nb is None:
        nb = cfg.B - b_start
    seed = BASE_SEED + cfg.index if seed is None else seed
    As, Bs, X0s = [], [], []
    for bi in range(b_start, b_start + nb):
        rng = np.random.default_rng([seed, bi])
        a, b, x0 = _draw_one(cfg, rng)
        As.append(a)
        Bs.append(b)
        X0s.append(x0)
    a = np.stack(As)
    b = np.stack(Bs)
    x0 = np.concatenate(X0s)
    if cfg.x0_scalar:
        x0 = x0[:1].copy()
    if cfg.bf16:
        a_bits = f32_to_bf16_bits(a)
        b_bits = f32_to_bf16_bits(b)
        return Batch(bf16_bits_to_f32(a_bits), bf16_bits_to_f32(b_bits), x0, a_bits, b_bits)
    return Batch(a, b, x0)
