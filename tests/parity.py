"""Shared helpers of the parity tests: run a workload through libheinsen on the GPU, run the same
stored inputs through the CPU oracle, and compare with the tolerances the benchmark states.

Tolerances (relative to the float64 sequential oracle):
  positive configurations:  |x_gpu - x_ref| <= 1e-4 |x_ref| + 1e-6
  signed configurations:    |x_gpu - x_ref| <= 1e-3 max_{1<=s<=t} |x_ref,s|
A log output (LOG_OUTPUT) is exponentiated in float64 on both sides and held to the positive bound.
"""
from __future__ import annotations

import numpy as np

import oracle
from paper_2311_06281_amd import workloads

POS_RTOL, POS_ATOL = 1e-4, 1e-6
SIGNED_RTOL = 1e-3


def oracle_layout(cfg):
    return oracle.LAYOUT_BND if cfg.layout == "BND" else oracle.LAYOUT_BDN


def reference(cfg, batch, threads=8):
    """float64 reference from the definition of the recurrence (log x_t for log-domain configs)."""
    if cfg.log_domain:
        return oracle.sequential_log(batch.a, batch.b, batch.x0, layout=oracle_layout(cfg), threads=threads)
    return oracle.sequential(batch.a, batch.b, batch.x0, layout=oracle_layout(cfg), threads=threads)


def violations(cfg, got: np.ndarray, ref: np.ndarray, log_output: bool | None = None):
    """Returns (number of elements outside the tolerance, worst ratio error/bound)."""
    got = np.asarray(got, dtype=np.float64)
    if log_output is None:
        log_output = "LOG_OUTPUT" in cfg.flags
    if log_output:
        with np.errstate(over="ignore"):
            got = np.exp(got)
            ref = np.exp(ref)
    err = np.abs(got - ref)
    if cfg.signed_tolerance:
        axis = 1 if cfg.layout == "BND" else 2
        bound = SIGNED_RTOL * np.maximum.accumulate(np.abs(ref), axis=axis)
    else:
        bound = POS_RTOL * np.abs(ref) + POS_ATOL
    bad = ~(err <= bound)  # NaN counts as a violation
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(bound > 0, err / bound, np.where(err > 0, np.inf, 0.0))
    return int(bad.sum()), float(np.nanmax(ratio)) if ratio.size else 0.0


def to_device(batch, cfg, torch, device="cuda:0"):
    """Uploads the stored inputs.  bf16 storage travels as int16 bit patterns."""
    if cfg.bf16:
        a = torch.from_numpy(batch.a_bits.view(np.int16)).to(device)
        b = torch.from_numpy(batch.b_bits.view(np.int16)).to(device)
    else:
        a = torch.from_numpy(batch.a).to(device)
        b = torch.from_numpy(batch.b).to(device)
    x0 = torch.from_numpy(batch.x0).to(device)
    return a, b, x0


def run_gpu(cfg, batch, torch, hb, B=None, out=None, device="cuda:0"):
    """One heinsen_scan call on torch's current stream; returns the float32 result as numpy."""
    a, b, x0 = to_device(batch, cfg, torch, device)
    B = cfg.B if B is None else B
    if out is None:
        out = torch.empty(a.shape, dtype=torch.float32, device=device)
    hb.heinsen_scan(a, b, x0, out, B, cfg.D, cfg.n, hb.LAYOUTS[cfg.layout], hb.flags_from_names(cfg.flags),
                    torch.cuda.current_stream())
    torch.cuda.synchronize()
    return out.cpu().numpy()
