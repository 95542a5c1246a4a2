"""Parity of the HIP path (through the C ABI) against the CPU oracle, element by element, on the
seeded workloads at oracle-friendly sizes that still span several tiles, groups and a ragged tail."""
import numpy as np
import pytest

from paper_2311_06281_amd import workloads

from parity import reference, run_gpu, violations

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch

    from paper_2311_06281_amd import binding as hb

    assert torch.cuda.is_available(), "these tests need the MI355X"
    hb.load()
    return torch, hb


def _check(cfg, gpu, label):
    torch, hb = gpu
    print(f"[parity] {label}: cfg {cfg.index} B={cfg.B} D={cfg.D} n={cfg.n} {cfg.layout} {cfg.flags}", flush=True)
    batch = workloads.generate(cfg)
    ref = reference(cfg, batch)
    got = run_gpu(cfg, batch, torch, hb)
    nbad, worst = violations(cfg, got, ref)
    print(f"[parity] {label}: worst error/bound = {worst:.3g}", flush=True)
    assert nbad == 0, f"{nbad} of {ref.size} elements outside the tolerance (worst ratio {worst:.3g})"
    return got, ref


# ---- configuration 1: one short positive sequence -------------------------------------------------------
def test_cfg1_single_sequence(gpu):
    _check(workloads.CONFIGS[1], gpu, "cfg1")


@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 511, 512, 513, 1000, 2047, 2048, 2049, 4095, 4097, 9000, 16383, 16385, 40000])
def test_cfg1_lengths(gpu, n):
    _check(workloads.CONFIGS[1].scaled(n=n), gpu, f"cfg1 n={n}")


# ---- configuration 2: [B, n, D], signed b and x0 ----------------------------------------------------------
@pytest.mark.parametrize("B,D,n", [(2, 256, 2500), (1, 192, 1111), (3, 67, 300), (2, 2, 129), (1, 130, 128)])
def test_cfg2_scaled(gpu, B, D, n):
    _check(workloads.CONFIGS[2].scaled(B=B, D=D, n=n), gpu, f"cfg2 {B}x{n}x{D}")


# ---- configuration 3: one long sequence (tiles chained through global memory) -------------------------------
@pytest.mark.parametrize("n", [16384 * 3, 16384 * 75 + 8, 16384 * 300 + 1])  # 6 half tiles; 3 groups of 32 tiles; 10 groups
def test_cfg3_scaled(gpu, n):
    _check(workloads.CONFIGS[3].scaled(n=n), gpu, f"cfg3 n={n}")


# ---- configuration 4: bf16 logs in, log out, [B, D, n] --------------------------------------------------------
@pytest.mark.parametrize("B,D,n", [(2, 64, 2048), (1, 33, 1000), (2, 5, 999), (1, 7, 100), (1, 3, 6000), (1, 2, 40000), (1, 1, 16384 * 20 + 8)])
def test_cfg4_scaled(gpu, B, D, n):
    _check(workloads.CONFIGS[4].scaled(B=B, D=D, n=n), gpu, f"cfg4 {B}x{D}x{n}")


# ---- configuration 5: everything signed ------------------------------------------------------------------------
@pytest.mark.parametrize("B,D,n", [(2, 130, 3000), (1, 64, 16384), (1, 3, 500)])
def test_cfg5_scaled(gpu, B, D, n):
    _check(workloads.CONFIGS[5].scaled(B=B, D=D, n=n), gpu, f"cfg5 {B}x{n}x{D}")


def test_cfg5_distribution_in_sequence_contiguous_layout(gpu):
    # the signed path of the [B, D, n] kernels (no benchmark configuration exercises it)
    base = workloads.CONFIGS[5]
    for D, n in ((4, 2048), (3, 777), (2, 16384 * 5 + 3)):
        cfg = workloads.Config(5, 2, D, n, "BDN", (), True, name="signed rows")
        _check(cfg, gpu, f"cfg5-as-rows {D}x{n}")


def test_results_are_bit_reproducible(gpu):
    torch, hb = gpu
    for cfg in (workloads.CONFIGS[5].scaled(B=2, D=256, n=4096), workloads.CONFIGS[3].scaled(n=16384 * 300)):
        batch = workloads.generate(cfg)
        first = run_gpu(cfg, batch, torch, hb)
        for _ in range(25):
            again = run_gpu(cfg, batch, torch, hb)
            assert np.array_equal(first.view(np.uint32), again.view(np.uint32))
