"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

Configurations 1-3 are generated and checked in full.  For the 5e8-element configurations 4 and 5 a
few batch items are generated and repeated to the full batch (generating all of them on the host
takes minutes); the generated items are checked against the oracle element by element and every
repeated item must equal its original bit for bit (sequences are independent)."""
import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

from paper_2311_06281_amd import workloads  # noqa: E402

from parity import reference, violations  # noqa: E402

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch

    from paper_2311_06281_amd import binding as hb

    assert torch.cuda.is_available()
    hb.load()
    return torch, hb


@pytest.mark.parametrize("idx", [1, 2, 3])
def test_full_size_generated_in_full(gpu, idx):
    torch, hb = gpu
    import bench

    cfg = workloads.CONFIGS[idx]
    print(f"[full] cfg{idx} {cfg.shape()}", flush=True)
    a, b, x0, out = bench.device_inputs(cfg, torch, distinct=cfg.B)
    hb.heinsen_scan(a, b, x0, out, cfg.B, cfg.D, cfg.n, hb.LAYOUTS[cfg.layout], hb.flags_from_names(cfg.flags),
                    torch.cuda.current_stream())
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    batch = workloads.generate(cfg)
    ref = reference(cfg, batch, threads=16)
    nbad, worst = violations(cfg, got, ref)
    print(f"[full] cfg{idx}: worst error/bound {worst:.3g}", flush=True)
    assert nbad == 0, f"{nbad} of {ref.size} outside the tolerance (worst {worst:.3g})"


@pytest.mark.parametrize("idx,distinct", [(4, 3), (5, 2)])
def test_full_size_repeated_items(gpu, idx, distinct):
    torch, hb = gpu
    import bench

    cfg = workloads.CONFIGS[idx]
    print(f"[full] cfg{idx} {cfg.shape()} with {distinct} distinct batch items", flush=True)
    a, b, x0, out = bench.device_inputs(cfg, torch, distinct=distinct)
    hb.heinsen_scan(a, b, x0, out, cfg.B, cfg.D, cfg.n, hb.LAYOUTS[cfg.layout], hb.flags_from_names(cfg.flags),
                    torch.cuda.current_stream())
    torch.cuda.synchronize()
    # replicas equal their originals bit for bit
    bits = out.view(torch.int32)
    for bi in range(distinct, cfg.B):
        assert torch.equal(bits[bi], bits[bi % distinct]), f"batch item {bi} differs from its original"
    got = out[:distinct].cpu().numpy()
    del a, b, x0, out, bits
    torch.cuda.empty_cache()
    sub = cfg.scaled(B=distinct)
    batch = workloads.generate(cfg, 0, distinct)
    ref = reference(sub, batch, threads=16)
    nbad, worst = violations(sub, got, ref)
    print(f"[full] cfg{idx}: worst error/bound {worst:.3g}", flush=True)
    assert nbad == 0, f"{nbad} of {ref.size} outside the tolerance (worst {worst:.3g})"


def test_longer_than_one_super_block(gpu):
    """One sequence a little longer than 4096 tiles (four super-blocks of 1024): the float64 state handed
    from one super-block of tiles to the next is the only carry that forms a chain."""
    torch, hb = gpu
    import bench

    cfg = workloads.CONFIGS[3].scaled(n=(1 << 26) + 16384 * 3 + 5)
    print(f"[full] cfg3 distribution, n={cfg.n}", flush=True)
    a, b, x0, out = bench.device_inputs(cfg, torch, distinct=1)
    hb.heinsen_scan(a, b, x0, out, cfg.B, cfg.D, cfg.n, hb.LAYOUTS[cfg.layout], hb.flags_from_names(cfg.flags),
                    torch.cuda.current_stream())
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    ref = reference(cfg, workloads.generate(cfg), threads=1)
    nbad, worst = violations(cfg, got, ref)
    print(f"[full] worst error/bound {worst:.3g}", flush=True)
    assert nbad == 0


@pytest.mark.parametrize("idx", [2, 3])
@pytest.mark.parametrize("mode", ["complex_log", "linear"])
def test_full_size_other_outputs(gpu, idx, mode):
    """The complex-logarithm output and the linear-domain comparison path at full size (configuration 2's
    data for the [B,n,D] kernel, configuration 3's for the chained tiles), held to the configuration's bound."""
    torch, hb = gpu
    import bench

    cfg = workloads.CONFIGS[idx]
    print(f"[full] cfg{idx} {cfg.shape()} {mode}", flush=True)
    a, b, x0, out = bench.device_inputs(cfg, torch, distinct=cfg.B)
    flags = hb.flags_from_names(cfg.flags)
    if mode == "complex_log":
        flags = (flags & ~hb.HEINSEN_POSITIVE) | hb.HEINSEN_LOG_OUTPUT | hb.HEINSEN_OUT_COMPLEX
        out = torch.empty(tuple(out.shape) + (2,), dtype=torch.float32, device=out.device)
    else:
        flags |= hb.HEINSEN_LINEAR
    hb.heinsen_scan(a, b, x0, out, cfg.B, cfg.D, cfg.n, hb.LAYOUTS[cfg.layout], flags, torch.cuda.current_stream())
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    if mode == "complex_log":
        assert np.all((got[..., 1] == 0) | (got[..., 1] == np.float32(np.pi)))
        with np.errstate(over="ignore"):
            got = np.exp(got[..., 0].astype(np.float64)) * np.where(got[..., 1] == 0, 1.0, -1.0)
    ref = reference(cfg, workloads.generate(cfg), threads=16)
    nbad, worst = violations(cfg, got, ref, log_output=False)
    print(f"[full] cfg{idx} {mode}: worst error/bound {worst:.3g}", flush=True)
    if mode == "linear" and idx == 3:
        # The comparison path is not expected to meet configuration 3's bound, and this is what it is there
        # to show: with a_t within 1e-4 of 1, a float32 product of many a_t carries the 6e-8 spacing of
        # floats around 1 into the large running state at every fold, while a float32 sum of log a_t keeps
        # the relative precision of numbers near 0.  Plain float32 arithmetic in the same blocked order
        # gives the same figures on the CPU (3e-5 at n = 2^13, growing to a few percent at 2^26), so the
        # test only holds the linear path to "a few percent" here.
        rel = np.abs(got - ref) / np.abs(ref)
        print(f"[full] cfg3 linear: max relative error {rel.max():.3g}", flush=True)
        assert rel.max() < 0.2
        return
    assert nbad == 0, f"{nbad} of {ref.size} outside the tolerance (worst {worst:.3g})"


@pytest.mark.parametrize("D,n", [(256, 1 << 19), (64, 1 << 20), (1024, 1 << 16)])
def test_long_sequences_of_few_columns(gpu, D, n):
    """[B,n,D] with 4, 1 and 16 columns of 64 channels and thousands of tiles along time: the launches whose
    carry structure has longer groups and (for 4 and 1 columns) a second level, at a length where every
    level is many records deep.  Configuration 2's distribution, generated and checked in full."""
    torch, hb = gpu
    import bench

    cfg = workloads.CONFIGS[2].scaled(B=1, D=D, n=n)
    print(f"[full] cfg2 distribution {cfg.shape()}", flush=True)
    a, b, x0, out = bench.device_inputs(cfg, torch, distinct=1)
    hb.heinsen_scan(a, b, x0, out, cfg.B, cfg.D, cfg.n, hb.LAYOUTS[cfg.layout], hb.flags_from_names(cfg.flags),
                    torch.cuda.current_stream())
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    ref = reference(cfg, workloads.generate(cfg), threads=16)
    nbad, worst = violations(cfg, got, ref)
    print(f"[full] worst error/bound {worst:.3g}", flush=True)
    assert nbad == 0, f"{nbad} of {ref.size} outside the tolerance (worst {worst:.3g})"


@pytest.mark.parametrize("B,D,n", [(1, 64, 1 << 22), (1, 64, 1 << 23), (4, 64, 1 << 20), (2, 8, 1 << 21), (2, 1024, 1 << 17)])
def test_long_slowly_decaying_sequences_channel_contiguous(gpu, B, D, n):
    """[B,n,D] with coefficients within 1e-4 of 1 (configuration 3's distribution) over millions of steps,
    held to the positive tolerance of the definition (1e-4 relative): the state that travels from one group
    of tiles to the next goes through n/1024 .. n/16384 links (one column: two carry levels of 8 x 8 tiles;
    four columns: 4 x 4; narrow channels packed side by side; 32 columns: plain groups of eight) and has to
    be carried in float64 to stay inside the bound.  Generated and checked in full against the float64
    sequential oracle."""
    torch, hb = gpu
    import bench

    cfg = workloads.Config(3, B, D, n, "BND", ("POSITIVE",), False, name="slowly decaying, channel-contiguous")
    print(f"[full] cfg3 distribution in [B,n,D] {cfg.shape()}", flush=True)
    a, b, x0, out = bench.device_inputs(cfg, torch, distinct=B)
    hb.heinsen_scan(a, b, x0, out, cfg.B, cfg.D, cfg.n, hb.LAYOUTS[cfg.layout], hb.flags_from_names(cfg.flags),
                    torch.cuda.current_stream())
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    del a, b, x0, out
    torch.cuda.empty_cache()
    ref = reference(cfg, workloads.generate(cfg), threads=16)
    rel = np.abs(got - ref) / np.abs(ref)
    print(f"[full] max relative error {rel.max():.3g} (bound 1e-4)", flush=True)
    nbad, worst = violations(cfg, got, ref)
    print(f"[full] worst error/bound {worst:.3g}", flush=True)
    assert nbad == 0, f"{nbad} of {ref.size} outside the tolerance (worst {worst:.3g})"
