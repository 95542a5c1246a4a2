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
    """One sequence a little longer than 4096 tiles: the float64 state handed from one super-block of
    tiles to the next is the only carry that forms a chain, and only such lengths exercise it."""
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
