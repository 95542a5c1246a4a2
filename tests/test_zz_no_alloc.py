"""heinsen_scan_static (the entry point that allocates nothing) against heinsen_scan, through the C ABI.

Both run the same kernels with the same fixed fold order, so the results must agree bit for bit -- which
is inside every tolerance the parity tests hold heinsen_scan to.  The static scratch keeps the previous
call's contents, so each case makes two calls in a row, the second on a smaller input."""
import numpy as np
import pytest

from paper_2311_06281_amd import workloads

from parity import to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch

    from paper_2311_06281_amd import binding as hb

    assert torch.cuda.is_available(), "these tests need the MI355X"
    hb.load()
    return torch, hb


def _both(cfg, torch, hb):
    batch = workloads.generate(cfg)
    a, b, x0 = to_device(batch, cfg, torch)
    layout, flags = hb.LAYOUTS[cfg.layout], hb.flags_from_names(cfg.flags)
    stream = torch.cuda.current_stream()
    want = torch.full(a.shape, float("nan"), dtype=torch.float32, device=a.device)
    got = torch.full(a.shape, float("nan"), dtype=torch.float32, device=a.device)
    hb.heinsen_scan(a, b, x0, want, cfg.B, cfg.D, cfg.n, layout, flags, stream)
    hb.heinsen_scan_static(a, b, x0, got, cfg.B, cfg.D, cfg.n, layout, flags, stream)
    torch.cuda.synchronize()
    return got.cpu().numpy(), want.cpu().numpy()


CASES = [
    # [B, n, D]: tiles chained through carry records; then fewer, shorter columns
    (workloads.CONFIGS[5].scaled(B=2, D=192, n=5000), workloads.CONFIGS[5].scaled(B=1, D=70, n=1300)),
    # one long row: two-level carry tree and a float64 super-block state; then a shorter row
    (workloads.CONFIGS[3].scaled(n=16384 * 1100 + 12), workloads.CONFIGS[3].scaled(n=16384 * 40 + 3)),
    # few columns: the second carry level of the [B, n, D] kernel; then a shape that needs no scratch at all
    (workloads.CONFIGS[2].scaled(B=1, D=64, n=40000), workloads.CONFIGS[2].scaled(B=2, D=128, n=64)),
]


@pytest.mark.parametrize("first,second", CASES)
def test_static_entry_point_matches_the_allocating_one(gpu, first, second):
    torch, hb = gpu
    for cfg in (first, second):
        print(f"[no-alloc] cfg {cfg.index} B={cfg.B} D={cfg.D} n={cfg.n} {cfg.layout}", flush=True)
        got, want = _both(cfg, torch, hb)
        assert np.isfinite(want).all()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_static_entry_point_with_narrower_tiles_than_the_allocating_one(gpu):
    """[16, 12288, 2048]: heinsen_scan takes its wide tiles (carries: 63 MiB), the fixed 48 MiB array only
    holds the narrower ones (31 MiB).  Both are the same method with different float32 rounding: the
    result is held to the signed tolerance with the allocating entry point's output as the reference."""
    torch, hb = gpu
    from parity import violations

    cfg = workloads.CONFIGS[5].scaled(n=12288)
    batch = workloads.generate(cfg, 0, 1)
    rep = lambda x: torch.from_numpy(x).to("cuda:0").repeat((cfg.B,) + (1,) * (x.ndim - 1)).contiguous()
    a, b = rep(batch.a), rep(batch.b)
    x0 = torch.from_numpy(batch.x0).to("cuda:0").repeat(cfg.B).contiguous()
    layout, flags = hb.LAYOUTS[cfg.layout], hb.flags_from_names(cfg.flags)
    stream = torch.cuda.current_stream()
    want = torch.empty_like(a)
    got = torch.empty_like(a)
    print(f"[no-alloc] cfg5 distribution B={cfg.B}: wide tiles against narrow tiles", flush=True)
    hb.heinsen_scan(a, b, x0, want, cfg.B, cfg.D, cfg.n, layout, flags, stream)
    hb.heinsen_scan_static(a, b, x0, got, cfg.B, cfg.D, cfg.n, layout, flags, stream)
    torch.cuda.synchronize()
    one = cfg.scaled(B=1)
    for bi in (0, cfg.B - 1):
        nbad, worst = violations(one, got[bi:bi + 1].cpu().numpy(), want[bi:bi + 1].cpu().numpy().astype(np.float64))
        print(f"[no-alloc] batch item {bi}: worst difference/bound {worst:.3g}", flush=True)
        assert nbad == 0


def test_static_entry_point_refuses_what_does_not_fit(gpu):
    torch, hb = gpu
    # [32, 32768, 2048] needs about 150 MiB of carry records; the pointers are never used
    dummy = torch.zeros(16, dtype=torch.float32, device="cuda:0")
    st = hb.heinsen_scan_static_status(dummy, dummy, dummy, dummy, 32, 2048, 32768, hb.HEINSEN_LAYOUT_BND, 0,
                                       torch.cuda.current_stream())
    assert st == hb.HEINSEN_ERR_SCRATCH_LIMIT
    assert "scratch" in hb.heinsen_status_string(st)
    torch.cuda.synchronize()
