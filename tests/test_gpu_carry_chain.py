"""The machinery between tiles: launch counter kept on the device (also when it comes round), the bounded
wait for carry records with its error report, per-tile time stamps.  Every kernel here ends normally: the
"lost record" is a tile that the library is told not to publish, with a small poll limit."""
import numpy as np
import pytest

from paper_2311_06281_amd import workloads

from parity import to_device

pytestmark = pytest.mark.gpu

LAST_EPOCH = (1 << 30) - 1


@pytest.fixture(scope="module")
def gpu():
    import torch

    from paper_2311_06281_amd import binding as hb

    assert torch.cuda.is_available(), "these tests need the MI355X"
    hb.load()
    return torch, hb


def _run(cfg, dev, torch, hb, static=False):
    a, b, x0 = dev
    out = torch.full(a.shape, float("nan"), dtype=torch.float32, device=a.device)
    fn = hb.heinsen_scan_static if static else hb.heinsen_scan
    fn(a, b, x0, out, cfg.B, cfg.D, cfg.n, hb.LAYOUTS[cfg.layout], hb.flags_from_names(cfg.flags), torch.cuda.current_stream())
    torch.cuda.synchronize()
    return out.cpu().numpy()


CHAINED = [
    workloads.CONFIGS[2].scaled(B=1, D=128, n=2048),   # [B, n, D]: 2 columns x 8 tiles, two groups
    workloads.CONFIGS[2].scaled(B=1, D=64, n=40000),   # one column: second carry level
    workloads.CONFIGS[3].scaled(n=16384 * 40 + 5),     # one row of 81 half tiles (8192 steps): two-level tree
    workloads.CONFIGS[3].scaled(n=16384 * 140 + 5),    # one row of 141 full tiles (16384 steps)
]


@pytest.mark.parametrize("cfg", CHAINED)
@pytest.mark.parametrize("static", [False, True])
def test_launch_counter_comes_round(gpu, cfg, static):
    torch, hb = gpu
    dev = to_device(workloads.generate(cfg), cfg, torch)
    want = _run(cfg, dev, torch, hb, static)  # also makes sure the scratch exists
    assert np.isfinite(want).all()
    stream = torch.cuda.current_stream()
    hb.heinsen_test_carry(0, 0xFFFFFFFF, LAST_EPOCH - 1, stream)
    # epochs 2^30 - 2, 2^30 - 1 (its last workgroup clears the records), 1, 2
    for i in range(4):
        print(f"[epoch] launch {i} after the jump, cfg{cfg.index} n={cfg.n} static={static}", flush=True)
        got = _run(cfg, dev, torch, hb, static)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), f"launch {i} after the jump differs"
    assert hb.heinsen_check(stream) == hb.HEINSEN_OK


@pytest.mark.parametrize("cfg,drop,bad_from_tile", [
    # tile 2 = chunk 1 of column 0 never publishes: chunks 2 and 3 of its group wait in vain
    (CHAINED[0], 2, 2),
    # tile 3 of the row never publishes: every later tile folds it
    (CHAINED[2], 3, 4),
    (CHAINED[3], 3, 4),
])
def test_lost_carry_ends_in_nan_and_a_report(gpu, cfg, drop, bad_from_tile):
    torch, hb = gpu
    stream = torch.cuda.current_stream()
    steps = hb.heinsen_tile_shape(cfg.B, cfg.D, cfg.n, hb.LAYOUTS[cfg.layout], hb.flags_from_names(cfg.flags))[1]
    assert steps == {0: 256, 2: 8192, 3: 16384}[CHAINED.index(cfg)]
    first_bad = bad_from_tile * steps
    dev = to_device(workloads.generate(cfg), cfg, torch)
    want = _run(cfg, dev, torch, hb)
    assert hb.heinsen_check(stream) == hb.HEINSEN_OK
    try:
        hb.heinsen_test_carry(20000, drop, 0, stream)  # about 20 ms of polling, then give up
        print(f"[lost] cfg{cfg.index}: tile {drop} does not publish", flush=True)
        got = _run(cfg, dev, torch, hb)
    finally:
        hb.heinsen_test_carry(0, 0xFFFFFFFF, 0, stream)
    assert hb.heinsen_check(stream) == hb.HEINSEN_ERR_CARRY_LOST
    assert hb.heinsen_check(stream) == hb.HEINSEN_OK  # reported once, scratch put back in order
    if cfg.layout == "BND":
        g, w = got[0], want[0]                         # [n, D]
        assert np.array_equal(g[:first_bad].view(np.uint32), w[:first_bad].view(np.uint32))
        assert np.isnan(g[first_bad:, :64]).all()      # column 0 from the waiting tiles on
        assert np.array_equal(g[:, 64:].view(np.uint32), w[:, 64:].view(np.uint32))  # column 1 untouched
    else:
        g, w = got.reshape(-1), want.reshape(-1)
        assert np.array_equal(g[:first_bad].view(np.uint32), w[:first_bad].view(np.uint32))
        assert np.isnan(g[first_bad:]).all()
    again = _run(cfg, dev, torch, hb)
    assert np.array_equal(again.view(np.uint32), want.view(np.uint32))


def test_per_tile_time_stamps(gpu):
    torch, hb = gpu
    cfg = workloads.CONFIGS[2].scaled(B=2, D=256, n=2048)  # 8 columns x 8 tiles
    dev = to_device(workloads.generate(cfg), cfg, torch)
    want = _run(cfg, dev, torch, hb)
    tiles = 64
    stamps = torch.zeros(tiles * 8, dtype=torch.int64, device="cuda:0")
    hb.heinsen_set_timeline(stamps, tiles)
    try:
        got = _run(cfg, dev, torch, hb)
    finally:
        hb.heinsen_set_timeline(None, 0)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    t = stamps.cpu().numpy().reshape(tiles, 8)
    assert (t[:, 0] > 0).all()
    for i in range(1, 8):
        assert (t[:, i] >= t[:, i - 1]).all(), f"stamp {i} before stamp {i - 1}"
    assert (t[:, 7] - t[:, 0]).max() < 100_000_000  # a tile lives microseconds, not seconds (100 MHz clock)
    stamps.zero_()
    _run(cfg, dev, torch, hb)
    assert int(stamps.abs().sum().item()) == 0  # switched off again


def test_stream_probe_adds(gpu):
    """The yardstick kernels compute out = a + b for every pattern that applies to the shape."""
    torch, hb = gpu
    B, n, D = 2, 512, 512
    a = torch.rand(B * n * D, dtype=torch.float32, device="cuda:0")
    b = torch.rand(B * n * D, dtype=torch.float32, device="cuda:0")
    for pattern in range(7):
        out = torch.zeros_like(a)
        assert hb.heinsen_stream_probe_status(a, b, out, B, n, D, pattern, torch.cuda.current_stream()) == hb.HEINSEN_OK
        torch.cuda.synchronize()
        assert torch.equal(out, a + b), f"pattern {pattern}"
    ah, bh = a.to(torch.bfloat16), b.to(torch.bfloat16)
    out = torch.zeros_like(a)
    assert hb.heinsen_stream_probe_status(ah, bh, out, B, n, D, 7, torch.cuda.current_stream()) == hb.HEINSEN_OK
    torch.cuda.synchronize()
    assert torch.equal(out, ah.float() + bh.float()), "pattern 7"
    assert hb.heinsen_stream_probe_status(a, b, a, B, 100, D, 1, None) == hb.HEINSEN_ERR_UNSUPPORTED
