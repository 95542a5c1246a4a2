"""Edge cases of the HIP path against the CPU oracle: zeros, exact cancellation, NaN, overflow,
in-place output, x0 handling, by-parts invariance, independent streams.  Every expected value comes
from the oracle (or from IEEE rules the header states); nothing is taken from the GPU."""
import numpy as np
import pytest

import oracle
from paper_2311_06281_amd import workloads

from parity import POS_ATOL, POS_RTOL, SIGNED_RTOL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch

    from paper_2311_06281_amd import binding as hb

    assert torch.cuda.is_available()
    hb.load()
    return torch, hb


def _scan(gpu, a, b, x0, layout, flags=(), out=None, stream=None):
    torch, hb = gpu
    a_t = torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda()
    b_t = torch.from_numpy(np.ascontiguousarray(b, np.float32)).cuda()
    x_t = torch.from_numpy(np.ascontiguousarray(x0, np.float32).reshape(-1)).cuda()
    if layout == "BND":
        B, n, D = a.shape
    else:
        B, D, n = a.shape
    o_t = torch.empty_like(a_t) if out is None else out(a_t, b_t)
    f = hb.flags_from_names(flags)
    if x_t.numel() == 1 and B * D > 1:
        f |= hb.HEINSEN_X0_SCALAR
    hb.heinsen_scan(a_t, b_t, x_t, o_t, B, D, n, hb.LAYOUTS[layout], f, stream or torch.cuda.current_stream())
    torch.cuda.synchronize()
    return o_t.cpu().numpy()


def _ref(a, b, x0, layout):
    lay = oracle.LAYOUT_BND if layout == "BND" else oracle.LAYOUT_BDN
    return oracle.sequential(np.asarray(a, np.float32), np.asarray(b, np.float32), np.asarray(x0, np.float32), layout=lay)


def _assert_signed(got, ref, layout):
    axis = 1 if layout == "BND" else 2
    bound = SIGNED_RTOL * np.maximum.accumulate(np.abs(ref), axis=axis)
    assert np.all(np.abs(got - ref) <= bound + 1e-30), float(np.max(np.abs(got - ref) / (bound + 1e-30)))


SHAPES = [("BDN", (2, 3, 700)), ("BDN", (1, 2, 9000)), ("BDN", (1, 1, 50000)), ("BND", (2, 900, 70)), ("BND", (1, 300, 130)),
          # several rows per wave (rows filling their lanes, and not), narrow channels, short sequences
          ("BDN", (4, 8, 64)), ("BDN", (2, 5, 100)), ("BND", (9, 300, 8)), ("BND", (3, 40, 70))]


@pytest.mark.parametrize("layout,shape", SHAPES)
def test_zero_coefficients_restart_the_sequence(gpu, layout, shape):
    rng = np.random.default_rng(1)
    a = rng.uniform(-1, 1, shape).astype(np.float32)
    b = rng.normal(0, 1, shape).astype(np.float32)
    taxis = 1 if layout == "BND" else 2
    # a_t = 0 at scattered steps (also at the first step and in runs): x_t = b_t there
    idx = [slice(None)] * 3
    nsteps = shape[taxis]
    for t in (0, 5, 6, 7, 63, 64, nsteps // 2, nsteps - 1):
        if t >= nsteps:
            continue
        idx[taxis] = t
        a[tuple(idx)] = 0.0
    B = shape[0]
    D = shape[2] if layout == "BND" else shape[1]
    x0 = rng.normal(0, 1, B * D).astype(np.float32)
    got = _scan(gpu, a, b, x0, layout)
    ref = _ref(a, b, x0, layout)
    assert np.isfinite(got).all()
    _assert_signed(got, ref, layout)
    for t in (0, 6, 64):
        if t >= nsteps:
            continue
        idx[taxis] = t
        np.testing.assert_allclose(got[tuple(idx)], b[tuple(idx)], rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("layout,shape", SHAPES)
def test_b_zero_is_running_product_and_a_one_is_running_sum(gpu, layout, shape):
    rng = np.random.default_rng(2)
    B = shape[0]
    D = shape[2] if layout == "BND" else shape[1]
    x0 = rng.uniform(0.5, 2.0, B * D).astype(np.float32) * np.where(rng.random(B * D) < 0.5, -1, 1).astype(np.float32)
    a = (1.0 + rng.normal(0, 0.01, shape)).astype(np.float32) * np.where(rng.random(shape) < 0.2, -1, 1).astype(np.float32)
    got = _scan(gpu, a, np.zeros(shape, np.float32), x0, layout)
    ref = _ref(a, np.zeros(shape, np.float32), x0, layout)
    np.testing.assert_allclose(got, ref, rtol=2e-4, atol=0)  # no additions: a pure product keeps relative accuracy
    b = rng.normal(0, 1, shape).astype(np.float32)
    got = _scan(gpu, np.ones(shape, np.float32), b, x0, layout)
    ref = _ref(np.ones(shape, np.float32), b, x0, layout)
    _assert_signed(got, ref, layout)


@pytest.mark.parametrize("layout,shape", SHAPES)
def test_wide_dynamic_range(gpu, layout, shape):
    """Coefficients and inputs spread over many orders of magnitude with random signs (|a| log-normal with
    sigma 3 around e^-1, |b| log-normal with sigma 5): every term is carried as a logarithm, so nothing
    overflows or flushes on the way as long as the values themselves fit float32."""
    rng = np.random.default_rng(13)
    sgn = lambda shp: np.where(rng.random(shp) < 0.5, -1.0, 1.0)
    a = (sgn(shape) * np.exp(rng.normal(-1.0, 3.0, shape))).astype(np.float32)
    b = (sgn(shape) * np.exp(rng.normal(0.0, 5.0, shape))).astype(np.float32)
    B = shape[0]
    D = shape[2] if layout == "BND" else shape[1]
    x0 = (sgn(B * D) * np.exp(rng.normal(0.0, 5.0, B * D))).astype(np.float32)
    ref = _ref(a, b, x0, layout)
    assert np.isfinite(ref).all() and np.abs(ref).max() < 1e30  # the data, not the kernel, keeps x inside float32
    got = _scan(gpu, a, b, x0, layout)
    assert np.isfinite(got).all()
    # running scale over s = 0..t: x_0 is huge for some channels and the first steps decay from it
    axis = 1 if layout == "BND" else 2
    shp = (B, 1, D) if layout == "BND" else (B, D, 1)
    scale = np.maximum(np.maximum.accumulate(np.abs(ref), axis=axis), np.abs(x0.astype(np.float64)).reshape(shp))
    assert np.all(np.abs(got - ref) <= SIGNED_RTOL * scale), float(np.max(np.abs(got - ref) / scale))


def test_all_zero_inputs_and_zero_x0(gpu):
    for layout, shape in SHAPES:
        B = shape[0]
        D = shape[2] if layout == "BND" else shape[1]
        z = np.zeros(shape, np.float32)
        got = _scan(gpu, z, z, np.zeros(B * D, np.float32), layout)
        assert np.array_equal(got, z)
        got = _scan(gpu, np.full(shape, 0.5, np.float32), z, np.zeros(B * D, np.float32), layout)
        assert np.array_equal(got, z)


def test_exact_cancellation_gives_zero_not_nan(gpu):
    # hand-worked: x0 = 0, a = (4, 3, -1, 5), b = (0, 2, 2, -7) -> x = (0, 2, 0, -7); repeated many times
    reps = 600
    a = np.tile(np.array([4, 3, -1, 5], np.float32), reps)
    b = np.tile(np.array([0, 2, 2, -7], np.float32), reps)
    a[4::4] = 0.0  # restart each block of four so the pattern repeats exactly
    ref = oracle.seq_f64(a, b, 0.0)
    for layout, shp in (("BDN", (1, 1, a.size)), ("BND", (1, a.size, 1))):
        got = _scan(gpu, a.reshape(shp), b.reshape(shp), np.zeros(1, np.float32), layout).reshape(-1)
        assert not np.isnan(got).any()
        np.testing.assert_allclose(got, ref, rtol=1e-5, atol=1e-5)
    # the same in a channel-contiguous batch
    A = np.repeat(a[None, :, None], 70, axis=2)
    Bm = np.repeat(b[None, :, None], 70, axis=2)
    got = _scan(gpu, A, Bm, np.zeros(70, np.float32), "BND")
    np.testing.assert_allclose(got[0, :, 33], ref, rtol=1e-5, atol=1e-5)


@pytest.mark.parametrize("layout,shape", [("BDN", (1, 3, 5000)), ("BND", (1, 600, 130))])
def test_nan_poisons_only_its_own_sequence_from_its_step_on(gpu, layout, shape):
    rng = np.random.default_rng(3)
    a = rng.uniform(0.5, 1.0, shape).astype(np.float32)
    b = rng.normal(0, 1, shape).astype(np.float32)
    taxis = 1 if layout == "BND" else 2
    caxis = 2 if layout == "BND" else 1
    t_nan = shape[taxis] // 3
    idx = [0, 0, 0]
    idx[taxis] = t_nan
    idx[caxis] = 1
    a[tuple(idx)] = np.nan           # NaN in a of channel 1
    idx[caxis] = 2
    b[tuple(idx)] = np.nan           # NaN in b of channel 2
    D = shape[caxis]
    x0 = np.ones(D, np.float32)
    got = _scan(gpu, a, b, x0, layout)
    got = np.moveaxis(got, taxis, -1)[0]  # [channel, time]
    assert np.isfinite(got[0]).all()
    for ch in (1, 2):
        assert np.isfinite(got[ch, :t_nan]).all()
        assert np.isnan(got[ch, t_nan:]).all()
    if D > 3:
        assert np.isfinite(got[3:]).all()


def test_overflow_goes_to_infinity_where_float32_ends(gpu):
    n = 300
    a = np.full((1, 1, n), 2.0, np.float32)
    b = np.zeros((1, 1, n), np.float32)
    got = _scan(gpu, a, b, np.ones(1, np.float32), "BDN").reshape(-1)
    ref = 2.0 ** np.arange(1, n + 1, dtype=np.float64)
    fin = ref < 3.0e38
    np.testing.assert_allclose(got[fin], ref[fin], rtol=1e-4)
    assert np.isinf(got[ref > 3.5e38]).all() and (got[ref > 3.5e38] > 0).all()


@pytest.mark.parametrize("layout,shape", [("BDN", (1, 2, 1500)), ("BDN", (1, 1, 40000)), ("BND", (1, 1200, 66))])
def test_complex_log_output_stays_finite_where_the_value_leaves_float32(gpu, layout, shape):
    """|x_t| grows like 3^t, far past float32 and float64: its complex logarithm is what can be stored."""
    torch, hb = gpu
    rng = np.random.default_rng(11)
    a = np.where(rng.random(shape) < 0.5, -3.0, 3.0).astype(np.float32)
    b = rng.normal(0, 0.3, shape).astype(np.float32)
    if layout == "BND":
        B, n, D = shape
    else:
        B, D, n = shape
    x0 = np.where(rng.random(B * D) < 0.5, -1.0, 1.0).astype(np.float32)
    a_t, b_t, x_t = (torch.from_numpy(v).cuda() for v in (a, b, x0))
    o_t = torch.full(shape + (2,), float("nan"), dtype=torch.float32, device="cuda")
    hb.heinsen_scan(a_t, b_t, x_t, o_t, B, D, n, hb.LAYOUTS[layout], hb.HEINSEN_LOG_OUTPUT | hb.HEINSEN_OUT_COMPLEX,
                    torch.cuda.current_stream())
    torch.cuda.synchronize()
    got = o_t.cpu().numpy()
    assert np.isfinite(got[..., 0]).all()
    assert np.all((got[..., 1] == 0) | (got[..., 1] == np.float32(np.pi)))
    for bi in range(B):
        for d in range(min(D, 6)):
            sel = (bi, slice(None), d) if layout == "BND" else (bi, d, slice(None))
            ref = oracle.seq_clog_scaled(a[sel], b[sel], x0[bi * D + d])
            re, im = got[sel][:, 0].astype(np.float64), got[sel][:, 1]
            assert np.all(np.abs(re - ref.real) <= 1e-5 * np.abs(ref.real) + 1e-3), float(np.max(np.abs(re - ref.real)))
            np.testing.assert_array_equal(im != 0, ref.imag != 0)


def test_large_local_product_times_small_state_does_not_overflow_on_the_way(gpu):
    # x grows from 1e-30 by 1e5 per step: every x_t fits float32 although prod(a) alone would not
    n = 12
    a = np.full((1, 1, n), 1e5, np.float32)
    b = np.zeros((1, 1, n), np.float32)
    got = _scan(gpu, a, b, np.array([1e-30], np.float32), "BDN").reshape(-1)
    ref = oracle.seq_f64(a.reshape(-1).astype(np.float64), np.zeros(n), float(np.float32(1e-30)))
    np.testing.assert_allclose(got, ref, rtol=1e-4)


@pytest.mark.parametrize("layout,shape", SHAPES)
def test_output_may_alias_an_input(gpu, layout, shape):
    rng = np.random.default_rng(4)
    a = rng.uniform(-1, 1, shape).astype(np.float32)
    b = rng.normal(0, 1, shape).astype(np.float32)
    B = shape[0]
    D = shape[2] if layout == "BND" else shape[1]
    x0 = rng.normal(0, 1, B * D).astype(np.float32)
    plain = _scan(gpu, a, b, x0, layout)
    on_a = _scan(gpu, a, b, x0, layout, out=lambda at, bt: at)
    on_b = _scan(gpu, a, b, x0, layout, out=lambda at, bt: bt)
    assert np.array_equal(plain.view(np.uint32), on_a.view(np.uint32))
    assert np.array_equal(plain.view(np.uint32), on_b.view(np.uint32))


@pytest.mark.parametrize("layout,shape,k", [("BDN", (1, 2, 40000), 16383), ("BDN", (1, 2, 40000), 16384), ("BDN", (2, 2, 1500), 777),
                                            ("BND", (1, 1000, 70), 255), ("BND", (1, 1000, 70), 256), ("BND", (1, 1000, 70), 513)])
def test_scan_by_parts_equals_scan_in_one_go(gpu, layout, shape, k):
    # Sec. 1 footnote: prefix sums can be computed by parts -- restart from x_k and continue
    rng = np.random.default_rng(5)
    a = rng.uniform(-1, 1, shape).astype(np.float32)
    b = rng.normal(0, 1, shape).astype(np.float32)
    B = shape[0]
    D = shape[2] if layout == "BND" else shape[1]
    x0 = rng.normal(0, 1, B * D).astype(np.float32)
    full = _scan(gpu, a, b, x0, layout)
    if layout == "BND":
        head = _scan(gpu, a[:, :k], b[:, :k], x0, layout)
        tail = _scan(gpu, a[:, k:], b[:, k:], head[:, -1, :].reshape(-1), layout)
        joined = np.concatenate([head, tail], axis=1)
    else:
        head = _scan(gpu, a[:, :, :k], b[:, :, :k], x0, layout)
        tail = _scan(gpu, a[:, :, k:], b[:, :, k:], head[:, :, -1].reshape(-1), layout)
        joined = np.concatenate([head, tail], axis=2)
    ref = _ref(a, b, x0, layout)
    _assert_signed(joined, ref, layout)
    _assert_signed(full, ref, layout)


def test_modes_agree_with_each_other_and_the_oracle(gpu):
    """raw / POSITIVE / LOG_INPUTS / LOG_OUTPUT on the same positive data, both layouts."""
    torch, hb = gpu
    rng = np.random.default_rng(6)
    for layout, shape in (("BDN", (2, 3, 2048)), ("BDN", (1, 2, 10000)), ("BND", (2, 700, 66))):
        a = rng.uniform(0.5, 1.0, shape).astype(np.float32)
        b = rng.uniform(0.0, 1.0, shape).astype(np.float32)
        B = shape[0]
        D = shape[2] if layout == "BND" else shape[1]
        x0 = rng.uniform(0.5, 2.0, B * D).astype(np.float32)
        ref = _ref(a, b, x0, layout)
        tol = POS_RTOL * np.abs(ref) + POS_ATOL
        signed = _scan(gpu, a, b, x0, layout)
        pos = _scan(gpu, a, b, x0, layout, flags=("POSITIVE",))
        assert np.all(np.abs(signed - ref) <= tol) and np.all(np.abs(pos - ref) <= tol)
        poslog = _scan(gpu, a, b, x0, layout, flags=("POSITIVE", "LOG_OUTPUT"))
        assert np.all(np.abs(np.exp(poslog.astype(np.float64)) - ref) <= tol)
        # log-domain inputs: the stored float32 logs define the problem, so take the oracle on them
        la, lb, lx0 = np.log(a), np.log(b + 1e-3).astype(np.float32), np.log(x0)
        lay = oracle.LAYOUT_BND if layout == "BND" else oracle.LAYOUT_BDN
        ref_log = oracle.sequential_log(la, lb, lx0, layout=lay)
        lin = _scan(gpu, la, lb, lx0, layout, flags=("LOG_INPUTS",))
        lg = _scan(gpu, la, lb, lx0, layout, flags=("LOG_INPUTS", "LOG_OUTPUT"))
        rl = np.exp(ref_log)
        tl = POS_RTOL * rl + POS_ATOL
        assert np.all(np.abs(lin - rl) <= tl)
        assert np.all(np.abs(np.exp(lg.astype(np.float64)) - rl) <= tl)


def test_log_inputs_accept_minus_infinity_as_zero(gpu):
    n = 3000
    la = np.full((1, 1, n), np.log(0.9), np.float32)
    lb = np.full((1, 1, n), -np.inf, np.float32)   # b = 0
    got = _scan(gpu, la, lb, np.array([0.0], np.float32), "BDN", flags=("LOG_INPUTS", "LOG_OUTPUT")).reshape(-1)
    want = np.arange(1, n + 1) * float(la[0, 0, 0])
    np.testing.assert_allclose(got, want, rtol=1e-5, atol=1e-5)
    got = _scan(gpu, la, lb, np.array([-np.inf], np.float32), "BDN", flags=("LOG_INPUTS", "LOG_OUTPUT")).reshape(-1)
    assert np.all(np.isneginf(got))


def test_scalar_x0_broadcasts(gpu):
    rng = np.random.default_rng(7)
    for layout, shape in (("BDN", (2, 5, 900)), ("BND", (2, 400, 70)), ("BDN", (6, 7, 32)), ("BDN", (2, 9, 50)), ("BND", (20, 300, 4)),
                          ("BND", (2, 30, 100))):
        a = rng.uniform(-1, 1, shape).astype(np.float32)
        b = rng.normal(0, 1, shape).astype(np.float32)
        B = shape[0]
        D = shape[2] if layout == "BND" else shape[1]
        one = _scan(gpu, a, b, np.array([0.75], np.float32), layout)
        full = _scan(gpu, a, b, np.full(B * D, 0.75, np.float32), layout)
        assert np.array_equal(one.view(np.uint32), full.view(np.uint32))


def test_channels_do_not_interact(gpu):
    rng = np.random.default_rng(8)
    shape = (2, 500, 200)  # [B, n, D]
    a = rng.uniform(-1, 1, shape).astype(np.float32)
    b = rng.normal(0, 1, shape).astype(np.float32)
    x0 = rng.normal(0, 1, 400).astype(np.float32)
    base = _scan(gpu, a, b, x0, "BND")
    perm = rng.permutation(200)
    got = _scan(gpu, a[:, :, perm], b[:, :, perm], x0.reshape(2, 200)[:, perm].reshape(-1), "BND")
    assert np.array_equal(got.view(np.uint32), base[:, :, perm].view(np.uint32))
    # the same sequences stored the other way round give the same values up to rounding order
    t = _scan(gpu, a.transpose(0, 2, 1), b.transpose(0, 2, 1), x0, "BDN")
    ref = _ref(a, b, x0, "BND")
    _assert_signed(t.transpose(0, 2, 1), ref, "BND")


def test_two_streams_use_separate_scratch(gpu):
    torch, hb = gpu
    cfgs = [workloads.CONFIGS[5].scaled(B=2, D=256, n=4096), workloads.CONFIGS[3].scaled(n=16384 * 40)]
    singles = []
    for cfg in cfgs:
        from parity import run_gpu
        singles.append(run_gpu(cfg, workloads.generate(cfg), torch, hb))
    from parity import to_device
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    bufs = []
    for cfg in cfgs:
        a, b, x0 = to_device(workloads.generate(cfg), cfg, torch)
        bufs.append((a, b, x0, torch.empty(a.shape, dtype=torch.float32, device="cuda")))
    torch.cuda.synchronize()
    for rep in range(5):
        for cfg, st, (a, b, x0, out) in zip(cfgs, streams, bufs):
            hb.heinsen_scan(a, b, x0, out, cfg.B, cfg.D, cfg.n, hb.LAYOUTS[cfg.layout], hb.flags_from_names(cfg.flags), st)
    torch.cuda.synchronize()
    for single, (a, b, x0, out) in zip(singles, bufs):
        assert np.array_equal(out.cpu().numpy().view(np.uint32), single.view(np.uint32))


def test_capture_without_existing_scratch_is_refused(gpu):
    """A call that needs carries cannot allocate its scratch while its stream is capturing: on a stream
    that has never run such a call it is refused, and nothing is recorded."""
    torch, hb = gpu
    cfg = workloads.CONFIGS[5].scaled(B=1, D=128, n=1024)
    from parity import to_device
    a, b, x0 = to_device(workloads.generate(cfg), cfg, torch)
    out = torch.empty(a.shape, dtype=torch.float32, device="cuda")
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        g.capture_begin()
        try:
            st = hb.heinsen_scan_status(a, b, x0, out, cfg.B, cfg.D, cfg.n, hb.LAYOUTS[cfg.layout], 0, s)
        finally:
            g.capture_end()
    assert st == hb.HEINSEN_ERR_UNSUPPORTED


@pytest.mark.parametrize("layout,shape", [("BND", (2, 1500, 256)), ("BDN", (1, 2, 16384 * 5 + 24)), ("BND", (40, 700, 8))])
def test_calls_with_carries_can_be_captured_once_the_stream_has_scratch(gpu, layout, shape):
    """After one ordinary call on the stream (a warm-up, which made the scratch) the same call may be
    captured: replays take their launch epoch and tickets from the scratch header.  Three replays on fresh
    inputs, with ordinary calls of this and of a larger shape (which replaces the stream's scratch) and
    synchronisations in between, each checked against the oracle and bit for bit against the ordinary call."""
    torch, hb = gpu
    rng = np.random.default_rng(31)
    if layout == "BND":
        B, n, D = shape
        big = (B, 2 * n, D)
    else:
        B, D, n = shape
        big = (B, D, 2 * n)

    def draw(shp):
        return (rng.uniform(-1.05, 1.05, shp).astype(np.float32), rng.normal(0, 1, shp).astype(np.float32),
                rng.normal(0, 1, B * D).astype(np.float32))

    side = torch.cuda.Stream()
    a_h, b_h, x_h = draw(shape)
    a_t, b_t, x_t = (torch.from_numpy(v).cuda() for v in (a_h, b_h, x_h))
    out_g = torch.zeros(shape, dtype=torch.float32, device="cuda")
    out_e = torch.zeros(shape, dtype=torch.float32, device="cuda")
    ab_big = [torch.from_numpy(v).cuda() for v in draw(big)]
    out_big = torch.zeros(big, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        hb.heinsen_scan(a_t, b_t, x_t, out_e, B, D, n, hb.LAYOUTS[layout], 0, side)  # warm-up: allocates the scratch
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        hb.heinsen_scan(a_t, b_t, x_t, out_g, B, D, n, hb.LAYOUTS[layout], 0, torch.cuda.current_stream())
    for rep in range(3):
        a_h, b_h, x_h = draw(shape)
        a_t.copy_(torch.from_numpy(a_h))
        b_t.copy_(torch.from_numpy(b_h))
        x_t.copy_(torch.from_numpy(x_h))
        out_g.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            g.replay()
        side.synchronize()
        with torch.cuda.stream(side):
            hb.heinsen_scan(a_t, b_t, x_t, out_e, B, D, n, hb.LAYOUTS[layout], 0, side)
            if rep == 1:  # a larger ordinary call replaces the stream's scratch; the graph keeps the old one
                nb = big[1] if layout == "BND" else big[2]
                hb.heinsen_scan(ab_big[0], ab_big[1], ab_big[2], out_big, B, D, nb, hb.LAYOUTS[layout], 0, side)
        side.synchronize()
        got = out_g.cpu().numpy()
        assert np.array_equal(got.view(np.uint32), out_e.cpu().numpy().view(np.uint32)), f"replay {rep} differs from the ordinary call"
        _assert_signed(got.astype(np.float64), _ref(a_h, b_h, x_h, layout), layout)


@pytest.mark.parametrize("layout,shape", [("BDN", (2, 8, 2048)), ("BDN", (70, 1, 16384)), ("BND", (2, 64, 128)), ("BDN", (64, 4, 64)), ("BND", (40, 33, 8))])
def test_scratch_free_shapes_can_be_captured_and_replayed(gpu, layout, shape):
    """Shapes that need no carries use no scratch and no launch counter, so a captured call may be replayed:
    three replays on fresh inputs, with eager calls and synchronisations in between, each checked against
    the oracle and bit for bit against the eager call."""
    torch, hb = gpu
    rng = np.random.default_rng(21)
    if layout == "BND":
        B, n, D = shape
    else:
        B, D, n = shape

    def draw():
        return (rng.uniform(-1.05, 1.05, shape).astype(np.float32), rng.normal(0, 1, shape).astype(np.float32),
                rng.normal(0, 1, B * D).astype(np.float32))

    a_h, b_h, x_h = draw()
    a_t, b_t, x_t = (torch.from_numpy(v).cuda() for v in (a_h, b_h, x_h))
    out_g = torch.zeros(shape, dtype=torch.float32, device="cuda")
    out_e = torch.zeros(shape, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        hb.heinsen_scan(a_t, b_t, x_t, out_g, B, D, n, hb.LAYOUTS[layout], 0, torch.cuda.current_stream())
    for rep in range(3):
        a_h, b_h, x_h = draw()
        a_t.copy_(torch.from_numpy(a_h))
        b_t.copy_(torch.from_numpy(b_h))
        x_t.copy_(torch.from_numpy(x_h))
        out_g.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        hb.heinsen_scan(a_t, b_t, x_t, out_e, B, D, n, hb.LAYOUTS[layout], 0, torch.cuda.current_stream())
        torch.cuda.synchronize()
        got = out_g.cpu().numpy()
        assert np.array_equal(got.view(np.uint32), out_e.cpu().numpy().view(np.uint32)), f"replay {rep} differs from the eager call"
        _assert_signed(got.astype(np.float64), _ref(a_h, b_h, x_h, layout), layout)


def test_sequential_baseline_kernel_matches_the_definition(gpu):
    torch, hb = gpu
    for n in (1, 5, 1023, 1024, 1025, 5000):
        cfg = workloads.CONFIGS[1].scaled(n=n)
        batch = workloads.generate(cfg)
        a = torch.from_numpy(batch.a).cuda()
        b = torch.from_numpy(batch.b).cuda()
        x0 = torch.from_numpy(batch.x0).cuda()
        out = torch.full_like(a, float("nan"))
        hb.heinsen_sequential(a, b, x0, out, n, torch.cuda.current_stream())
        torch.cuda.synchronize()
        ref = oracle.seq_f64(batch.a.reshape(-1), batch.b.reshape(-1), 1.0)
        np.testing.assert_allclose(out.cpu().numpy().reshape(-1), ref, rtol=1e-4, atol=1e-6)
