"""Flag x layout x storage-type cross product at small sizes, awkward shapes and pointer alignments,
and interleaved calls of different shapes on one stream (they share one scratch buffer)."""
import itertools

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


def _inputs(rng, shape, layout, mode):
    """Stored inputs (float32 arrays holding exactly what the GPU reads) for one mode."""
    B = shape[0]
    D = shape[2] if layout == "BND" else shape[1]
    if mode in ("signed", "signed_clog", "linear"):
        a = rng.uniform(-1.1, 1.1, shape)
        b = rng.normal(0, 1, shape)
        x0 = rng.normal(0, 1, B * D)
    elif mode in ("positive", "positive_logout"):
        a = rng.uniform(0.4, 1.05, shape)
        b = rng.uniform(0, 1, shape)
        x0 = rng.uniform(0.1, 2, B * D)
    else:  # log inputs
        a = -np.logaddexp(0.0, rng.normal(0, 1, shape))
        b = rng.normal(-1, 1, shape)
        x0 = rng.normal(0, 0.5, B * D)
    return a.astype(np.float32), b.astype(np.float32), x0.astype(np.float32)


MODES = {
    "signed": (),
    "positive": ("POSITIVE",),
    "positive_logout": ("POSITIVE", "LOG_OUTPUT"),
    "log": ("LOG_INPUTS",),
    "log_logout": ("LOG_INPUTS", "LOG_OUTPUT"),
    "signed_clog": ("LOG_OUTPUT", "OUT_COMPLEX"),
    "linear": ("LINEAR",),  # comparison path: same data and bound as the signed log-space path
}
SHAPES = {
    "BDN": [(2, 3, 1), (1, 5, 17), (4, 8, 64), (3, 5, 256), (2, 70, 8), (1, 9, 100), (2, 3, 520), (1, 2, 2048), (1, 3, 2056), (1, 2, 6000), (1, 1, 12004), (1, 1, 16384 * 3 + 8),
            (3, 2, 16384 + 1)],
    "BND": [(2, 1, 5), (1, 17, 3), (2, 300, 64), (1, 257, 66), (1, 513, 130), (1, 40, 1000), (2, 1025, 7), (70, 40, 4), (9, 600, 32),
            (5, 520, 2), (3, 1100, 33), (2, 100, 70), (4, 120, 8), (1, 256 * 19 + 5, 66),
            # few columns: groups of eight tiles (20 columns), second carry level (3 columns: 4 x 4 tiles, 2 columns: 8 x 8)
            (20, 256 * 19 + 5, 64), (3, 4096 * 2 + 700, 64), (1, 16384 * 2 + 300, 70),
            # the same with narrow channels (several batch items per column)
            (20, 4096 * 2 + 700, 8), (5, 16384 * 2 + 300, 2), (300, 256 * 9 + 1, 4)],
}


def _run(gpu, a, b, x0, layout, flag_names, bf16, offset_elems=0):
    torch, hb = gpu
    if layout == "BND":
        B, n, D = a.shape
    else:
        B, D, n = a.shape

    def dev(arr, as_bf16):
        flat = arr.reshape(-1)
        if as_bf16:
            bits = workloads.f32_to_bf16_bits(flat).view(np.int16)
            buf = torch.zeros(bits.size + offset_elems + 8, dtype=torch.int16, device="cuda")
            buf[offset_elems:offset_elems + bits.size] = torch.from_numpy(bits).cuda()
            return buf, buf[offset_elems:]
        buf = torch.zeros(flat.size + offset_elems + 8, dtype=torch.float32, device="cuda")
        buf[offset_elems:offset_elems + flat.size] = torch.from_numpy(flat).cuda()
        return buf, buf[offset_elems:]

    keep_a, a_t = dev(a, bf16)
    keep_b, b_t = dev(b, bf16)
    x_t = torch.from_numpy(x0).cuda()
    ow = 2 if "OUT_COMPLEX" in flag_names else 1  # floats per output element
    keep_o = torch.full((ow * (a.size + offset_elems) + 8,), float("nan"), dtype=torch.float32, device="cuda")
    o_t = keep_o[ow * offset_elems:]
    flags = hb.flags_from_names(flag_names) | (hb.HEINSEN_IN_BF16 if bf16 else 0)
    hb.heinsen_scan(a_t, b_t, x_t, o_t, B, D, n, hb.LAYOUTS[layout], flags, torch.cuda.current_stream())
    torch.cuda.synchronize()
    res = keep_o.cpu().numpy()
    # nothing outside the output range was touched
    assert np.isnan(res[:ow * offset_elems]).all() and np.isnan(res[ow * (offset_elems + a.size):]).all()
    res = res[ow * offset_elems:ow * (offset_elems + a.size)]
    return res.reshape(a.shape + (2,)) if ow == 2 else res.reshape(a.shape)


def _check(got, a, b, x0, layout, mode):
    lay = oracle.LAYOUT_BND if layout == "BND" else oracle.LAYOUT_BDN
    if mode in ("log", "log_logout"):
        ref = np.exp(oracle.sequential_log(a, b, x0, layout=lay))
    else:
        ref = oracle.sequential(a, b, x0, layout=lay)
    if mode == "signed_clog":
        # complex logarithm: the imaginary part is exactly 0 or float32(pi); back in the linear domain
        # the value is held to the signed bound
        re, im = got[..., 0].astype(np.float64), got[..., 1]
        assert np.all((im == 0) | (im == np.float32(np.pi)))
        val = np.exp(re) * np.where(im == 0, 1.0, -1.0)
    else:
        val = np.exp(got.astype(np.float64)) if mode.endswith("logout") else got.astype(np.float64)
    err = np.abs(val - ref)
    if mode in ("signed", "signed_clog", "linear"):
        # running scale max_{0<=s<=t} |x_s|: it starts at |x_0|, which is a member of the sequence (a first
        # step that cancels, x_1 = a_1 x_0 + b_1 ~ 0, has no other scale to be measured against)
        axis = 1 if layout == "BND" else 2
        shp = (a.shape[0], 1, a.shape[2]) if layout == "BND" else (a.shape[0], a.shape[1], 1)
        scale = np.maximum(np.maximum.accumulate(np.abs(ref), axis=axis), np.abs(x0.astype(np.float64)).reshape(shp))
        bound = SIGNED_RTOL * scale
    else:
        bound = POS_RTOL * np.abs(ref) + POS_ATOL
    assert np.all(err <= bound), f"worst error/bound {np.max(err / (bound + 1e-300)):.3g}"


@pytest.mark.parametrize("layout", ["BDN", "BND"])
@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("bf16", [False, True])
def test_every_mode_layout_and_storage_type(gpu, layout, mode, bf16):
    seed = sum(ord(ch) for ch in layout + mode) * 2 + int(bf16)  # fixed: hash() of str is salted per process
    rng = np.random.default_rng(seed)
    for shape in SHAPES[layout]:
        a, b, x0 = _inputs(rng, shape, layout, mode)
        if bf16:  # the bf16-rounded values are what is stored: they define the problem
            a = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(a)).reshape(shape)
            b = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(b)).reshape(shape)
        print(f"[cross] {layout} {mode} bf16={bf16} shape={shape}", flush=True)
        got = _run(gpu, a, b, x0, layout, MODES[mode], bf16)
        _check(got, a, b, x0, layout, mode)


# [B, n, D] with at least 256 columns of 128 channels and n >= 1024 takes the wide tile (two waves side by
# side, 128 steps per tile): a ragged tail (9 tiles and 77 steps: two waves and a half of the last tile have
# steps, the other one and a half have none) and a last column that ends with the array
@pytest.mark.parametrize("mode,bf16", [(m, False) for m in MODES] + [("signed", True), ("log_logout", True)])
def test_wide_tiles_every_mode(gpu, mode, bf16):
    torch, hb = gpu
    shape = (2, 1024 + 205, 16384)
    flags = hb.flags_from_names(MODES[mode]) | (hb.HEINSEN_IN_BF16 if bf16 else 0)
    tile = hb.heinsen_tile_shape(shape[0], shape[2], shape[1], hb.HEINSEN_LAYOUT_BND, flags)
    assert tile == ((64, 256) if mode == "signed_clog" else (128, 128))  # the complex output has a tile of its own
    print(f"[wide] {mode} bf16={bf16} shape={shape} tile={tile}", flush=True)
    rng = np.random.default_rng(4100 + sum(ord(ch) for ch in mode) + int(bf16))
    a, b, x0 = _inputs(rng, shape, "BND", mode)
    if bf16:
        a = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(a)).reshape(shape)
        b = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(b)).reshape(shape)
    got = _run(gpu, a, b, x0, "BND", MODES[mode], bf16)
    _check(got, a, b, x0, "BND", mode)


@pytest.mark.parametrize("layout,shape", [("BDN", (2, 3, 2048)), ("BDN", (1, 2, 16384 * 2 + 16)), ("BND", (1, 300, 128)), ("BND", (2, 64, 66))])
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("offset", [1, 2, 3])
def test_pointers_that_are_only_element_aligned(gpu, layout, shape, bf16, offset):
    # the vector paths need 16-byte alignment; anything less must fall back, not fault or smear
    rng = np.random.default_rng(99 + offset)
    a, b, x0 = _inputs(rng, shape, layout, "signed")
    if bf16:
        a = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(a)).reshape(shape)
        b = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(b)).reshape(shape)
    got = _run(gpu, a, b, x0, layout, (), bf16, offset_elems=offset)
    _check(got, a, b, x0, layout, "signed")


@pytest.mark.parametrize("layout,shape", [("BDN", (2, 3, 2048)), ("BDN", (1, 2, 16384 * 2 + 16)), ("BND", (1, 300, 128)), ("BND", (2, 64, 66))])
@pytest.mark.parametrize("bf16", [False, True])
def test_complex_output_with_element_aligned_pointers(gpu, layout, shape, bf16):
    rng = np.random.default_rng(7)
    a, b, x0 = _inputs(rng, shape, layout, "signed_clog")
    if bf16:
        a = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(a)).reshape(shape)
        b = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(b)).reshape(shape)
    got = _run(gpu, a, b, x0, layout, MODES["signed_clog"], bf16, offset_elems=1)
    _check(got, a, b, x0, layout, "signed_clog")


def test_interleaved_shapes_on_one_stream_share_scratch_safely(gpu):
    """Carry records of earlier launches (other shapes, other layouts) must never be taken for current ones."""
    torch, hb = gpu
    rng = np.random.default_rng(5)
    cases = []
    for layout, shape in (("BND", (1, 1030, 130)), ("BDN", (1, 2, 16384 * 5 + 4)), ("BND", (2, 520, 64)),
                          ("BDN", (2, 1, 16384 * 2 + 4)), ("BND", (1, 2100, 70))):
        a, b, x0 = _inputs(rng, shape, layout, "signed")
        cases.append((layout, shape, a, b, x0))
    order = [0, 1, 2, 3, 4, 1, 0, 3, 2, 4, 4, 0, 1]
    first = {}
    for rep, i in enumerate(order):
        layout, shape, a, b, x0 = cases[i]
        got = _run(gpu, a, b, x0, layout, (), False)
        if i not in first:
            _check(got, a, b, x0, layout, "signed")
            first[i] = got
        else:
            assert np.array_equal(got.view(np.uint32), first[i].view(np.uint32)), f"call {rep} (case {i}) changed"


def test_release_scratch_then_continue(gpu):
    torch, hb = gpu
    rng = np.random.default_rng(6)
    a, b, x0 = _inputs(rng, (1, 1100, 70), "BND", "signed")
    one = _run(gpu, a, b, x0, "BND", (), False)
    assert hb.heinsen_release_scratch() == hb.HEINSEN_OK
    two = _run(gpu, a, b, x0, "BND", (), False)
    assert np.array_equal(one.view(np.uint32), two.view(np.uint32))


def test_many_launches_in_a_row_without_synchronising(gpu):
    torch, hb = gpu
    cfg = workloads.CONFIGS[5].scaled(B=1, D=192, n=2000)
    from parity import reference, to_device, violations
    batch = workloads.generate(cfg)
    a, b, x0 = to_device(batch, cfg, torch)
    outs = [torch.empty(a.shape, dtype=torch.float32, device="cuda") for _ in range(40)]
    for o in outs:
        hb.heinsen_scan(a, b, x0, o, cfg.B, cfg.D, cfg.n, hb.LAYOUTS[cfg.layout], 0, torch.cuda.current_stream())
    torch.cuda.synchronize()
    ref = reference(cfg, batch)
    first = outs[0].cpu().numpy()
    assert violations(cfg, first, ref)[0] == 0
    for o in outs[1:]:
        assert torch.equal(o.view(torch.int32), outs[0].view(torch.int32))
