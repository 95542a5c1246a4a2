"""Seeded random draw of shapes, layouts, modes, storage types and pointer offsets, every case checked in
full against the float64 definition (the helpers and bounds of test_gpu_cross_product.py).  The lists of
sizes sit on the edges of the launch plans: wave, tile and group boundaries, narrow and ragged channels,
one to thousands of sequences."""
import numpy as np
import pytest

from paper_2311_06281_amd import workloads

import test_gpu_cross_product as cross
from test_gpu_cross_product import gpu  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu

CHANNELS = [1, 2, 3, 4, 5, 7, 8, 9, 16, 17, 31, 32, 33, 40, 63, 64, 65, 127, 128, 129, 192, 256, 320, 384, 1024, 2048, 4096]
BATCHES = [1, 1, 2, 3, 5, 8, 17, 40, 300]
STEPS_BND = [1, 2, 3, 5, 31, 32, 33, 63, 64, 65, 70, 127, 128, 129, 255, 256, 257, 300, 511, 512, 513, 1000, 1023, 1024, 1025,
             1100, 2047, 2049, 4095, 4097, 9000, 20000, 33000, 70000, 300000]
ROWS = [1, 1, 2, 3, 7, 63, 64, 65, 200, 500, 3000]
STEPS_BDN = [1, 2, 7, 8, 9, 60, 64, 65, 200, 255, 256, 257, 511, 512, 513, 1023, 1024, 1025, 2047, 2048, 2049, 4095, 4096, 4097,
             8191, 8192, 8193, 16383, 16384, 16385, 40000, 200000, 1050000, 1200000]
MAX_ELEMENTS = 1_500_000


def _draw(rng):
    while True:
        if rng.random() < 0.55:
            layout = "BND"
            n = int(rng.choice(STEPS_BND)) + (int(rng.integers(0, 300)) if rng.random() < 0.3 else 0)
            shape = (int(rng.choice(BATCHES)), n, int(rng.choice(CHANNELS)))
        else:
            layout = "BDN"
            rows = int(rng.choice(ROWS))
            n = int(rng.choice(STEPS_BDN)) + (int(rng.integers(0, 40)) if rng.random() < 0.3 else 0)
            B = int(rng.choice([1, 2, 3]))
            shape = (B, max(1, rows // B), n)
        if shape[0] * shape[1] * shape[2] <= MAX_ELEMENTS:
            return layout, shape


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_shapes_modes_and_offsets(gpu, seed):
    rng = np.random.default_rng(seed)
    modes = list(cross.MODES)
    for case in range(150):
        layout, shape = _draw(rng)
        mode = modes[int(rng.integers(len(modes)))]
        bf16 = bool(rng.random() < 0.3)
        offset = int(rng.choice([0, 0, 0, 1, 2, 4]))
        a, b, x0 = cross._inputs(rng, shape, layout, mode)
        if bf16:  # the bf16-rounded values are what is stored: they define the problem
            a = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(a)).reshape(shape)
            b = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(b)).reshape(shape)
        print(f"[random] seed {seed} case {case}: {layout} {shape} {mode} bf16={bf16} offset={offset}", flush=True)
        got = cross._run(gpu, a, b, x0, layout, cross.MODES[mode], bf16, offset_elems=offset)
        cross._check(got, a, b, x0, layout, mode)
