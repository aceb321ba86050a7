"""CPU check of bench.py's byte accounting: the algorithmic bytes per step that the
roofline fraction is computed from, for the five workloads, against the figures
that follow from the method's definition (per worker and index: one gradient read,
error memory read + write, momentum read + write; x read once everywhere when weight
decay needs it, else read on the block; x written on the block; y adds one write of
d floats, plus a read of x where the step did not read it already)."""
import pytest

import bench
from paper_2004_05298_amd import workloads as wl

# name: (d, W, B, weight decay?, bytes per step, bytes per step with y)
EXPECTED = {
    "tiny": (65_536, 4, 4_096, False, 5_275_648, 5_799_936),
    "resnet56_shaped": (853_018, 8, 26_657, False, 136_696_136, 143_520_280),
    "resnet18_shaped": (11_689_512, 16, 182_649, False, 3_742_105_032, 3_835_621_128),
    "resnet50_shaped": (25_557_032, 16, 199_665, True, 8_281_277_028, 8_383_505_156),
    "vgg16_shaped": (138_357_544, 32, 540_460, False, 88_553_151_840, 89_660_012_192),
}


@pytest.mark.parametrize("name", sorted(EXPECTED))
def test_algorithmic_bytes_per_step(name):
    d, W, B, decay, plain, with_y = EXPECTED[name]
    w = wl.by_name(name)
    assert (w.d, w.W, w.B, w.weight_decay != 0) == (d, W, B, decay)
    # the table above, re-derived
    state = 20 * W * d
    assert plain == state + (4 * d + 4 * B if decay else 8 * B)
    assert with_y == plain + (4 * d if decay else 8 * d)
    assert bench.algorithmic_bytes(w)["step"] == plain
    assert bench.algorithmic_bytes(w, y_out=True)["step"] == with_y
    # the streaming kernel's share: everything but the block-sized terms
    assert bench.algorithmic_bytes(w)["stream_kernel"] == state + (4 * d if decay else 0)
    # detached points: one more write per (worker, index), and x is then read everywhere
    assert bench.algorithmic_bytes(w, detach=True)["step"] == 24 * W * d + 4 * d + 4 * B


def test_time_at_peak_of_the_benchmark_workload():
    """8.281 GB per step at 8 TB/s is 1.035 ms: 966 steps/s at 100 %, 773 at 80 %."""
    w = wl.by_name("resnet50_shaped")
    seconds = bench.algorithmic_bytes(w)["step"] / (bench.HBM_PEAK_GBS * 1e9)
    assert round(seconds * 1e3, 3) == 1.035
    assert int(1 / seconds) == 966 and int(0.8 / seconds) == 772
