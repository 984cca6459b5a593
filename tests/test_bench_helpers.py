"""The byte accounting behind bench.py's figures, against numbers worked out by hand (CPU only)."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import bench
from paper_2602_06694_amd import synth


def test_algorithmic_bytes_of_the_headline_layer():
    shp = synth.CONFIGS[2].block[0]                       # 4096 x 4096, r = 1024
    assert (shp.d_out, shp.d_in, shp.r) == (4096, 4096, 1024)
    weights, everything = bench.algorithmic_bytes(shp, 1)
    # bits of both factors + two fp16 scale vectors
    assert weights == 1024 * (4096 + 4096) // 8 + 2 * (4096 + 4096) == 1064960
    # + bf16 x, fp32 y, and the intermediate t written once and read once (fp32)
    assert everything == weights + 4096 * 2 + 4096 * 4 + 2 * 1024 * 4
    # 1024 layers: the figures the headline line carries
    assert 1024 * weights == 1090519040 and 1024 * everything == 1124073472


def test_stage_bytes_of_the_headline_launches():
    shp = synth.CONFIGS[2].block[0]
    s1, s2 = bench.stage_bytes(shp, 1, 4, (True, True))   # both launches quantise their own input
    # stage 1: V bits, bf16 x, fp16 s_in, fp32 t out;  stage 2: U bits, fp16 s_out, fp32 t in, fp32 y out
    assert s1 == 4096 * 1024 // 8 + 2 * 4096 + 2 * 4096 + 4 * 1024 == 544768
    assert s2 == 4096 * 1024 // 8 + 2 * 4096 + 4 * 1024 + 4 * 4096 == 552960
    assert 1024 * s1 == 557842432 and 1024 * s2 == 566231040
    # launches fed by a quantisation launch read 3 bytes per input element instead
    q1, q2 = bench.stage_bytes(shp, 8, 4, (False, False))
    assert q1 == 4096 * 1024 // 8 + 3 * 8 * 4096 + 4 * 8 * 1024
    assert q2 == 4096 * 1024 // 8 + 2 * 4096 + 3 * 8 * 1024 + 4 * 8 * 4096


def test_profile_traffic_is_tied_to_the_profiled_kernel():
    wl = "cfg2: 1024 x [4096x4096 r=1024], decode batch 1, bf16 x"
    t1 = bench.measured_traffic(wl, "stage1", "nq::stage_selfq_kernel<W=4>")
    t2 = bench.measured_traffic(wl, "stage2", "nq::stage_selfq_kernel<W=1>")
    assert t1 and t2 and 0.98 < t1 / 557842432 < 1.10 and 0.98 < t2 / 566231040 < 1.10
    assert bench.measured_traffic(wl, "stage1", "nq::stage_split_kernel<W=4>") is None        # another kernel ran
    assert bench.measured_traffic("cfg4: something else", "stage1", "nq::stage_selfq_kernel<W=4>") is None


def test_window_statistics():
    s = bench.window_stats([3.0, 1.0, 2.0, 5.0, 4.0])
    assert s == {"median": 3.0, "min": 1.0, "max": 5.0, "windows": 5}
