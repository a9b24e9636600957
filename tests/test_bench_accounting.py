"""bench.py's byte accounting against sums written out by hand (CPU only): the figures that turn
kernel and step times into fractions of the HBM peak."""
import importlib.util
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("_bench", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_kernel_bytes_are_each_input_once_each_output_once():
    b = _bench()
    p, d = b.KERNEL_BYTES["packed"], b.KERNEL_BYTES["dense"]
    bit = 1.0 / 8
    # worker compression, deferred error: R g, z (8), momentum bits and own previous bits; W z, bits
    assert p["compress_deferred"][0] == 4 + 4 + bit + bit + 4 + bit
    assert d["compress_deferred"][0] == 4 + 4 + 4 + bit + 4 + bit
    # ... with a chunk barrier: R g, err, momentum bits; W err, bits
    assert p["compress_resident"][0] == 4 + 4 + bit + 4 + bit
    # ratio pass: R new and old bits, v_fresh, v_frozen; W v_fresh.  update: R bits, v_frozen, x; W x
    assert p["ratios_pass"][0] == 2 * bit + 4 + 4 + 4
    assert p["decompress_apply"][0] == bit + 4 + 4 + 4
    # both in one kernel: v_frozen and the new bits are read once
    assert p["ratios_apply_resident"][0] == p["ratios_pass"][0] + p["decompress_apply"][0] - (4 + bit)
    assert b.KERNEL_BYTES["both"]["warmup_resident"][0] == 16 + 12


def test_step_bytes():
    b = _bench()
    W = 64
    bit = 1.0 / 8
    all_fused = b.algorithmic_step_bytes_per_param(W, "packed", 1.0, "deferred", False)
    assert abs(all_fused - (12.375 + 20.25 + bit + 8.375 / W)) < 1e-12
    none_fused = b.algorithmic_step_bytes_per_param(W, "packed", 0.0, "barrier", True)
    assert abs(none_fused - (12.25 + 12.25 + 12.125 + bit + 8.125 / W)) < 1e-12
    two_pass = b.algorithmic_step_bytes_per_param(W, "dense", 0.0, "two_pass", False)
    assert abs(two_pass - (16.0 + 8.125 + 16.125 + 16.125 + bit + 16.125 / W)) < 1e-12
    # the accounting with an fp32 momentum and two update calls that the step is NOT measured against
    assert abs(b.fp32_momentum_equivalent_bytes_per_param(W) - (16.125 + bit + 8.125 / W + 16.125 + 12.0)) < 1e-12
    assert b.HBM_PEAK_GBS == 8000.0


def test_bytes_with_the_variance_in_deferred_form():
    b = _bench()
    bit = 1.0 / 8
    # one momentum step applied and the array written: the same accesses as the kernel that rewrites
    # the array at every step
    assert b.hist_kernel_bytes_per_param({1: 3}, 1) == b.KERNEL_BYTES["packed"]["ratios_apply_resident"][0]
    # period 4: three steps that write nothing (2, 3, 4 momenta's sign words) and one that reads 5 and writes
    per_step = [4 + 4 + 4 + 4 + 2 * bit, 16 + 3 * bit, 16 + 4 * bit, 16 + 5 * bit + 4]
    assert abs(b.hist_kernel_bytes_per_param({1: 1, 2: 1, 3: 1, 4: 1}, 4) - sum(per_step) / 4) < 1e-12
    # ... weighted by how often each length occurred
    assert abs(b.hist_kernel_bytes_per_param({1: 2, 4: 1}, 4) - (2 * per_step[0] + per_step[3]) / 3) < 1e-12
    W = 64
    step = b.algorithmic_step_bytes_per_param(W, "packed", 0.9, "deferred", False, fused_bytes=17.0)
    assert abs(step - (12.375 + 0.9 * 17.0 + 0.1 * (12.25 + 12.125) + bit + 8.375 / W)) < 1e-12
    # part of the parameters in layers too large for that kernel: ratio pass from the history on big tiles
    assert b.hist_big_ratio_bytes_per_param({1: 1, 2: 1, 3: 1, 4: 1}, 4) == (8 + 2 * bit + 8 + 3 * bit + 8 + 4 * bit + 8 + 5 * bit + 4) / 4
    step = b.algorithmic_step_bytes_per_param(W, "packed", 0.5, "deferred", False, fused_bytes=17.0, big_frac=0.3,
                                              big_ratio_bytes=9.5)
    assert abs(step - (12.375 + 0.5 * 17.0 + 0.3 * (9.5 + 12.125) + 0.2 * (12.25 + 12.125) + bit + 8.375 / W)) < 1e-12
