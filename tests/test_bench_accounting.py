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
