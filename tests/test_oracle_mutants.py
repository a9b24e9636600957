"""Do the oracle's pins catch a plausible mistake anywhere in it?

Each case below plants ONE mistake in a scratch copy of oracle/obref.cpp (a dropped term, a wrong
sign or index, swapped operands, a wrong divisor or order), compiles the copy and runs the pins of
tests/test_oracle_pins.py against it in a child process: at least one pin must fail.  The oracle's
own source is never touched, and nothing here runs on a GPU.

A case names the text it replaces; the text must occur in obref.cpp exactly as often as stated, so
that a case cannot silently stop applying when the oracle's source changes.
"""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "obref.cpp")

# (name, text to replace, replacement, occurrences expected, which occurrence to replace)
MUTANTS = [
    # C[z] and the error feedback (Section 2; Algorithm 1 lines 7 and 10)
    ("scale_divides_by_n_minus_1", "const T s = (T)std::sqrt(S / (double)n);",
     "const T s = (T)std::sqrt(S / (double)(n - 1));", 1, 0),
    ("scale_is_mean_absolute_value", "for (int64_t i = 0; i < n; ++i) S += (double)z[i] * (double)z[i];\n  const T s = (T)std::sqrt(S / (double)n);",
     "for (int64_t i = 0; i < n; ++i) S += std::fabs((double)z[i]);\n  const T s = (T)(S / (double)n);", 1, 0),
    ("sign_of_zero_is_minus", "const bool b = (zi >= (T)0);", "const bool b = (zi > (T)0);", 1, 0),
    ("bits_packed_msb_first", "if (b) byte |= (1u << j);", "if (b) byte |= (1u << (7 - j));", 1, 0),
    ("error_added_instead_of_subtracted", "err[i + j] = zi - d;", "err[i + j] = zi + d;", 1, 0),
    ("decompress_sign_reversed", "out[i] = get_bit(bits, i) ? scale : -scale;",
     "out[i] = get_bit(bits, i) ? -scale : scale;", 1, 0),
    # the worker (lines 6-7, A.5.2)
    ("worker_drops_the_carried_error", "err[i] = k * mloc + err[i];", "err[i] = k * mloc;", 1, 0),
    ("worker_scales_the_error_too", "err[i] = k * mloc + err[i];", "err[i] = k * (mloc + err[i]);", 1, 0),
    ("worker_ignores_momentum_scale", "err[i] = k * mloc + err[i];", "err[i] = mloc + err[i];", 1, 0),
    ("worker_swaps_beta1_and_its_complement", "      const T mloc = beta1 * m[i] + omb1 * g[i];\n      err[i] = k",
     "      const T mloc = omb1 * m[i] + beta1 * g[i];\n      err[i] = k", 1, 0),
    ("worker_one_scale_for_the_whole_buffer", "compress_chunk<T>(err + c * n_c, n_c, bits + c * (n_c / 8), scales + c, err + c * n_c);",
     "{ if (c == 0) { compress_chunk<T>(err, n_pad, bits, scales, err); for (int32_t q = 1; q < W; ++q) scales[q] = scales[0]; } }", 1, 0),
    # the server (line 10)
    ("server_sums_workers_in_reverse", "for (int32_t w = 0; w < W; ++w) {\n      const T s = scales_in[w];",
     "for (int32_t w = W - 1; w >= 0; --w) {\n      const T s = scales_in[w];", 1, 0),
    ("server_input_element_major", "get_bit(bits_in + (int64_t)w * (n_c / 8), j)", "get_bit(bits_in, j * (int64_t)W + w)", 1, 0),
    ("server_drops_its_carried_error", "err_server[j] = acc * invW + err_server[j];", "err_server[j] = acc * invW;", 1, 0),
    ("server_sum_not_divided", "err_server[j] = acc * invW + err_server[j];", "err_server[j] = acc + err_server[j];", 1, 0),
    ("server_divides_each_term", "acc = acc + (get_bit(bits_in + (int64_t)w * (n_c / 8), j) ? s : -s);\n    }\n    err_server[j] = acc * invW + err_server[j];",
     "acc = acc + (get_bit(bits_in + (int64_t)w * (n_c / 8), j) ? s : -s) * invW;\n    }\n    err_server[j] = acc + err_server[j];", 1, 0),
    # the global momentum (line 13, A.5.2)
    ("momentum_multiplied_by_k", "mt[i] = mom_scale ? d / mom_scale[l] : d;", "mt[i] = mom_scale ? d * mom_scale[l] : d;", 1, 0),
    ("momentum_uses_first_chunk_scale", "const T s = server_scales[i / n_c];", "const T s = server_scales[0];", 1, 0),
    # ratio and coefficient (lines 15-20)
    ("gradient_drops_beta1", "const T gr = (mt[i] - beta1 * m[i]) / omb1;", "const T gr = (mt[i] - m[i]) / omb1;", 1, 0),
    ("gradient_not_divided", "const T gr = (mt[i] - beta1 * m[i]) / omb1;", "const T gr = (mt[i] - beta1 * m[i]);", 1, 0),
    ("variance_of_unsquared_gradient", "const T vf = beta2 * v_fresh[i] + omb2 * (gr * gr);", "const T vf = beta2 * v_fresh[i] + omb2 * gr;", 1, 0),
    ("variance_swaps_beta2_and_its_complement", "const T vf = beta2 * v_fresh[i] + omb2 * (gr * gr);",
     "const T vf = omb2 * v_fresh[i] + beta2 * (gr * gr);", 1, 0),
    ("fresh_variance_not_stored", "      v_fresh[i] = vf;\n", "", 1, 0),
    ("ratio_inverted", "const T q = v_frozen[i] / vf;", "const T q = vf / v_frozen[i];", 1, 0),
    ("ratio_of_square_roots", "const T q = v_frozen[i] / vf;", "const T q = std::sqrt(v_frozen[i]) / std::sqrt(vf);", 1, 0),
    ("ratio_is_minimum", "T r = (T)0;\n    for (int64_t i = off[l]; i < off[l + 1]; ++i) {\n      const T gr",
     "T r = (T)1e30;\n    for (int64_t i = off[l]; i < off[l + 1]; ++i) {\n      const T gr", 1, 0),
    ("ratio_is_minimum_b", "if (q > r) r = q;", "if (q < r) r = q;", 1, 0),
    ("clips_in_reverse_order", "r = clip<T>(r, lo, hi);       // line 18\n    r = clip<T>(r, r_min, r_max); // line 19",
     "r = clip<T>(r, r_min, r_max);\n    r = clip<T>(r, lo, hi);", 1, 0),
    ("threshold_additive", "const T lo = ((T)1 - r_thr) * r_prev[l];", "const T lo = r_prev[l] - r_thr;", 1, 0),
    ("threshold_upper_additive", "const T hi = ((T)1 + r_thr) * r_prev[l];", "const T hi = r_prev[l] + r_thr;", 1, 0),
    ("previous_ratio_not_committed", "    r_prev[l] = r;\n", "", 1, 0),
    ("coefficient_without_c_avg", "coeff_c[l] = r * c_avg[l];", "coeff_c[l] = r;", 1, 0),
    # the update (line 21)
    ("eta_inside_the_root", "const T u = mt[i] / (std::sqrt(v_frozen[i]) + eta);", "const T u = mt[i] / std::sqrt(v_frozen[i] + eta);", 1, 0),
    ("update_added", "x[i] = x[i] - a * u;", "x[i] = x[i] + a * u;", 1, 0),
    ("update_without_coefficient", "const T a = lr * coeff_c[l];", "const T a = lr;", 1, 0),
    ("momentum_not_committed", "      m[i] = mt[i];\n", "", 1, 0),
    # LAMB, eq. (1), and line 2
    ("lamb_momentum_swapped_weights", "m[i] = beta1 * m[i] + omb1 * g[i];", "m[i] = omb1 * m[i] + beta1 * g[i];", 1, 0),
    ("lamb_variance_of_unsquared_gradient", "v[i] = beta2 * v[i] + omb2 * (g[i] * g[i]);", "v[i] = beta2 * v[i] + omb2 * g[i];", 1, 0),
    ("lamb_eta_inside_the_root", "T ui = m[i] / (std::sqrt(v[i]) + eta);", "T ui = m[i] / std::sqrt(v[i] + eta);", 1, 0),
    ("lamb_weight_decay_subtracted", "ui = ui + wd * x[i];", "ui = ui - wd * x[i];", 1, 0),
    ("lamb_trust_ratio_inverted", "clip<T>(nx / nu, c_min, c_max)", "clip<T>(nu / nx, c_min, c_max)", 1, 0),
    ("lamb_norms_squared", "const T nx = (T)std::sqrt(Sx), nu = (T)std::sqrt(Su);", "const T nx = (T)Sx, nu = (T)Su;", 1, 0),
    ("lamb_x_norm_after_the_update", "Sx += (double)x[i] * (double)x[i];\n      Su", "Sx += (double)(x[i] - lr * ui) * (double)(x[i] - lr * ui);\n      Su", 1, 0),
    ("lamb_step_without_coefficient", "const T step = lr * c;", "const T step = lr;", 1, 0),
    ("lamb_c_avg_swapped_weights", "c_avg[l] = beta3 * c_avg[l] + omb3 * c;", "c_avg[l] = omb3 * c_avg[l] + beta3 * c;", 1, 0),
    ("clip_lets_nan_through", "T y = (x > a) ? x : a;", "T y = (x < a) ? a : x;", 1, 0),
    # A.5.2 (reading) and the padding rule
    ("momentum_scale_inverted", "(float)(mean / s)", "(float)(s / mean)", 1, 0),
    ("momentum_scale_of_squares", "return std::sqrt(S / (double)n);", "return S / (double)n;", 1, 0),
    ("momentum_scale_counts_empty_layers", "    if (off[l + 1] - off[l] <= 0) continue;\n", "", 1, 0),
    ("momentum_scale_zero_for_a_zero_layer", "(s > 0.0) ? (float)(mean / s) : 1.0f", "(s > 0.0) ? (float)(mean / s) : 0.0f", 1, 0),
    # the 16-bit formats of the mixed-precision variant (Section 6)
    ("lp_ties_away_from_zero", "double q = std::nearbyint(std::ldexp(a, F.fbits - ex));",
     "double q = std::round(std::ldexp(a, F.fbits - ex));", 1, 0),
    ("lp_truncates", "double q = std::nearbyint(std::ldexp(a, F.fbits - ex));",
     "double q = std::floor(std::ldexp(a, F.fbits - ex));", 1, 0),
    ("lp_overflow_saturates", "if (ex > emax) return sign | exp_all;", "if (ex > emax) return sign | (uint16_t)(exp_all - 1);", 1, 0),
    ("lp_subnormals_flushed", "else if (e == 0) v = std::ldexp((double)f, 1 - bias - F.fbits);", "else if (e == 0) v = 0.0;", 1, 0),
    ("lp_binary16_has_8_exponent_bits", "return fmt == 1 ? LpFormat{5, 10} : LpFormat{8, 7};", "return fmt == 1 ? LpFormat{8, 7} : LpFormat{5, 10};", 1, 0),
    ("lp_decode_ignores_the_scale", "out[i] = (float)lp_value(fmt, bits[i]) * scale;", "out[i] = (float)lp_value(fmt, bits[i]);", 1, 0),
    ("padding_to_32_per_worker", "const int64_t q = 256 * (int64_t)W;", "const int64_t q = 32 * (int64_t)W;", 1, 0),
]


def build_mutant(m, base):
    """Compile the copy of obref.cpp with mistake m = (name, old, new, count, which) planted, under
    the directory `base`; -> (name, path of the library)."""
    from oracle.build import FLAGS
    name, old, new, count, which = m
    text = open(SRC).read()
    assert text.count(old) == count, f"{name}: the text to replace occurs {text.count(old)} times, not {count}"
    parts = text.split(old)
    mutated = old.join(parts[:which + 1]) + new + old.join(parts[which + 1:])
    d = os.path.join(str(base), name)
    os.makedirs(d)
    shutil.copy(os.path.join(ROOT, "oracle", "obref.h"), os.path.join(d, "obref.h"))
    with open(os.path.join(d, "obref.cpp"), "w") as f:
        f.write(mutated)
    lib = os.path.join(d, "libobref_mutant.so")
    flags = [f for f in FLAGS if f != "-O2"] + ["-O1", "-w"]
    r = subprocess.run(["g++"] + flags + [os.path.join(d, "obref.cpp"), "-o", lib], capture_output=True, text=True)
    assert r.returncode == 0, f"{name}: the mutated copy does not compile:\n{r.stderr[-2000:]}"
    return name, lib


@pytest.fixture(scope="module")
def mutant_libs(tmp_path_factory):
    """name -> path of the library built from the mutated copy (all built up front, in parallel)."""
    base = tmp_path_factory.mktemp("mutants")
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        return dict(ex.map(lambda m: build_mutant(m, base), MUTANTS))


def run_pins(lib=None):
    env = dict(os.environ)
    env.pop("OBREF_LIB", None)
    if lib:
        env["OBREF_LIB"] = lib
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                           os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                          cwd=ROOT, env=env, capture_output=True, text=True)


def test_pins_pass_on_an_unmodified_copy(tmp_path):
    """The harness itself: a verbatim copy built the same way passes every pin."""
    from oracle.build import FLAGS
    shutil.copy(SRC, tmp_path / "obref.cpp")
    shutil.copy(os.path.join(ROOT, "oracle", "obref.h"), tmp_path / "obref.h")
    lib = str(tmp_path / "libobref_copy.so")
    flags = [f for f in FLAGS if f != "-O2"] + ["-O1", "-w"]
    subprocess.run(["g++"] + flags + [str(tmp_path / "obref.cpp"), "-o", lib], check=True)
    r = run_pins(lib)
    assert r.returncode == 0, r.stdout[-3000:]


@pytest.mark.parametrize("name", [m[0] for m in MUTANTS])
def test_a_pin_fails_on_the_mutant(mutant_libs, name):
    r = run_pins(mutant_libs[name])
    assert r.returncode == 1, (f"no pin noticed the planted mistake '{name}' (pytest exit {r.returncode}):\n"
                               + r.stdout[-1500:] + r.stderr[-500:])
    assert " failed" in r.stdout
