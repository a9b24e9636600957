"""Would the GPU parity tests notice if the device and the oracle disagreed?

Each case plants ONE mistake in a scratch copy of the ORACLE (on the CPU, as in
tests/test_oracle_mutants.py -- the device code is never modified), then runs a selection of
tests/test_gpu_parity.py against that copy in a child process: the selection must fail, i.e. the
comparison is sharp enough to tell the (correct) device result from the (now wrong) expected one.
Every mistake of tests/test_oracle_mutants.py has a case here, except the ones listed in
NOT_REACHED with the reason.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

from tests.test_oracle_mutants import MUTANTS, ROOT, build_mutant

PH = "test_phasewise_single_step and "
WU = "test_warmup_and_freeze and 0.0- and "
# planted mistake -> -k selection of tests/test_gpu_parity.py that has to fail
SELECT = {
    "scale_divides_by_n_minus_1": PH + "small",
    "scale_is_mean_absolute_value": PH + "small",
    "sign_of_zero_is_minus": "test_degenerate_values and tiny",
    "bits_packed_msb_first": PH + "odd",
    "error_added_instead_of_subtracted": PH + "w1",
    "worker_drops_the_carried_error": PH + "small",
    "worker_scales_the_error_too": PH + "bert_mini",
    "worker_ignores_momentum_scale": PH + "bert_mini",
    "worker_swaps_beta1_and_its_complement": PH + "tiny",
    "worker_one_scale_for_the_whole_buffer": PH + "small",
    "server_sums_workers_in_reverse": "test_server_sum_order_and_single_division",
    "server_divides_each_term": "test_server_sum_order_and_single_division",
    "server_input_element_major": "test_server_reduce_forms and 300000-3-1",
    "server_drops_its_carried_error": "test_server_reduce_forms and 300000-3-1",
    "server_sum_not_divided": "test_server_reduce_forms and 300000-3-1",
    "momentum_multiplied_by_k": PH + "bert_mini",
    "momentum_uses_first_chunk_scale": PH + "tiny",
    "gradient_drops_beta1": PH + "tiny",
    "gradient_not_divided": PH + "tiny",
    "variance_of_unsquared_gradient": PH + "tiny",
    "variance_swaps_beta2_and_its_complement": PH + "tiny",
    "fresh_variance_not_stored": PH + "tiny",
    "ratio_inverted": PH + "tiny",
    "ratio_of_square_roots": "test_trajectory and tiny-10-False-False",
    "ratio_is_minimum": PH + "tiny",
    "ratio_is_minimum_b": PH + "tiny",
    "clips_in_reverse_order": "test_previous_ratio_outside_its_bounds",
    "threshold_additive": "test_previous_ratio_outside_its_bounds",
    "threshold_upper_additive": "test_previous_ratio_outside_its_bounds",
    "previous_ratio_not_committed": "test_trajectory and tiny-10-False-False",
    "coefficient_without_c_avg": PH + "tiny",
    "eta_inside_the_root": PH + "small",
    "update_added": PH + "small",
    "update_without_coefficient": PH + "small",
    "momentum_not_committed": PH + "small",
    "lamb_momentum_swapped_weights": WU + "small",
    "lamb_variance_of_unsquared_gradient": WU + "small",
    "lamb_eta_inside_the_root": WU + "small",
    "lamb_weight_decay_subtracted": "test_warmup_and_freeze and 0.01 and small",
    "lamb_trust_ratio_inverted": WU + "small",
    "lamb_norms_squared": WU + "small",
    "lamb_x_norm_after_the_update": WU + "tiny",
    "lamb_step_without_coefficient": WU + "small",
    "lamb_c_avg_swapped_weights": WU + "small",
    "clip_lets_nan_through": "test_warmup_and_freeze and odd",
    "momentum_scale_inverted": "test_momentum_scale_generation and odd",
    "momentum_scale_of_squares": "test_momentum_scale_generation and odd",
    "momentum_scale_counts_empty_layers": "test_momentum_scale_generation and odd",
    "momentum_scale_zero_for_a_zero_layer": "test_momentum_scale_generation",
    "lp_ties_away_from_zero": "test_mixed_precision_variant and bert_mini",
    "lp_truncates": "test_mixed_precision_variant and bert_mini",
    "lp_overflow_saturates": "test_mixed_precision_variant",
    "lp_subnormals_flushed": "test_mixed_precision_variant",
    "lp_binary16_has_8_exponent_bits": "test_mixed_precision_variant and bert_mini",
    "lp_decode_ignores_the_scale": "test_mixed_precision_variant and bert_mini",
}
NOT_REACHED = {
    "padding_to_32_per_worker": "the parity tests size their buffers with workloads.shapes.padded_len and check that the "
                                "device agrees with it; obref_padded_len serves the pins",
    "decompress_sign_reversed": "obref_decompress_chunk serves the pins only; the step decodes through obref_global_momentum",
}


def test_every_planted_mistake_has_a_case():
    names = {m[0] for m in MUTANTS}
    assert names == set(SELECT) | set(NOT_REACHED)
    assert not set(SELECT) & set(NOT_REACHED)


@pytest.fixture(scope="module")
def children(tmp_path_factory):
    """name -> finished child process; four at a time (each builds its scratch copy of the oracle
    with g++, then runs its selection of the parity tests on the GPU)."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    base = tmp_path_factory.mktemp("wrong_oracles")
    by_name = {m[0]: m for m in MUTANTS}

    def run(name):
        _, lib = build_mutant(by_name[name], base)
        env = dict(os.environ, OBREF_LIB=lib)
        return name, subprocess.run(
            [sys.executable, "-m", "pytest", "-x", "-q", "-m", "gpu", "-p", "no:cacheprovider", "-k", SELECT[name],
             os.path.join(ROOT, "tests", "test_gpu_parity.py")],
            cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    with ThreadPoolExecutor(max_workers=4) as ex:
        return dict(ex.map(run, sorted(SELECT)))


@pytest.mark.gpu
@pytest.mark.parametrize("name", sorted(SELECT))
def test_gpu_parity_fails_against_a_wrong_oracle(children, name):
    r = children[name]
    assert r.returncode == 1 and " failed" in r.stdout, (
        f"the selection '{SELECT[name]}' did not notice the oracle's planted mistake '{name}' "
        f"(pytest exit {r.returncode}):\n" + r.stdout[-1500:] + r.stderr[-500:])
