"""The pins must be able to fail: each plausible mistake planted in a copy of the oracle's C
source (on the CPU, in a temporary build) has to be caught by at least one pin."""
import os
import subprocess

import pytest

import oracle
import test_oracle_ext as ext_pins
import test_oracle_plan as plan_pins
import test_oracle_step as step_pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "se_oracle.c")

MUTANTS = {
    "sign of the learning-rate term": ("xhat[r] = fmaf(-lr, vn, params[idx]);", "xhat[r] = fmaf(lr, vn, params[idx]);"),
    "momentum operands transposed": ("vn = fmaf(mu, momentum[idx], gg);", "vn = fmaf(mu, gg, momentum[idx]);"),
    "momentum term dropped": ("vn = fmaf(mu, momentum[idx], gg);", "vn = gg;"),
    "momentum not written back": ("                    momentum[idx] = vn;\n                } else {\n                    vn = gg;",
                                  "                } else {\n                    vn = gg;"),
    "learning rate applied to g instead of v'": ("xhat[r] = fmaf(-lr, vn, params[idx]);", "xhat[r] = fmaf(-lr, gg, params[idx]);"),
    "mean not scaled": ("mean = sum_in_order(xhat, m) * inv_m;", "mean = sum_in_order(xhat, m);"),
    "scaled by groups instead of group size": ("inv_m = 1.0f / (float)m;", "inv_m = 1.0f / (float)k;"),
    "mean written to the first member only": ("params[(int64_t)mem[r] * pitch + e] = mean;", "params[(int64_t)mem[0] * pitch + e] = mean;"),
    "first member counted twice": ("float part = val[b];", "float part = val[b] + (b == 0 ? val[0] : 0.0f);"),
    # --- the summation order
    "plain left-to-right sum": ("#define ORACLE_BLOCK 8", "#define ORACLE_BLOCK 4096"),
    "blocks of 7": ("#define ORACLE_BLOCK 8", "#define ORACLE_BLOCK 7"),
    "blocks of 9": ("#define ORACLE_BLOCK 8", "#define ORACLE_BLOCK 9"),
    "blocks of 4": ("#define ORACLE_BLOCK 8", "#define ORACLE_BLOCK 4"),
    "block sums added last to first": ("for (b = 0; b < m; b += ORACLE_BLOCK) {\n        float part = val[b];",
                                       "for (b = (m - 1) / ORACLE_BLOCK * ORACLE_BLOCK; b >= 0; b -= ORACLE_BLOCK) {\n        float part = val[b];"),
    "first block sum restarted by the second": ("total = (b == 0) ? part : total + part;", "total = (b <= ORACLE_BLOCK) ? part : total + part;"),
    "last member of a block dropped": ("for (r = b + 1; r < m && r < b + ORACLE_BLOCK; ++r)", "for (r = b + 1; r < m && r < b + ORACLE_BLOCK - 1; ++r)"),
    "unfused multiply-add": ("xhat[r] = fmaf(-lr, vn, params[idx]);", "xhat[r] = params[idx] + (-lr * vn);"),
    "groups cut by remainder": ("group_of[i] = below / m;", "group_of[i] = below % (n / m);"),
    "hash shift": ("z ^= z >> 15;", "z ^= z >> 13;"),
    "hash skips the iteration word": ("w[2] = (uint32_t)(t & 0xFFFFFFFFu);", "w[2] = 0;"),
    "ring mean not scaled": ("gbar = sum_in_order(gcol, n) * inv_n;", "gbar = sum_in_order(gcol, n);"),
    "ring reads worker 0 in place of the last worker": ("gcol[i] = load_grad(grads, grads_are_bf16, (int64_t)i * pitch + e);",
                                                         "gcol[i] = load_grad(grads, grads_are_bf16, (int64_t)(i == n - 1 ? 0 : i) * pitch + e);"),
    "ring update sign": ("params[idx] = fmaf(-lr, vn, params[idx]);", "params[idx] = fmaf(lr, vn, params[idx]);"),
    # --- the extended functions
    "decay sign (corrected form)": ("float d = (wd != 0.0f) ? fmaf(wd, params[idx], gg) : gg;",
                                    "float d = (wd != 0.0f) ? fmaf(-wd, params[idx], gg) : gg;"),
    "decay applied to the gradient, not the parameter": ("float d = (wd != 0.0f) ? fmaf(wd, params[idx], gg) : gg;",
                                                         "float d = (wd != 0.0f) ? fmaf(wd, gg, gg) : gg;"),
    "decay dropped in the gradient-averaging form": ("float d = (wd != 0.0f) ? fmaf(wd, params[idx], gbar) : gbar;",
                                                     "float d = gbar;"),
    "gradient mean not scaled": ("gbar = sum_in_order(val, m) * inv_m;", "gbar = sum_in_order(val, m);"),
    "gradient-averaging form averages parameters too": ("                    params[idx] = fmaf(-lr, vn, params[idx]);\n                }\n            } else {",
                                                        "                    params[idx] = fmaf(-lr, vn, params[(int64_t)mem[0] * pitch + e]);\n                }\n            } else {"),
    "global average skips the last worker": ("mean = sum_in_order(xcol, n) * inv_n;", "mean = sum_in_order(xcol, n - (n > 1)) * inv_n;"),
    "consensus uses the sum as the mean": ("mean = s / (double)n;", "mean = s;"),
    "consensus forgets the square": ("d += t * t;", "d += t;"),
    "ring time drops the latency term": ("(layer_bytes / ((double)workers * nu) + t_tau)", "(layer_bytes / ((double)workers * nu))"),
    "handshakes count one direction only": ("return (long)layers * 2L * (long)(workers - 1);", "return (long)layers * (long)(workers - 1);"),
}


def battery(golden_dir):
    """A fast subset of the pins; returns the names of those that fail."""
    checks = [
        ("worked example", lambda: step_pins.test_worked_example_by_hand(golden_dir)),
        ("sign/operand", step_pins.test_sign_and_operand_order_are_observable),
        ("brute n=2", lambda: step_pins.test_brute_force_exact_rational(2)),
        ("brute n=4", lambda: step_pins.test_brute_force_exact_rational(4)),
        ("summation order by hand", lambda: step_pins.test_summation_order_examples_by_hand(golden_dir)),
        ("brute n=20, m=10", lambda: step_pins.test_brute_force_exact_rational_for_groups_of_more_than_eight(20, 10)),
        ("ring brute n=17", lambda: step_pins.test_ring_brute_force_exact_rational_for_more_than_eight_workers(17)),
        ("ring brute n=5", lambda: step_pins.test_ring_brute_force_exact_rational(5)),
        ("conservation", step_pins.test_conservation_of_the_all_worker_sum),
        ("consensus", step_pins.test_members_of_a_group_end_bit_identical),
        ("torch sgd", step_pins.test_group_size_one_is_the_library_sgd_optimizer),
        ("ring = torch", step_pins.test_full_group_is_ring_sgd_is_library_sgd_on_the_mean_gradient),
        ("no-momentum", step_pins.test_no_momentum_buffer_equals_zero_mu_with_zero_buffer),
        ("partition n=4", lambda: plan_pins.test_partition_brute_force_small_n(4)),
        ("keys", plan_pins.test_keys_match_independent_python_implementation),
        ("seed/iter dependence", plan_pins.test_same_seed_same_plan_and_seed_matters),
        ("ex = basic", ext_pins.test_general_step_reduces_to_the_basic_step),
        ("grad-avg = ring", ext_pins.test_gradient_averaging_over_all_workers_is_ring_sgd),
        ("ex brute n=4", lambda: ext_pins.test_general_step_against_exact_rational_brute_force(4)),
        ("decay = torch", ext_pins.test_weight_decay_is_the_library_optimizer_convention),
        ("global average", ext_pins.test_global_average_pins),
        ("consensus", ext_pins.test_consensus_closed_forms),
        ("cost model", ext_pins.test_cost_model_numbers_of_the_paper),
    ]
    failed = []
    for name, fn in checks:
        try:
            fn()
        except Exception:            # AssertionError or an oracle error raised by the mutant
            failed.append(name)
    return failed


def test_unmutated_oracle_passes_the_battery(golden_dir):
    assert battery(golden_dir) == []


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name, tmp_path, monkeypatch, golden_dir):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, f"pattern for '{name}' not found in the oracle source"
    mutated = text.replace(old, new, 1)
    c_path, so_path = tmp_path / "mutant.c", tmp_path / "mutant.so"
    c_path.write_text(mutated)
    subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-shared", "-fPIC", "-o", str(so_path),
                    str(c_path), "-lm"], check=True)
    monkeypatch.setattr(oracle, "_lib_handle", oracle.bind(str(so_path)))
    failed = battery(golden_dir)
    assert failed, f"no pin noticed: {name}"
