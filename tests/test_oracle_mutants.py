"""Planted-mistake check of the oracle pins (CPU only).

Each case rewrites one expression of the oracle source into a plausible mistake
(dropped term, wrong sign, wrong index, transposed layout, wrong gate), compiles
the mutant into a temporary library and runs the pin functions against it: at
least one pin must fail.  The mistakes are planted in the oracle, on the CPU.
"""
import os

import pytest

import oracle as O
import test_oracle_pins as P

MUTANTS = [
    ("mean_without_division", "sum = sum + s[static_cast<uint64_t>(m) * n + i];\n    return sum / static_cast<R>(M);",
     "sum = sum + s[static_cast<uint64_t>(m) * n + i];\n    return sum;"),
    ("mean_drops_a_worker", "for (int m = 1; m < M; ++m) sum = sum + s[", "for (int m = 2; m < M; ++m) sum = sum + s["),
    ("post_mean_drops_a_worker", "for (int m = 1; m < M; ++m) sum = sum + a[", "for (int m = 2; m < M; ++m) sum = sum + a["),
    ("mean_transposed_index", "sum = sum + s[static_cast<uint64_t>(m) * n + i];",
     "sum = sum + s[i * static_cast<uint64_t>(M) + m];"),
    ("adam_u_missing_one_minus_beta", "const R un = b1 * uin + omb1 * gh[m];\n                const R vn",
     "const R un = b1 * uin + gh[m];\n                const R vn"),
    ("adam_v_not_squared", "const R vn = b2 * vin + omb2 * (gh[m] * gh[m]);\n                u[k] = un;",
     "const R vn = b2 * vin + omb2 * gh[m];\n                u[k] = un;"),
    ("adam_step_sign", "x[k] = xin - adam_direction(c, s, un, vn);", "x[k] = xin + adam_direction(c, s, un, vn);"),
    ("adam_bias2_inside_root_wrong", "std::sqrt(vsel) / s.sbc2 + s.eps", "std::sqrt(vsel / s.sbc2) + s.eps"),
    ("adam_eps_inside_root", "std::sqrt(vsel) / s.sbc2 + s.eps", "std::sqrt(vsel / (s.sbc2 * s.sbc2) + s.eps)"),
    ("bias_exponent_off_by_one", "static_cast<double>(t) + 1.0", "static_cast<double>(t) + 2.0"),
    ("bias_betas_swapped", "const double bc1 = 1.0 - std::pow(static_cast<double>(s.b1), tp1);",
     "const double bc1 = 1.0 - std::pow(static_cast<double>(s.b2), tp1);"),
    ("adam_literal_lambda_not_squared", "std::sqrt(vsel + s.eps * s.eps)", "std::sqrt(vsel + s.eps)"),
    ("adopt_normaliser_uses_new_v", "const R root = std::sqrt(vnorm);", "const R root = std::sqrt(b2 * vin + omb2 * (gh[m] * gh[m]));"),
    ("adopt_multiplies_by_normaliser", "omb1 * (gh[m] / nrm)", "omb1 * (gh[m] * nrm)"),
    ("adopt_floor_is_min", "root > eps ? root : eps", "root < eps ? root : eps"),
    ("adopt_step_uses_old_momentum", "x[k] = xin - lr * mn;", "x[k] = xin - lr * uin;"),
    ("adopt_avg_normaliser_ignored", "(c->adopt_avg_normaliser && sv) ? vbar : vprev", "vprev"),
    ("adopt_init_moves_parameters", "u[k] = uin;\n                    x[k] = xin;", "u[k] = uin;\n                    x[k] = xin - lr * gh[m];"),
    ("sgdm_steps_along_gradient", "x[k] = xin - lr * un;\n                continue;", "x[k] = xin - lr * gh[m];\n                continue;"),
    ("sgdm_heavy_ball_form", "const R un = b1 * uin + omb1 * gh[m];\n                u[k] = un;\n                x[k] = xin - lr * un;",
     "const R un = b1 * uin + gh[m];\n                u[k] = un;\n                x[k] = xin - lr * un;"),
    ("clip_takes_max", "R c = a < rho ? a : rho;", "R c = a > rho ? a : rho;"),
    ("clip_loses_sign", "return std::copysign(c, g);", "return c;"),
    ("gate_u_sets_v_bit", "if (c->Ku != 0 && t % c->Ku == 0) mask |= 2u;", "if (c->Ku != 0 && t % c->Ku == 0) mask |= 4u;"),
    ("gate_x_uses_Ku", "if (c->Kx != 0 && t % c->Kx == 0) mask |= 1u;", "if (c->Kx != 0 && t % c->Ku == 0) mask |= 1u;"),
    ("gate_fires_one_step_late", "t % c->Kv == 0", "t % c->Kv == 1"),
    ("sgdm_gets_v_bit", "c->variant != ORACLE_SGDM && c->Kv != 0", "c->Kv != 0"),
    ("x_mean_taken_over_u", "sx ? worker_mean(x, n, i, M)", "sx ? worker_mean(u, n, i, M)"),
    ("v_gate_follows_u_gate", "const R vin = sv ? vbar : vprev;", "const R vin = su ? vbar : vprev;"),
    ("x_not_replaced_by_mean", "const R xin = sx ? xbar : x[k];", "const R xin = x[k];"),
    ("u_not_replaced_by_mean", "const R uin = su ? ubar : u[k];", "const R uin = u[k];"),
    ("gradient_of_wrong_worker", "const R gm = g[static_cast<uint64_t>(m) * n + i];",
     "const R gm = g[static_cast<uint64_t>(c->M - 1 - m) * n + i];"),
    ("sync_count_off_by_one", "for (uint64_t t = 0; t < T; ++t)\n        if (K != 0", "for (uint64_t t = 1; t <= T; ++t)\n        if (K != 0"),
    ("norm_without_sqrt", "const R nrm = static_cast<R>(std::sqrt(ss));", "const R nrm = static_cast<R>(ss);"),
    ("norm_scale_inverted", "gscale[m] = nrm > rho ? rho / nrm : static_cast<R>(1);", "gscale[m] = nrm > rho ? nrm / rho : static_cast<R>(1);"),
    ("norm_scale_always_applied", "gscale[m] = nrm > rho ? rho / nrm : static_cast<R>(1);", "gscale[m] = rho / nrm;"),
    ("norm_sum_not_squared", "ss += static_cast<double>(g[i]) * static_cast<double>(g[i]);", "ss += std::fabs(static_cast<double>(g[i]));"),
    ("norm_shared_across_workers", "double ss = sum_squares(g + static_cast<uint64_t>(m) * n, n);", "double ss = sum_squares(g, n);"),
    ("norm_mode_also_clips_coordinates", "gh[m] = c->norm_clip ? gm * gscale[m] : clip_coord(gm, rho);", "gh[m] = c->norm_clip ? clip_coord(gm * gscale[m], rho * static_cast<R>(0.25)) : clip_coord(gm, rho);"),
    ("norm_rest_ignored", "if (sumsq_rest) ss += sumsq_rest[m];", ""),
    ("post_mean_taken_before_update", "for (int m = 0; m < M; ++m) un[m] = b1 * u[static_cast<uint64_t>(m) * n + i] + omb1 * gh[m];\n        if (su) {\n            const R ubar = mean_of(un, M);",
     "for (int m = 0; m < M; ++m) un[m] = b1 * u[static_cast<uint64_t>(m) * n + i] + omb1 * gh[m];\n        if (su) {\n            for (int m = 0; m < M; ++m) un[m] = u[static_cast<uint64_t>(m) * n + i];\n            const R ubar = b1 * mean_of(un, M) + omb1 * gh[0];"),
    ("post_x_mean_skips_the_step", "xl[m] = x[k] - d;", "xl[m] = sx ? x[k] : x[k] - d;"),
    ("post_v_gate_uses_u_gate", "if (sv) {\n                const R vbar = mean_of(vn, M);", "if (su) {\n                const R vbar = mean_of(vn, M);"),
    ("amsgrad_takes_min", "vsel = vn[m] > prev ? vn[m] : prev;", "vsel = vn[m] < prev ? vn[m] : prev;"),
    ("amsgrad_max_not_stored", "vmax[k] = vsel;", ""),
    ("amsgrad_overwrites_v", "v[k] = vn[m];\n            } else {\n                d = lr * un[m];", "v[k] = vsel;\n            } else {\n                d = lr * un[m];"),
    ("post_mean_drops_division", "sum = sum + a[m];\n    return sum / static_cast<R>(M);", "sum = sum + a[m];\n    return sum;"),
    ("bf16_widen_wrong_half", "static_cast<uint32_t>(h) << 16", "static_cast<uint32_t>(h)"),
    ("change_is_a_sum_not_a_difference", "dd += (a - b) * (a - b);\n            rr += b * b;\n        }\n        change[m]",
     "dd += (a + b) * (a + b);\n            rr += b * b;\n        }\n        change[m]"),
    ("change_base_from_current_state", "rr += b * b;\n        }\n        change[m]", "rr += a * a;\n        }\n        change[m]"),
    ("change_without_root", "change[m] = static_cast<float>(std::sqrt(dd));", "change[m] = static_cast<float>(dd);"),
    ("change_shared_across_workers", "const double a = static_cast<double>(s[static_cast<uint64_t>(m) * n + i]);\n            const double b = static_cast<double>(ref[static_cast<uint64_t>(m) * n + i]);\n            dd += (a - b) * (a - b);\n            rr += b * b;\n        }\n        change[m]",
     "const double a = static_cast<double>(s[i]);\n            const double b = static_cast<double>(ref[static_cast<uint64_t>(m) * n + i]);\n            dd += (a - b) * (a - b);\n            rr += b * b;\n        }\n        change[m]"),
    ("tensor_change_offset_not_advanced", "        start += numel[k];\n", ""),
    ("tensor_change_transposed_output", "change[k * static_cast<uint64_t>(M) + m] = ", "change[m * n_tensors + k] = "),
    ("tensor_change_base_from_current_state", "rr += b * b;\n            }\n            change[k", "rr += a * a;\n            }\n            change[k"),
    ("tensor_change_range_one_short", "i < start + numel[k]; ++i", "i + 1 < start + numel[k]; ++i"),
    ("tensor_change_reads_with_tensor_stride", "for (uint64_t i = start; i < start + numel[k]; ++i) {\n                const double a = static_cast<double>(s[static_cast<uint64_t>(m) * n + i]);",
     "for (uint64_t i = start; i < start + numel[k]; ++i) {\n                const double a = static_cast<double>(s[static_cast<uint64_t>(m) * numel[k] + i]);"),
]


def _pins():
    """A compact, fast list of pin calls covering every part of the oracle."""
    calls = [
        (P.test_sync_count_closed_form, dict(T=65, K=16)),
        (P.test_sync_count_closed_form, dict(T=64, K=3)),
        (P.test_never_period, {}),
        (P.test_every_gate_fires_at_t0, {}),
        (P.test_full_sync_instants_are_multiples_of_lcm, dict(Ks=(2, 3, 5))),
        (P.test_full_sync_instants_are_multiples_of_lcm, dict(Ks=(6, 4, 9))),
        (P.test_paper_communication_ratios, {}),
        (P.test_benchmark_config_sync_counts, dict(variant=O.SGDM, T=512, Ks=(16, 64, 0), expect=(32, 8, 0))),
        (P.test_half_life_of_the_moment_emas, dict(beta=0.95, key="half_life_beta_0.95")),
        (P.test_adam_reduces_to_torch_adam, dict(M=1, Ks=(3, 5, 7))),
        (P.test_adam_reduces_to_torch_adam, dict(M=4, Ks=(3, 5, 7))),
        (P.test_sgdm_reduces_to_torch_sgd, dict(M=4, Ks=(5, 2, 0))),
        (P.test_adopt_reduces_to_textbook_adopt, dict(M=1, Ks=(3, 4, 5), init_g0sq=True)),
        (P.test_adopt_reduces_to_textbook_adopt, dict(M=4, Ks=(2, 7, 3), init_g0sq=False)),
        (P.test_adam_constant_gradient_closed_form, dict(c=0.3, M=4, Ks=(3, 5, 2))),
        (P.test_adam_literal_constant_gradient_closed_form, {}),
        (P.test_sgdm_constant_gradient_closed_form, {}),
        (P.test_adopt_constant_gradient_closed_form, {}),
        (P.test_adopt_literal_first_step_divides_by_eps, {}),
        (P.test_adopt_normaliser_is_floored_at_eps, {}),
        (P.test_clip_is_coordinatewise_sign_preserving, dict(variant=O.ADAM)),
        (P.test_sync_step_replaces_previous_state_by_worker_mean, dict(variant=O.ADAM)),
        (P.test_sync_step_replaces_previous_state_by_worker_mean, dict(variant=O.SGDM)),
        (P.test_sgdm_averaged_iterates_follow_centralised_sgdm, dict(M=3)),
        (P.test_adaptive_averaged_moments_follow_mean_dynamics, dict(variant=O.ADAM)),
        (P.test_adaptive_averaged_moments_follow_mean_dynamics, dict(variant=O.ADOPT)),
        (P.test_post_sync_workers_differ_only_by_their_last_local_step, {}),
        (P.test_clip_bounds_of_the_max_change_lemma, {}),
        (P.test_worker_mean_fixed_order_and_preserved, {}),
        (P.test_bf16_widening_is_exact, {}),
    ]
    calls += [
        (P.test_norm_clip_matches_torch_clip_grad_norm_then_adam, {}),
        (P.test_norm_clip_constant_gradient_closed_form, {}),
        (P.test_norm_clip_inactive_below_the_bound_and_per_worker, {}),
        (P.test_norm_clip_subset_with_rest_equals_whole, {}),
        (P.test_norm_clip_brute_force, dict(variant=O.ADAM, M=3, Ks=(2, 3, 4))),
        (P.test_norm_clip_brute_force, dict(variant=O.SGDM, M=4, Ks=(2, 3, 0))),
    ]
    calls += [
        (P.test_post_average_sgdm_with_Kx1_Ku_never_is_minibatch_sgdm, {}),
        (P.test_post_average_workers_identical_after_sync_and_mean_dynamics, dict(variant=O.ADAM)),
        (P.test_post_average_differs_from_pre_average_only_in_ordering, {}),
        (P.test_amsgrad_matches_torch_amsgrad, {}),
        (P.test_amsgrad_literal_direction_and_local_max, {}),
        (P.test_post_average_brute_force, dict(variant=O.ADAM, M=4, Ks=(3, 2, 5), ams=True, lit=True)),
        (P.test_post_average_brute_force, dict(variant=O.SGDM, M=3, Ks=(2, 3, 0), ams=False, lit=False)),
    ]
    calls += [
        (P.test_state_change_matches_numpy_norms, {}),
        (P.test_state_change_of_a_decaying_moment_is_one_minus_beta_to_the_K, dict(beta=0.9, K=16)),
        (P.test_state_change_per_tensor_matches_numpy_norms, {}),
        (P.test_state_change_per_tensor_of_a_decaying_moment, {}),
    ]
    calls += [(P.test_brute_force_generic_listing, dict(variant=v, flags=f, M=M, Ks=Ks))
              for v, f, M, Ks in P.BRUTE_CASES]
    return calls


def test_pins_pass_on_the_unmodified_oracle(orc):
    for fn, kw in _pins():
        fn(orc, **kw)


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    src = open(O.SOURCE).read()
    assert src.count(old) == 1, f"mutation site for {name} must be unique, found {src.count(old)}"
    mutant_src = tmp_path / "mutant.cpp"
    mutant_src.write_text(src.replace(old, new))
    lib = str(tmp_path / f"libmutant_{name}.so")
    O.build(source=str(mutant_src), library=lib, extra_flags=("-Wno-unused-parameter", "-Wno-unused-variable",
                                                              "-Wno-unused-but-set-variable", "-Wno-error"))
    mutant = O.Oracle(lib)
    killed_by = None
    for fn, kw in _pins():
        try:
            with_np_err = __import__("numpy").errstate(all="ignore")
            with with_np_err:
                fn(mutant, **kw)
        except (AssertionError, ZeroDivisionError, ValueError, OverflowError):
            killed_by = fn.__name__
            break
    assert killed_by is not None, f"no pin notices the planted mistake '{name}'"
    assert os.path.exists(lib)
