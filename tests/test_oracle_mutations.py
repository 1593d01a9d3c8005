"""Mutation check of the oracle's pins, on the CPU.

Each case plants ONE plausible mistake in a private copy of the oracle's source (a dropped term, a wrong
sign or index, a transposed operand, a misplaced constant), loads that copy as a module of its own, points
the pin tests at it and requires that at least one pin fails.  The drift guard against the stored oracle
output is excluded: a mutant has to be caught by something other than the oracle itself.  Nothing here
touches the GPU or the HIP path; the real oracle module is never modified.
"""
import inspect
import os
import types

import pytest

import test_oracle_pins as pins

ORACLE_SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "dp_oracle.py")

# (name, [(old, new, which occurrence or None = must be unique)], pin expected to notice it first)
MUTANTS = [
    ("dense_weight_grad_transposed", [("gW = A_i.T @ G_i", "gW = (G_i.T @ A_i) if A_i.shape[1] == G_i.shape[1] else A_i.T @ G_i", None)],
     "test_dense_orientation"),
    ("dense_bias_grad_is_mean", [("gb = G_i.sum(axis=0)", "gb = G_i.mean(axis=0)", None)], "test_autograd_bruteforce_tiny_bert"),
    ("dense_norm_drops_bias", [("        if has_bias:\n            n[i] += np.sum(gb * gb)", "        if False:\n            n[i] += np.sum(gb * gb)", None)],
     "test_dense_T1_closed_form"),
    ("dense_norm_not_squared", [("n[i] = np.sum(gW * gW)", "n[i] = np.sum(np.abs(gW))", None)], "test_dense_T1_closed_form"),
    ("layernorm_gain_without_xhat", [("return (G_i * X_i).sum(axis=0), G_i.sum(axis=0)", "return G_i.sum(axis=0), G_i.sum(axis=0)", None)],
     "test_autograd_bruteforce_tiny_bert"),
    ("layernorm_norm_drops_offset", [("n[i] = np.sum(gg * gg) + np.sum(gb * gb)", "n[i] = np.sum(gg * gg)", None)],
     "test_autograd_bruteforce_tiny_bert"),
    ("embedding_repeated_ids_overwrite", [("R[inv[t]] += G_i[t]", "R[inv[t]] = G_i[t]", None)], "test_embedding_counts_and_index_add"),
    ("embedding_no_range_check", [('raise IndexError("token id out of range")', "pass", None)], "test_embedding_rejects_out_of_range"),
    ("tied_drops_output_projection", [("        g += np.outer(dL_i[m], H_i[m])", "        pass", None)], "test_tied_embedding_against_autograd"),
    ("tied_output_projection_sign", [("        g += np.outer(dL_i[m], H_i[m])", "        g -= np.outer(dL_i[m], H_i[m])", None)],
     "test_tied_embedding_special_cases_and_cross_term"),
    ("tied_outer_product_transposed", [("np.outer(dL_i[m], H_i[m])", "(np.outer(H_i[m], dL_i[m]) if dL_i.shape[1] == H_i.shape[1] else np.outer(dL_i[m], H_i[m]))", None)],
     "test_tied_embedding_square_table"),
    ("tied_norms_add_instead_of_norm_of_sum", [("        g = tied_embedding_example_grad(ids[i], dY[i], H[i], dL[i])\n        n[i] = np.sum(g * g)",
                                                "        g = tied_embedding_example_grad(ids[i], dY[i], H[i], np.zeros_like(dL[i]))\n"
                                                "        h = tied_embedding_example_grad(ids[i], np.zeros_like(dY[i]), H[i], dL[i])\n"
                                                "        n[i] = np.sum(g * g) + np.sum(h * h)", None)],
     "test_tied_embedding_against_autograd"),
    ("tied_sum_unweighted", [("S_E += c[i] * tied_embedding_example_grad", "S_E += tied_embedding_example_grad", None)],
     "test_tied_embedding_special_cases_and_cross_term"),
    ("clip_uses_squared_norm", [("float(C) / np.sqrt(n[pos])", "float(C) / n[pos]", None)], "test_clip_invariant_and_all_clipped"),
    ("clip_without_min", [("np.minimum(1.0, float(C) / np.sqrt(n[pos]))", "float(C) / np.sqrt(n[pos])", None)], "test_clip_noop_equals_flat_gemm"),
    ("clip_zero_gradient_gets_zero", [("c = np.ones_like(n)", "c = np.zeros_like(n)", None)], "test_clip_zero_gradient_gets_factor_one"),
    ("dense_sum_unweighted", [("S_W += c[i] * gW", "S_W += gW", None)], "test_clip_mixed_branches"),
    ("dense_bias_sum_unweighted", [("S_b += c[i] * gb", "S_b += gb", 0)], "test_clip_mixed_branches"),
    ("dense_entries_unweighted", [("out += c[i] * entry_i", "out += entry_i", None)], "test_sampled_entries_equal_full_sum"),
    ("layernorm_sum_unweighted", [("S_g += c[i] * gg", "S_g += gg", None)], "test_autograd_bruteforce_tiny_bert"),
    ("embedding_sum_unweighted", [("S_E[rows] += c[i] * R", "S_E[rows] += R", None)], "test_autograd_bruteforce_tiny_bert"),
    ("global_norm_is_max_over_layers", [("                n_i += float(np.sum(g * g))", "                n_i = max(n_i, float(np.sum(g * g)))", 1)],
     "test_autograd_bruteforce_tiny_bert"),
    ("microbatch_norms_skip_embedding", [("                if isinstance(g, tuple):\n                    g = g[1]\n                n_i += float(np.sum(g * g))",
                                         "                if isinstance(g, tuple):\n                    continue\n                n_i += float(np.sum(g * g))", 0)],
     "test_autograd_bruteforce_tiny_bert"),
    ("microbatch_embedding_rows_unweighted", [("dst[rows] += c_i * R", "dst[rows] += R", None)], "test_autograd_bruteforce_tiny_bert"),
    ("microbatch_restarts_sums", [("                    dst += c_i * g", "                    dst[...] = c_i * g", None)],
     "test_accumulation_is_linear_over_microbatches"),
    ("philox_multipliers_swapped", [("p0 = _M0 * c0\n        p1 = _M1 * c2", "p0 = _M1 * c0\n        p1 = _M0 * c2", None)],
     "test_philox_against_bigint_and_inverse"),
    ("philox_nine_rounds", [("for r in range(10):", "for r in range(9):", None)], "test_philox_against_bigint_and_inverse"),
    ("philox_key_not_advanced", [("k0 = (k0 + _W0) & _MASK", "k0 = k0 & _MASK", None)], "test_philox_against_bigint_and_inverse"),
    ("philox_round_output_order", [("c0, c1, c2, c3 = (hi1 ^ c1 ^ k0), lo1, (hi0 ^ c3 ^ k1), lo0", "c0, c1, c2, c3 = (hi0 ^ c1 ^ k0), lo0, (hi1 ^ c3 ^ k1), lo1", None)],
     "test_philox_against_bigint_and_inverse"),
    ("philox_step_in_wrong_counter_word", [("j & _MASK, j >> _S32, np.uint64(step & 0xFFFFFFFF), np.uint64((step >> 32) & 0xFFFFFFFF)",
                                           "j & _MASK, np.uint64(step & 0xFFFFFFFF), j >> _S32, np.uint64((step >> 32) & 0xFFFFFFFF)", None)],
     "test_philox_mapping_and_slicing"),
    ("philox_seed_high_word_dropped", [("seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF", "seed & 0xFFFFFFFF, 0", None)], "test_philox_mapping_and_slicing"),
    ("philox_offset_ignored_within_block", [("    s = elem_offset - 4 * first\n    return words[s:s + n]", "    return words[:n]", None)],
     "test_philox_mapping_and_slicing"),
    ("uniform_24_bits", [("(np.asarray(r, dtype=np.uint32) >> np.uint32(9)).astype(np.float64) + 0.5) * (2.0 ** -23)",
                          "(np.asarray(r, dtype=np.uint32) >> np.uint32(8)).astype(np.float64) + 0.5) * (2.0 ** -24)", None)],
     "test_uniforms_exact_in_fp32_and_open_interval"),
    ("uniform_closed_at_zero", [(".astype(np.float64) + 0.5) * (2.0 ** -23)", ".astype(np.float64) + 0.0) * (2.0 ** -23)", None)],
     "test_uniforms_exact_in_fp32_and_open_interval"),
    ("box_muller_sin_cos_swapped", [("np.stack([rho * np.cos(ang), rho * np.sin(ang)], axis=1)", "np.stack([rho * np.sin(ang), rho * np.cos(ang)], axis=1)", None)],
     "test_box_muller_structure"),
    ("box_muller_radius_without_factor_two", [("rho = np.sqrt(-2.0 * np.log(u[:, 0]))", "rho = np.sqrt(-1.0 * np.log(u[:, 0]))", None)],
     "test_normal_moments_and_ks"),
    ("box_muller_half_turn", [("ang = 2.0 * np.pi * u[:, 1]", "ang = np.pi * u[:, 1]", None)], "test_normal_moments_and_ks"),
    ("box_muller_radius_from_odd_word", [("rho = np.sqrt(-2.0 * np.log(u[:, 0]))\n    ang = 2.0 * np.pi * u[:, 1]",
                                         "rho = np.sqrt(-2.0 * np.log(u[:, 1]))\n    ang = 2.0 * np.pi * u[:, 0]", None)],
     "test_box_muller_structure"),
    ("noise_std_without_clip_norm", [("g = (S + sigma * C * z) / float(batch_size)", "g = (S + sigma * z) / float(batch_size)", None)],
     "test_noise_scale_on_the_mean_gradient"),
    ("noise_not_divided_by_batch", [("g = (S + sigma * C * z) / float(batch_size)", "g = S / float(batch_size) + sigma * C * z", None)],
     "test_noise_scale_on_the_mean_gradient"),
    ("noise_variance_instead_of_std", [("g = (S + sigma * C * z) / float(batch_size)", "g = (S + sigma * sigma * C * C * z) / float(batch_size)", None)],
     "test_noise_scale_on_the_mean_gradient"),
    ("adam_eps_inside_sqrt", [("np.sqrt(v_hat) + eps", "np.sqrt(v_hat + eps)", None)], "test_adamw_hand_worked_element"),
    ("adam_no_first_moment_correction", [("m_hat = m_new / (1.0 - beta1 ** step)", "m_hat = m_new", None)], "test_adamw_matches_torch_optim_five_steps"),
    ("adam_second_moment_corrected_with_beta1", [("v_hat = v_new / (1.0 - beta2 ** step)", "v_hat = v_new / (1.0 - beta1 ** step)", None)],
     "test_adamw_matches_torch_optim_five_steps"),
    ("adam_second_moment_not_squared", [("(1.0 - beta2) * g * g", "(1.0 - beta2) * np.abs(g)", None)], "test_adamw_matches_torch_optim_five_steps"),
    ("adam_moment_weights_swapped", [("m_new = beta1 * m + (1.0 - beta1) * g", "m_new = (1.0 - beta1) * m + beta1 * g", None)],
     "test_adamw_matches_torch_optim_five_steps"),
    ("decay_not_scaled_by_lr", [("theta - lr * (m_hat / (np.sqrt(v_hat) + eps) + wd * theta)", "theta - lr * (m_hat / (np.sqrt(v_hat) + eps)) - wd * theta", None)],
     "test_adamw_zero_gradient_is_pure_decay"),
    ("decay_coupled_into_gradient", [("    m_new = beta1 * m", "    g = g + wd * theta\n    m_new = beta1 * m", None),
                                     ("+ eps) + wd * theta)", "+ eps))", None)], "test_adamw_matches_torch_optim_five_steps"),
    ("decay_sign_flipped", [("+ eps) + wd * theta)", "+ eps) - wd * theta)", None)], "test_adamw_zero_gradient_is_pure_decay"),
    ("snr_signal_not_squared", [("signal_sq = float(np.sum(S * S))", "signal_sq = float(np.sum(np.abs(S)))", None)], "test_gradient_snr_closed_forms"),
    ("snr_noise_without_clip_norm", [("noise = sigma * C * normals(S.shape[0], elem_offset, seed, step)", "noise = sigma * normals(S.shape[0], elem_offset, seed, step)", None)],
     "test_gradient_snr_closed_forms"),
    ("snr_noise_ignores_offset", [("noise = sigma * C * normals(S.shape[0], elem_offset, seed, step)", "noise = sigma * C * normals(S.shape[0], 0, seed, step)", None)],
     "test_gradient_snr_noise_is_what_the_update_adds"),
    ("snr_noise_from_another_step", [("noise = sigma * C * normals(S.shape[0], elem_offset, seed, step)", "noise = sigma * C * normals(S.shape[0], elem_offset, seed, 1)", None)],
     "test_gradient_snr_noise_is_what_the_update_adds"),
    ("snr_ratio_of_squares", [("return float(np.sqrt(signal_sq / noise_sq)) if noise_sq > 0", "return float(signal_sq / noise_sq) if noise_sq > 0", None)],
     "test_gradient_snr_closed_forms"),
    ("snr_inverted", [("return float(np.sqrt(signal_sq / noise_sq)) if noise_sq > 0", "return float(np.sqrt(noise_sq / signal_sq)) if noise_sq > 0", None)],
     "test_gradient_snr_closed_forms"),
    ("batch_schedule_jump_one_step_early", [("    done = step - 1\n", "    done = step\n", None)], "test_batch_size_schedule_reproduces_the_papers_numbers"),
    ("batch_schedule_linear_ramp", [("k = min(n_increments, (done * n_increments) // ramp_steps)", "k = min(n_increments, (done * n_increments) / ramp_steps)", None)],
     "test_batch_size_schedule_reproduces_the_papers_numbers"),
    ("batch_schedule_never_reaches_end", [("    if k == n_increments:\n        return b_end\n", "", None)], "test_batch_size_schedule_general_and_errors"),
    ("lr_decay_linear", [("return peak * frac * frac", "return peak * frac", None)], "test_lr_schedule_shape"),
    ("lr_warmup_lags_one_step", [("return peak * step / warmup_steps", "return peak * (step - 1) / warmup_steps", None)], "test_lr_schedule_shape"),
    ("lr_decay_measured_from_step_zero", [("frac = (total_steps - step) / (total_steps - warmup_steps)", "frac = (total_steps - step) / total_steps", None)],
     "test_lr_schedule_shape"),
    ("rdp_divides_by_alpha", [("return float(total.ln() / (alpha - 1))", "return float(total.ln() / alpha)", None)], "test_rdp_closed_forms"),
    ("rdp_exponent_k_squared_plus_k", [("Decimal(k * k - k) / (2 * sd * sd)", "Decimal(k * k + k) / (2 * sd * sd)", None)], "test_rdp_closed_forms"),
    ("rdp_exponent_without_the_half", [("Decimal(k * k - k) / (2 * sd * sd)", "Decimal(k * k - k) / (sd * sd)", None)], "test_rdp_closed_forms"),
    ("rdp_binomial_weights_dropped", [("Decimal(comb(alpha, k)) * power(1 - qd, alpha - k)", "power(1 - qd, alpha - k)", None)], "test_rdp_closed_forms"),
    ("rdp_conversion_divides_by_alpha", [("eps = rdp + math.log(1.0 / delta) / (alpha - 1)", "eps = rdp + math.log(1.0 / delta) / alpha", None)],
     "test_rdp_epsilon_composition_over_a_batch_size_schedule"),
    ("rdp_composition_ignores_step_counts", [("rdp = sum(n * rdp_sampled_gaussian(qq, sigma, alpha) for qq, n in zip(q, steps))", "rdp = sum(rdp_sampled_gaussian(qq, sigma, alpha) for qq, n in zip(q, steps))", None)],
     "test_rdp_epsilon_composition_over_a_batch_size_schedule"),
    ("sigma_search_returns_the_end_that_misses", [("        else:\n            lo = mid\n    return hi", "        else:\n            lo = mid\n    return lo", None)],
     "test_rdp_noise_multiplier_inverts_the_guarantee"),
    ("sigma_search_bisects_the_wrong_way", [("        if eps_of(mid) <= eps_target:\n            hi = mid", "        if eps_of(mid) > eps_target:\n            hi = mid", None)],
     "test_rdp_noise_multiplier_inverts_the_guarantee"),
    ("sigma_search_stops_at_the_first_bracket", [("    while hi - lo > rel_tol * hi:", "    while hi - lo > 0.25 * hi:", None)],
     "test_rdp_noise_multiplier_inverts_the_guarantee"),
    ("rdp_takes_the_worst_order", [("        if eps < best[0]:\n            best = (eps, alpha)", "        if eps > best[0] or best[1] == 0:\n            best = (eps, alpha)", None)],
     "test_rdp_epsilon_composition_over_a_batch_size_schedule"),
    ("bf16_widening_shift", [("<< np.uint32(16)", "<< np.uint32(15)", None)], "test_bf16_widening_matches_torch"),
]

EXCLUDED = {"test_oracle_matches_its_stored_reference"}


def _replace(src, old, new, which):
    n = src.count(old)
    assert n >= 1, f"mutation site not found: {old!r}"
    if which is None:
        assert n == 1, f"mutation site not unique ({n}x): {old!r}"
        return src.replace(old, new)
    parts = src.split(old)
    assert which < n
    return old.join(parts[: which + 1]) + new + old.join(parts[which + 1:])


def _mutant_module(name, edits):
    src = open(ORACLE_SRC).read()
    for old, new, which in edits:
        src = _replace(src, old, new, which)
    mod = types.ModuleType(f"oracle_mutant_{name}")
    mod.__file__ = ORACLE_SRC
    exec(compile(src, f"<oracle mutant {name}>", "exec"), mod.__dict__)
    return mod


def _pin_calls():
    """Every pin test as a list of (label, zero-argument callable); parametrised ones once per parameter set."""
    calls = []
    for name, fn in inspect.getmembers(pins, inspect.isfunction):
        if not name.startswith("test_") or name in EXCLUDED:
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            calls.append((name, fn))
            continue
        assert len(marks) == 1
        argnames, values = marks[0].args
        argnames = [a.strip() for a in argnames.split(",")] if isinstance(argnames, str) else list(argnames)
        for val in values:
            val = val if isinstance(val, (tuple, list)) and len(argnames) > 1 else (val,)
            calls.append((f"{name}[{val}]", (lambda f=fn, kw=dict(zip(argnames, val)): f(**kw))))
    return calls


def _first_failure(calls, hint):
    ordered = sorted(calls, key=lambda c: not c[0].startswith(hint))
    for label, call in ordered:
        try:
            call()
        except (Exception, pytest.fail.Exception) as e:  # an assertion, or the mutant raising / not raising where the pin expects
            return label, e
    return None, None


def test_unmutated_copy_passes_every_pin(monkeypatch):
    """The harness itself: an unmodified copy of the source passes all pins."""
    monkeypatch.setattr(pins, "orc", _mutant_module("identity", []))
    label, err = _first_failure(_pin_calls(), "")
    assert label is None, (label, err)


@pytest.mark.parametrize("name,edits,hint", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(monkeypatch, name, edits, hint):
    monkeypatch.setattr(pins, "orc", _mutant_module(name, edits))
    label, err = _first_failure(_pin_calls(), hint)
    assert label is not None, f"no pin notices the planted mistake '{name}'"
