"""Planted mistakes for the oracle (CPU only): each entry rewrites one expression of one oracle function.

tests/test_oracle_pins_catch_mistakes.py runs the oracle's pin tests once per entry, with the mistake
planted, and expects them to fail: the pins are only worth something if a plausible slip anywhere in the
oracle (a dropped term, a wrong sign or index, a swapped bound) is caught by one of them.  The mistake is
planted in the oracle's source text at import time of the test session (see conftest.py) when the
environment variable PG_ORACLE_MUTANT names an entry; nothing here ever touches the GPU path."""
import inspect
import textwrap

# name -> (oracle function, expression as written, planted replacement)
MUTANTS = {
    "returns_discount_off_by_one": ("returns", "g ** (tp - t)", "g ** (tp - t + 1)"),
    "returns_sums_from_the_first_turn": ("returns", "for tp in range(t, Tm):", "for tp in range(0, Tm):"),
    "reward_cap_missing": ("reward_eq1", "np.minimum(np.asarray(speedup, dtype=np.float64), cap)",
                           "np.asarray(speedup, dtype=np.float64)"),
    "trloo_divides_by_n": ("trloo_advantage", "others / (len(members) - 1)", "others / len(members)"),
    "trloo_baseline_includes_self": ("trloo_advantage", "if j != i:", "if True:"),
    "trloo_ignores_validity": ("trloo_advantage", "members = [k for k in range(K) if valid[p, k, t]]",
                               "members = list(range(K))"),
    "grpo_leaves_one_out": ("grpo_advantage", "sum(G[p, j, t] for j in members) / len(members)",
                            "sum(G[p, j, t] for j in members) / max(1, len(members) - 1)"),
    "temperature_multiplies": ("logits", "(H @ W.T) / _f32(tau)", "(H @ W.T) * _f32(tau)"),
    "entropy_sign": ("logprob_entropy_from_logits", "ent = lse - (p * z).sum(axis=1)", "ent = lse + (p * z).sum(axis=1)"),
    "logsumexp_without_max_shift_term": ("logprob_entropy_from_logits", "lse = (M + np.log(s))[:, 0]", "lse = np.log(s)[:, 0]"),
    "logp_of_the_wrong_token": ("logprob_entropy_from_logits", "z[np.arange(z.shape[0]), y] - lse",
                                "z[np.arange(z.shape[0]), (y + 1) % z.shape[1]] - lse"),
    "merge_drops_rescaling_of_u": ("merge_softmax_partials", "u = a1 * (u + (m - mm) * s) + a2 * (u2 + (m2 - mm) * s2)",
                                   "u = a1 * u + a2 * u2"),
    "shard_merge_takes_max_of_zy": ("merge_shard_partials", "a1 * (u1 + (m1 - m) * s1) + a2 * (u2 + (m2 - m) * s2), z1 + z2)",
                                    "a1 * (u1 + (m1 - m) * s1) + a2 * (u2 + (m2 - m) * s2), max(z1, z2))"),
    "shard_state_ignores_offset": ("head_shard_partials", "yl = y[t] - v_offset", "yl = y[t]"),
    "mrs_arithmetic_mean_of_ratios": ("mismatch_weights", "w = np.exp(d.sum() / len(idx))", "w = np.exp(d).sum() / len(idx)"),
    "mrs_mean_over_all_rows": ("mismatch_weights", "idx = idx[loss_mask[idx]]", "idx = idx"),
    "mrs_veto_inclusive": ("mismatch_weights", "np.exp(d.min()) < veto", "np.exp(d.min()) <= veto"),
    "mrs_window_open": ("mismatch_weights", "(_f32(prm.geo_lo) <= w) and (w <= _f32(prm.geo_hi))",
                        "(_f32(prm.geo_lo) < w) and (w < _f32(prm.geo_hi))"),
    "veto_rejects_the_whole_batch": ("mismatch_weights", "keep[s] = in_window and not vetoed", "keep[:] = in_window and not vetoed"),
    "truncation_uses_max": ("mismatch_weights", "c[idx] = np.minimum(ratio, _f32(prm.trunc_c))", "c[idx] = np.maximum(ratio, _f32(prm.trunc_c))"),
    "surrogate_max_instead_of_min": ("surrogate", "-np.minimum(r * A, np.clip(r, lo, hi) * A)", "-np.maximum(r * A, np.clip(r, lo, hi) * A)"),
    "surrogate_clip_bounds_swapped": ("surrogate", "lo, hi = 1.0 - _f32(prm.clip_eps_lo), 1.0 + _f32(prm.clip_eps_hi)",
                                      "lo, hi = 1.0 - _f32(prm.clip_eps_hi), 1.0 + _f32(prm.clip_eps_lo)"),
    "surrogate_gradient_ignores_clip": ("surrogate", "g = np.where(flows, -A * r, 0.0)", "g = -A * r"),
    "dS_sign": ("pg_loss_fwd_bwd", "dS = -p * (coef / tau)[:, None]", "dS = p * (coef / tau)[:, None]"),
    "dS_without_onehot": ("pg_loss_fwd_bwd", "dS[np.arange(len(r_)), y[r_]] += coef / tau", "pass"),
    "dS_forgets_temperature": ("pg_loss_fwd_bwd", "dS = -p * (coef / tau)[:, None]", "dS = -p * coef[:, None]"),
    "coef_without_mismatch_weight": ("pg_loss_fwd_bwd", "coef = c[r_] * g / norm", "coef = g / norm"),
    "normaliser_counts_all_loss_rows": ("pg_loss_fwd_bwd", "float(max(1, n_active))", "float(max(1, int(loss_mask.sum())))"),
    "dW_from_the_wrong_rows": ("pg_loss_fwd_bwd", "dW += dS.T @ H[r_]", "dW += dS.T @ H[:len(r_)]"),
    "advantage_of_the_wrong_segment": ("pg_loss_fwd_bwd", "A_tok[cu[s]:cu[s + 1]] = float(adv_seg[s])",
                                       "A_tok[cu[s]:cu[s + 1]] = float(adv_seg[(s + 1) % S])"),
    "dropped_segment_keeps_its_rows": ("drop_filtered_segments", "mask[cu[s]:cu[s + 1]] = False", "pass"),
    "sft_gradient_sign": ("sft_ce_fwd_bwd", "dS = p / (norm * tau)", "dS = -p / (norm * tau)"),
    "sft_loss_not_negated": ("sft_ce_fwd_bwd", "total += float(-lp.sum())", "total += float(lp.sum())"),
    "reward_pr_for_incorrect_kernels": ("turn_reward", "pr = np.where(C > 0, profiling_ratio(t_generated, t_total), 0.0)",
                                        "pr = profiling_ratio(t_generated, t_total)"),
    "profiling_ratio_inverted": ("profiling_ratio", "np.asarray(t_generated, np.float64) / np.asarray(t_total, np.float64)",
                                 "np.asarray(t_total, np.float64) / np.asarray(t_generated, np.float64)"),
    "prs_probability_unclipped": ("prs_probability", "np.clip((pr - _f32(tau)) / _f32(s), 0.0, 1.0)", "(pr - _f32(tau)) / _f32(s)"),
    "prs_keeps_when_above": ("prs_retain", "prs_uniform(i, seed) < p[i]", "prs_uniform(i, seed) > p[i]"),
    "philox_key_schedule": ("philox4x32_10", "k0 = (k0 + _PHILOX_W0) & 0xFFFFFFFF", "k0 = (k0 + _PHILOX_W1) & 0xFFFFFFFF"),
    "philox_nine_rounds": ("philox4x32_10", "for _ in range(10):", "for _ in range(9):"),
    "monitor_ppl_sign": ("monitors", 'out["ppl_train"] = float(np.exp(-np.asarray(logp_train, np.float64)[m].sum() / den))',
                         'out["ppl_train"] = float(np.exp(np.asarray(logp_train, np.float64)[m].sum() / den))'),
    "monitor_norm_not_rooted": ("monitors", 'float(np.sqrt((np.asarray(dW, np.float64) ** 2).sum()))', 'float(((np.asarray(dW, np.float64) ** 2).sum()))'),
    "rmsnorm_eps_outside_root": ("rmsnorm_fwd", "1.0 / np.sqrt((X * X).mean(axis=1) + _f32(eps))", "1.0 / (np.sqrt((X * X).mean(axis=1)) + _f32(eps))"),
    "rmsnorm_bwd_drops_projection": ("rmsnorm_bwd", "dX = rstd[:, None] * (gg - xhat * ((gg * xhat).sum(axis=1) / d)[:, None])",
                                     "dX = rstd[:, None] * gg"),
    "rmsnorm_dgamma_uses_x": ("rmsnorm_bwd", "dgamma = (dH * xhat).sum(axis=0)", "dgamma = (dH * X).sum(axis=0)"),
}


def plant(oracle_module, name: str) -> None:
    """Re-defines one oracle function with the named mistake in it (in the module's own namespace, so every
    caller inside and outside the module sees it)."""
    fn_name, old, new = MUTANTS[name]
    src = textwrap.dedent(inspect.getsource(getattr(oracle_module, fn_name)))
    assert src.count(old) >= 1, f"mutant {name}: the oracle no longer contains {old!r}; update the mutant"
    exec(compile(src.replace(old, new, 1), f"<mutant {name}>", "exec"), oracle_module.__dict__)
