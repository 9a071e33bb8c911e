"""Every plausible mistake planted in the oracle must trip at least one pin.

The mistakes are planted on the CPU, in a patched copy of the oracle's C source
compiled to a temporary library; the real oracle is untouched.
"""
import os

import pytest

import oracle
from oracle_pins import ALL_PINS

SRC = open(os.path.join(os.path.dirname(oracle.__file__), "linattn_oracle.c")).read()

# (name, text in the source, replacement)
MUTANTS = [
    ("phi_drops_plus_one", "x > 0.0 ? x + 1.0 : exp(x)", "x > 0.0 ? x : exp(x)"),
    ("phi_branch_flipped", "x > 0.0 ? x + 1.0 : exp(x)", "x < 0.0 ? x + 1.0 : exp(x)"),
    ("quadratic_excludes_diagonal", "for (int i = 0; i <= t; ++i) {", "for (int i = 0; i < t; ++i) {"),
    ("quadratic_not_causal", "for (int i = 0; i <= t; ++i) {", "for (int i = 0; i < L; ++i) {"),
    ("quadratic_den_drops_z0", "if (z0) den += dot(fqt, z0, d);", ""),
    ("quadratic_S0_transposed", "num[c] += fqt[i] * S0[(size_t)i * d + c];", "num[c] += fqt[i] * S0[(size_t)c * d + i];"),
    ("quadratic_uses_raw_q", "fq[e] = oracle_phi(q[e]);", "fq[e] = q[e];"),
    ("quadratic_uses_raw_k", "fk[e] = oracle_phi(k[e]);", "fk[e] = k[e];"),
    ("quadratic_S_out_transposed", "s += fk[(size_t)t * d + i] * v[(size_t)t * d + c];",
     "s += fk[(size_t)t * d + c] * v[(size_t)t * d + i];"),
    ("quadratic_eps_dropped", "double den = eps;", "double den = 0.0;"),
    ("conv_reads_the_future", "vext_row(v, hist, Kc, d, t - j);\n        if (row) acc", "vext_row(v, hist, Kc, d, t + j < L ? t + j : t);\n        if (row) acc"),
    ("conv_window_excludes_current", "vext_row(v, hist, Kc, d, t - j);\n        if (row) acc", "vext_row(v, hist, Kc, d, t - j - 1);\n        if (row) acc"),
    ("conv_hist_reversed", "return hist + (size_t)(Kc - 1 + s) * d;", "return hist + (size_t)(-s - 1) * d;"),
    ("conv_weights_of_wrong_head", "conv_head(L, d, Kc, v + (size_t)bh * L * d, w + (size_t)h * d * Kc,",
     "conv_head(L, d, Kc, v + (size_t)bh * L * d, w + (size_t)(bh / H) * d * Kc,"),
    ("hist_after_off_by_one", "int s = n - Hn + r; /* index into the extended sequence */", "int s = n - Hn + r - 1;"),
    ("step_state_after_readout", "z[i] += fk;", "z[i] += (i == 0 ? 0.5 : 1.0) * fk;"),
    ("step_drops_z_update", "z[i] += fk;", ""),
    ("step_S_transposed_readout", "num += fq[i] * S[(size_t)i * d + c];", "num += fq[i] * S[(size_t)c * d + i];"),
    ("step_S_transposed_update", "S[(size_t)i * d + c] += fk * v[c];", "S[(size_t)c * d + i] += fk * v[c];"),
    ("step_eps_dropped", "double den = dot(fq, z, d) + eps;", "double den = dot(fq, z, d);"),
    ("step_hist_taps_reversed", "hist[(size_t)(Kc - 1 - j) * d + c];", "hist[(size_t)(j - 1) * d + c];"),
    ("step_hist_not_shifted", "if (Kc > 1) memcpy(hist + (size_t)(Kc - 2) * d, v, sizeof(double) * d);",
     "if (Kc > 1) memcpy(hist, v, sizeof(double) * d);"),
    ("step_uses_raw_q", "fq[i] = oracle_phi(q[i]);", "fq[i] = q[i];"),
    ("verify_commits_one_late", "if (j + 1 == n) {", "if (j == n) {"),
    ("verify_commits_everything", "int n = n_commit ? n_commit[b] : kk;", "int n = kk; (void)b;"),
    ("verify_n_commit_per_head", "int n = n_commit ? n_commit[b] : kk;", "int n = n_commit ? n_commit[h % B] : kk; (void)b;"),
    ("recurrent_ignores_incoming_hist", "hist0 ? hist0 + bh * nh : NULL, S, z, hs);", "NULL, S, z, hs);"),
    ("relu_keeps_negatives", "if (g_feature_map == 1) return x > 0.0 ? x : 0.0;", "if (g_feature_map == 1) return x;"),
    ("relu_adds_one", "if (g_feature_map == 1) return x > 0.0 ? x : 0.0;", "if (g_feature_map == 1) return x > 0.0 ? x + 1.0 : 0.0;"),
    ("relu_setting_ignored", "void oracle_set_feature_map(int kind) { g_feature_map = kind; }", "void oracle_set_feature_map(int kind) { (void)kind; }"),
    ("tree_sees_the_stored_neighbour", "for (int a = i; a >= 0; a = parent[a]) path[len++] = a;\n      const double *fqi",
     "for (int a = i; a >= 0; a = a - 1) path[len++] = a;\n      const double *fqi"),
    ("tree_excludes_the_candidate_itself", "for (int a = i; a >= 0; a = parent[a]) path[len++] = a;\n      const double *fqi",
     "for (int a = parent[i]; a >= 0; a = parent[a]) path[len++] = a;\n      const double *fqi"),
    ("tree_den_drops_z", "for (int f = 0; f < d; ++f) den += fqi[f] * zh[f];", ""),
    ("tree_S_transposed", "acc += fqi[f] * Sh[(size_t)f * d + c];", "acc += fqi[f] * Sh[(size_t)c * d + f];"),
    ("tree_window_runs_forward", "double x = t < len ? vh[(size_t)path[t] * d + c]", "double x = t < len ? vh[(size_t)path[len - 1 - t] * d + c]"),
    ("tree_history_off_by_one", ": hh[(size_t)(Kc - 1 - (t - len + 1)) * d + c];", ": hh[(size_t)(Kc - 1 - (t - len + 1) > 0 ? Kc - 2 - (t - len + 1) : 0) * d + c];"),
    ("tree_commits_newest_first_hist", "const double *src = back <= len ? vh + (size_t)path[back - 1] * d",
     "const double *src = back <= len ? vh + (size_t)path[len - back] * d"),
    ("tree_commit_skips_the_root", "for (int m = len - 1; m >= 0; --m) { /* oldest first */", "for (int m = len - 2; m >= 0; --m) {"),
    ("tree_accept_per_head", "int acc_node = accept ? accept[b] : -1;", "int acc_node = accept ? accept[h % B] : -1; (void)b;"),
    ("tree_uses_raw_k", "fk[e] = oracle_phi(kh[e]);", "fk[e] = kh[e];"),
    ("grouped_local_not_causal", "for (int i = g0; i <= t; ++i)", "for (int i = g0; i < g1; ++i)"),
    ("grouped_logit_scale_dropped", "dot(qt, k + (size_t)i * d, d) * inv_sqrt_d;", "dot(qt, k + (size_t)i * d, d);"),
    ("grouped_logit_scale_is_1_over_d", "const double inv_sqrt_d = 1.0 / sqrt((double)d);", "const double inv_sqrt_d = 1.0 / (double)d;"),
    ("grouped_largest_logit_not_taken_out", "logit[i - g0] = exp(logit[i - g0] - top);", "logit[i - g0] = exp(logit[i - g0]);"),
    ("grouped_alpha_on_the_local_branch", "alpha * glob + loc / mass", "glob + alpha * loc / mass"),
    ("grouped_local_not_normalised", "alpha * glob + loc / mass", "alpha * glob + loc"),
    ("grouped_sums_skip_a_groups_first_token", "for (int t = g0; t < g1; ++t)\n      for (int i = 0; i < d; ++i) {\n        double fk = oracle_phi(k[",
     "for (int t = g0 + 1; t < g1; ++t)\n      for (int i = 0; i < d; ++i) {\n        double fk = oracle_phi(k["),
    ("grouped_normaliser_counts_own_group", "any token of this group */\n      double gden = dot(fq, z, d) + eps;",
     "any token of this group */\n      double gden = dot(fq, z, d) + eps; for (int i2 = g0; i2 < t; ++i2) for (int f = 0; f < d; ++f) gden += fq[f] * oracle_phi(k[(size_t)i2 * d + f]);"),
    ("grouped_linear_branch_uses_raw_q", "fq[i] = oracle_phi(qt[i]);", "fq[i] = qt[i];"),
    ("grouped_local_branch_uses_phi_q", "logit[i - g0] = dot(qt, k + (size_t)i * d, d) * inv_sqrt_d;", "logit[i - g0] = dot(fq, k + (size_t)i * d, d) * inv_sqrt_d;"),
    ("grouped_eps_dropped", "double gden = dot(fq, z, d) + eps;", "double gden = dot(fq, z, d);"),
    ("grouped_S_transposed", "gnum += fq[i] * S[(size_t)i * d + c];", "gnum += fq[i] * S[(size_t)c * d + i];"),
    ("grouped_ignores_incoming_state", "load_state(d, Kc, S0, z0, hist0, S, z, hs);", "load_state(d, Kc, NULL, NULL, hist0, S, z, hs);"),
    ("grouped_conv_dropped", "alpha * glob + loc / mass + u[(size_t)t * d + c];", "alpha * glob + loc / mass;"),
    ("grouped_state_uses_raw_k", "double fk = oracle_phi(k[(size_t)t * d + i]);", "double fk = k[(size_t)t * d + i];"),
    ("gstep_token_not_in_its_own_window", "for (int r = 0; r <= n; ++r)", "for (int r = 0; r < n; ++r)"),
    ("gstep_closed_group_misses_its_last_token", "for (int r = 0; r < C; ++r)\n      for (int i = 0; i < d; ++i) {\n        double fk = oracle_phi(kwin",
     "for (int r = 0; r < C - 1; ++r)\n      for (int i = 0; i < d; ++i) {\n        double fk = oracle_phi(kwin"),
    ("gstep_closed_group_missing_from_z", "double fk = oracle_phi(kwin[(size_t)r * d + i]);\n        z[i] += fk;", "double fk = oracle_phi(kwin[(size_t)r * d + i]);"),
    ("gstep_closed_group_uses_raw_k", "double fk = oracle_phi(kwin[(size_t)r * d + i]);", "double fk = kwin[(size_t)r * d + i];"),
    ("gstep_window_not_restarted", "    n = 0;\n  }\n  *fill = n;", "    n = 1;\n  }\n  *fill = n;"),
    ("gstep_local_branch_uses_phi_q", "wt[r] = dot(q, kwin + (size_t)r * d, d) * inv_sqrt_d;", "wt[r] = dot(fq, kwin + (size_t)r * d, d) * inv_sqrt_d;"),
    ("gstep_alpha_on_the_local_branch", "alpha * (gden != 0.0 ? gnum / gden : 0.0) + loc / mass + u", "(gden != 0.0 ? gnum / gden : 0.0) + alpha * loc / mass + u"),
    ("gstep_S_transposed", "for (int i = 0; i < d; ++i) gnum += fq[i] * S[(size_t)i * d + c];\n    for (int r = 0; r <= n; ++r) loc",
     "for (int i = 0; i < d; ++i) gnum += fq[i] * S[(size_t)c * d + i];\n    for (int r = 0; r <= n; ++r) loc"),
    ("gverify_fill_not_advanced", "if (h == 0) fill_after[b] = fw;", "if (h == 0) fill_after[b] = fill[b];"),
    ("gverify_window_not_written_back", "memcpy(kwin + bh * nw, kw, sizeof(double) * nw);", ""),
    ("gverify_commits_everything", "int n = n_commit ? n_commit[b] : kk;\n    size_t o = (size_t)bh * kk * d;\n    double *Sw = (double *)malloc(sizeof(double) * nS);\n    double *zw = (double *)malloc(sizeof(double) * (size_t)d);\n    double *hw = (double *)malloc(sizeof(double) * (nh ? nh : 1));\n    double *kw",
     "int n = kk;\n    size_t o = (size_t)bh * kk * d;\n    double *Sw = (double *)malloc(sizeof(double) * nS);\n    double *zw = (double *)malloc(sizeof(double) * (size_t)d);\n    double *hw = (double *)malloc(sizeof(double) * (nh ? nh : 1));\n    double *kw"),
    ("recurrent_ignores_incoming_S", "load_state(d, Kc, S0 ? S0 + bh * nS : NULL, z0", "load_state(d, Kc, NULL, z0"),
    # the gradient of the three-branch form
    ("gbwd_denominator_gradient_sign", "double dden = -alpha * nd / (gden * gden);", "double dden = alpha * nd / (gden * gden);"),
    ("gbwd_denominator_not_squared", "double dden = -alpha * nd / (gden * gden);", "double dden = -alpha * nd / gden;"),
    ("gbwd_numerator_gradient_drops_alpha", "dnum[c] = alpha * dot_[c] / gden;", "dnum[c] = dot_[c] / gden;"),
    ("gbwd_query_gradient_drops_the_z_term", "double dfq = z[i] * dden;", "double dfq = 0.0;"),
    ("gbwd_dz_dropped", "gz[i] += fq[i] * dden;", ""),
    ("gbwd_dS_transposed", "gS[(size_t)i * d + c] += fq[i] * dnum[c];", "gS[(size_t)c * d + i] += fq[i] * dnum[c];"),
    ("gbwd_dq_drops_the_maps_derivative", "dq[(size_t)t * d + i] += dfq * dphi(qt[i]);", "dq[(size_t)t * d + i] += dfq;"),
    ("gbwd_dk_drops_the_maps_derivative", "dk[(size_t)t * d + i] += dfk * dphi(kti);", "dk[(size_t)t * d + i] += dfk;"),
    ("gbwd_derivative_of_elu_is_one", "return x > 0.0 ? 1.0 : exp(x);", "return 1.0;"),
    ("gbwd_derivative_of_relu_is_one", "if (g_feature_map == 1) return x > 0.0 ? 1.0 : 0.0;", "if (g_feature_map == 1) return 1.0;"),
    ("gbwd_later_groups_gradient_dropped", "for (size_t e = 0; e < nS; ++e) DS[e] += gS[e];", "for (size_t e = 0; e < nS; ++e) DS[e] = gS[e];"),
    ("gbwd_key_gradient_drops_dz", "double dfk = DZ[i];", "double dfk = 0.0;"),
    ("gbwd_value_gradient_from_sums_transposed", "dv[(size_t)t * d + c] += fk * DS[(size_t)i * d + c];", "dv[(size_t)t * d + c] += fk * DS[(size_t)c * d + i];"),
    ("gbwd_softmax_drops_the_mean_term", "double dl = p[i - g0] * (dp[i - g0] - pbar);", "double dl = p[i - g0] * dp[i - g0];"),
    ("gbwd_local_dq_drops_the_logit_scale", "dq[(size_t)t * d + f] += dl * k[(size_t)i * d + f] * inv_sqrt_d;", "dq[(size_t)t * d + f] += dl * k[(size_t)i * d + f];"),
    ("gbwd_local_dk_uses_the_key", "dk[(size_t)i * d + f] += dl * qt[f] * inv_sqrt_d;", "dk[(size_t)i * d + f] += dl * k[(size_t)i * d + f] * inv_sqrt_d;"),
    ("gbwd_local_weights_not_normalised", "p[i - g0] /= mass;", ""),
    ("gbwd_conv_taps_reversed", "dv[(size_t)s2 * d + c] += w[(size_t)c * Kc + j] * go;", "dv[(size_t)s2 * d + c] += w[(size_t)c * Kc + (Kc - 1 - j)] * go;"),
    ("gbwd_dw_of_one_batch_row_only", "dw[(size_t)(bh % H) * nw + e] += dw_bh[(size_t)bh * nw + e];", "dw[(size_t)(bh % H) * nw + e] = dw_bh[(size_t)bh * nw + e];"),
    ("gbwd_dw_misses_the_history", "dw[(size_t)c * Kc + j] += go * hist0[(size_t)(Kc - 1 + s2) * d + c];", ""),
    ("gbwd_dhist_reversed", "dhist0[(size_t)(Kc - 1 + s2) * d + c] += w", "dhist0[(size_t)(-s2 - 1) * d + c] += w"),
    ("gbwd_gradient_into_the_final_state_ignored", "if (dS1) memcpy(DS, dS1, sizeof(double) * nS);", ""),
    ("gbwd_queries_read_their_own_groups_sums", "const double *S = Sg + (size_t)g * nS, *z = zg + (size_t)g * d;",
     "const double *S = Sg + (size_t)(g + 1) * nS, *z = zg + (size_t)(g + 1) * d;"),
    ("gbwd_empty_denominator_not_skipped", "      if (gden != 0.0) {\n        double nd = 0.0;", "      {\n        double nd = 0.0;"),
]


def _run_pins(lib):
    failed = []
    for pin in ALL_PINS:
        try:
            pin(lib)
        except AssertionError:
            failed.append(pin.__name__)
        except (KeyError, ValueError, FloatingPointError, ZeroDivisionError):
            failed.append(pin.__name__)
    return failed


def test_mutant_list_still_applies():
    for name, old, new in MUTANTS:
        assert SRC.count(old) >= 1, f"mutant {name}: its source text is gone"


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    src = tmp_path / "mutant.c"
    src.write_text(SRC.replace(old, new, 1) if SRC.count(old) == 1 else SRC.replace(old, new))
    so = tmp_path / "libmutant.so"
    oracle.build(force=True, src=str(src), out=str(so))
    lib = oracle._load(str(so))
    failed = _run_pins(lib)
    assert failed, f"planted mistake {name!r} passed every pin"


def test_real_oracle_passes_every_pin():
    assert _run_pins(None) == []
