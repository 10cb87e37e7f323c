"""CPU-only: the oracle against its pins, and the pins against planted mistakes."""
import os
import types

import pytest

import oracle.lqsgd_oracle as oracle_mod
from paper_2506_17974_amd import workloads as wl
from tests import oracle_pins as pins

_RES = wl.resnet18()
CHECKS = pins.all_checks(list(_RES.layers), sum(_RES.vectors))


@pytest.mark.parametrize("name,check", CHECKS, ids=[c[0] for c in CHECKS])
def test_pin(name, check):
    check(oracle_mod)


# ---------------------------------------------------------------------------
# Planted mistakes: each entry rewrites one line of the oracle's source; at
# least one pin must then fail.  (The mistakes are planted in a copy of the
# oracle on the CPU; nothing here touches the GPU path.)
# ---------------------------------------------------------------------------
MUTANTS = [
    ("compand_unnormalised", "np.log1p(alpha * np.abs(x)) / np.log1p(alpha)", "np.log1p(alpha * np.abs(x))"),
    ("compand_drops_sign", "return np.sign(x) * np.log1p(alpha * np.abs(x))", "return np.log1p(alpha * np.abs(x))"),
    ("expand_misses_minus_one", "np.expm1(np.abs(q) * np.log1p(alpha)) / alpha", "np.exp(np.abs(q) * np.log1p(alpha)) / alpha"),
    ("levels_off_by_one", "lv = (1 << bits) - 1\n    s = ", "lv = (1 << bits)\n    s = "),
    ("truncate_instead_of_round", "k = np.floor(t + 0.5)", "k = np.floor(t)"),
    ("round_down_ties_shifted", "k = np.floor(t + 0.5)", "k = np.floor(t + 0.75)"),
    ("ties_downward", "k = np.floor(t + 0.5)", "k = np.ceil(t - 0.5)"),
    ("nearest_in_x_domain", "t = lv * np.log1p(f64(alpha) * u.astype(f64)) / np.log1p(f64(alpha))", "t = lv * u.astype(f64)"),
    ("log_map_unnormalised", "t = lv * np.log1p(f64(alpha) * u.astype(f64)) / np.log1p(f64(alpha))", "t = lv * np.log1p(f64(alpha) * u.astype(f64))"),
    ("threshold_form_levels_off_by_one", "nlev = (1 << bits) - 1", "nlev = (1 << bits)"),
    ("threshold_form_truncates", "expand((np.arange(nlev) + 0.5) / nlev, alpha).astype(f32)", "expand((np.arange(nlev) + 1.0) / nlev, alpha).astype(f32)"),
    ("threshold_form_ties_downward", 'np.searchsorted(level_thresholds(bits, alpha), u, side="right")', 'np.searchsorted(level_thresholds(bits, alpha), u, side="left")'),
    ("threshold_form_in_q_domain", "expand((np.arange(nlev) + 0.5) / nlev, alpha).astype(f32)", "((np.arange(nlev) + 0.5) / nlev).astype(f32)"),
    ("threshold_form_sign_inverted", "sign_t = ((x < 0) & (kt > 0))", "sign_t = ((x > 0) & (kt > 0))"),
    ("scale_not_absmax", "s = f32(np.max(np.abs(x))) if x.size", "s = f32(np.max(x)) if x.size"),
    ("sign_inverted", "sign = ((x < 0) & (k > 0))", "sign = ((x > 0) & (k > 0))"),
    ("dequant_ignores_sign", "sgn = np.where(np.asarray(sign) != 0, -1.0, 1.0)", "sgn = 1.0"),
    ("dequant_levels_off", "q = np.asarray(k, dtype=f64) / lv", "q = np.asarray(k, dtype=f64) / (lv + 1)"),
    ("dequant_forgets_scale", "return sgn * f64(s) * mag", "return sgn * mag"),
    ("pack_msb_first", 'mag_bytes = np.packbits(bitmat.ravel().astype(np.uint8), bitorder="little")',
     'mag_bytes = np.packbits(bitmat.ravel().astype(np.uint8), bitorder="big")'),
    ("wire_forgets_sign_plane", "total += (n_el * b + 7) // 8 + (n_el + 7) // 8 + 4", "total += (n_el * b + 7) // 8 + 4"),
    ("wire_rank_unclipped", "r = min(rank, rows, cols)\n        for n_el", "r = rank\n        for n_el"),
    ("gs_no_projection", "v[:, k] -= (v[:, j] @ v[:, k]) * v[:, j]", "pass"),
    ("gs_projection_sign", "v[:, k] -= (v[:, j] @ v[:, k]) * v[:, j]", "v[:, k] += (v[:, j] @ v[:, k]) * v[:, j]"),
    ("gs_no_normalise", "v[:, k] /= np.sqrt(n2)", "v[:, k] /= 1.0"),
    ("gs_norm_not_sqrt", "v[:, k] /= np.sqrt(n2)", "v[:, k] /= n2"),
    ("sum_instead_of_mean", "return (acc / W).astype(f32), packets", "return (acc).astype(f32), packets"),
    ("feedback_subtracted", "M = (G[w].astype(f64) + E[w].astype(f64)).astype(f32)", "M = (G[w].astype(f64) - E[w].astype(f64)).astype(f32)"),
    ("feedback_dropped", "M = (G[w].astype(f64) + E[w].astype(f64)).astype(f32)", "M = (G[w].astype(f64)).astype(f32)"),
    ("p_uses_gradient_not_m", "P = (M.astype(f64) @ Q.astype(f64)).astype(f32)", "P = (G[w].astype(f64) @ Q.astype(f64)).astype(f32)"),
    ("orthonormalise_skipped", "Po = orthonormalize(P).astype(f32)", "Po = P"),
    ("q_uses_own_p", 'Qw = (out["M"][w].astype(f64).T @ out["P_bar"].astype(f64)).astype(f32)',
     'Qw = (out["M"][w].astype(f64).T @ out["P_orth"][w].astype(f64)).astype(f32)'),
    ("q_uses_gradient_not_m", 'Qw = (out["M"][w].astype(f64).T @ out["P_bar"].astype(f64)).astype(f32)',
     'Qw = (G[w].astype(f64).T @ out["P_bar"].astype(f64)).astype(f32)'),
    ("q_exchange_uses_bits_p", 'exchange(out["Q_w"], bits_q, alpha)', 'exchange(out["Q_w"], bits_p if bits_p == 0 else max(1, bits_p - 4), alpha)'),
    ("residual_sign", '(out["M"][w].astype(f64) - G_hat.astype(f64)).astype(f32)', '(G_hat.astype(f64) - out["M"][w].astype(f64)).astype(f32)'),
    ("residual_from_own_factors", 'G_hat = (out["P_bar"].astype(f64) @ out["Q_bar"].astype(f64).T).astype(f32)',
     'G_hat = (out["P_orth"][0].astype(f64) @ out["Q_bar"].astype(f64).T).astype(f32)'),
    ("warm_start_dropped", 'Q[l] = o["Q_bar"]', "pass"),
    ("error_not_carried", 'E[w][l] = o["E_new"][w]', "pass"),
    ("vector_sum", "return (acc / len(vs)).astype(f32)", "return (acc).astype(f32)"),
    ("agg_first_orthonormalises_too_early", 'res["P_pre"].append(Pw)', 'res["P_pre"].append(orthonormalize(Pw).astype(f32))'),
    ("agg_first_skips_orthonormalise", 'P_hat = orthonormalize(res["P_mean"]).astype(f32)', 'P_hat = res["P_mean"]'),
    ("agg_first_q_uses_raw_mean", '(res["M"][w].astype(f64).T @ P_hat.astype(f64)).astype(f32)',
     '(res["M"][w].astype(f64).T @ res["P_mean"].astype(f64)).astype(f32)'),
    ("agg_first_feedback_dropped", "Mw = (G[w].astype(f64) + E[w].astype(f64)).astype(f32)", "Mw = (G[w].astype(f64)).astype(f32)"),
    ("agg_first_p_transposed_q", "Pw = (Mw.astype(f64) @ Q.astype(f64)).astype(f32)", "Pw = (Mw.astype(f64) @ Q.astype(f64)[:, ::-1]).astype(f32)"),
    ("agg_first_ghat_from_mean", 'Gh = (P_hat.astype(f64) @ res["Q_bar"].astype(f64).T).astype(f32)',
     'Gh = (res["P_mean"].astype(f64) @ res["Q_bar"].astype(f64).T).astype(f32)'),
    ("agg_first_residual_sign", '(res["M"][w].astype(f64) - Gh.astype(f64)).astype(f32)', '(Gh.astype(f64) - res["M"][w].astype(f64)).astype(f32)'),
    ("agg_first_q_bits", 'exchange(res["Q_w"], bits_q, alpha)', 'exchange(res["Q_w"], bits_p, alpha)'),
    ("update_sign", "(np.asarray(weights, f32).astype(f64) - step).astype(f32)", "(np.asarray(weights, f32).astype(f64) + step).astype(f32)"),
    ("update_forgets_eta", "step = f64(f32(eta)) * np.asarray(g_hat, f32).astype(f64)", "step = np.asarray(g_hat, f32).astype(f64)"),
    ("update_eta_not_f32", "step = f64(f32(eta)) * np.asarray(g_hat, f32).astype(f64)", "step = f64(eta) * np.asarray(g_hat, f32).astype(f64)"),
]


def _mutant(old, new):
    path = oracle_mod.__file__
    with open(path) as fh:
        src = fh.read()
    assert src.count(old) >= 1, "mutation target not found: %r" % old
    m = types.ModuleType("oracle_mutant")
    m.__file__ = path
    exec(compile(src.replace(old, new), path, "exec"), m.__dict__)
    return m


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, old, new):
    mod = _mutant(old, new)
    failed = []
    for cname, check in CHECKS:
        try:
            check(mod)
        except Exception:          # assertion, shape error, NaN handling: all count
            failed.append(cname)
            break
    assert failed, "no pin notices the planted mistake %s" % name
