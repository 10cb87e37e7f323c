"""Shared machinery of the GPU parity tests: run the HIP path through the C ABI
and compare every stage with the CPU oracle fed the same inputs.

The comparison is stage-wise: fp32 summation order differs between the two
sides, so a free-running comparison of quantised codes is meaningless (a
1e-7 difference in a factor flips a code when the value sits on a bucket
boundary, and a flipped code moves everything downstream).  Each stage of the
HIP path is therefore checked against the oracle applied to the HIP path's own
upstream tensors; a free-running end-to-end comparison is done on the tensors
that are insensitive to single code flips (E and G-hat).
"""
from __future__ import annotations

import os

import numpy as np

import oracle.lqsgd_oracle as orc
from paper_2506_17974_amd import binding as B

f32, f64 = np.float32, np.float64
FP_TOL = 1e-4          # relative Frobenius error allowed on fp32 factors and residuals
MEAN_TOL = 2e-6        # dequantise-and-mean: a handful of fp32 roundings
# Codes are compared with the oracle's quantiser, which takes Eq. (5) and the nearest of the 2^b
# levels in float64 (Section 4.1).  The HIP path decides in float32 against a float32 threshold
# table, so it may land one level off where u lies within one float32 step of a bucket boundary;
# every such element is verified to be exactly that, counted and reported, and the count is held to
# CODE_BAND_BUDGET of the elements checked (on sets below SMALL_SET elements, where that would be a
# fraction of one element, to at most SMALL_SET_BAND verified boundary cases).  Outside that band
# the codes must be equal.  The HIP path's codes must also equal, all of them, the oracle's
# float32 threshold-table form of the same decision.
CODE_BAND_BUDGET = 1e-5
SMALL_SET = 200000
SMALL_SET_BAND = 2


# Per test (pytest's current test id): [codes at a bucket boundary, codes checked]; printed by
# tests/conftest.py in the terminal summary, so that the counts reach the log of a quiet run too.
BAND_COUNTS = {}


def code_band_budget(n_elems):
    return SMALL_SET_BAND if n_elems < SMALL_SET else int(CODE_BAND_BUDGET * n_elems)


def rel_fro(a, b):
    a = np.asarray(a, f64)
    b = np.asarray(b, f64)
    d = np.linalg.norm(a - b)
    n = np.linalg.norm(b)
    return d / n if n > 0 else d


def to_device(arrs):
    import torch
    return [[torch.from_numpy(np.ascontiguousarray(a)).cuda() for a in row] for row in arrs]


def check_codes(x_gpu, k_gpu, s_gpu, scale_gpu, bits, alpha):
    """Oracle quantiser (float64 nearest-level rule) applied to the HIP path's own
    pre-quantisation tensor.  Returns the number of elements whose code differs; each of them
    has been verified here to be a one-level difference at a bucket boundary (moving u by one
    float32 step reaches the HIP path's code under the float64 rule) -- anything else fails at
    once.  The caller adds the counts up and holds them to the budget."""
    k, sg, s = orc.log_quantize(x_gpu, bits, alpha)
    assert f32(scale_gpu) == s, "absmax scale differs: %r vs %r" % (scale_gpu, s)
    diff = k.astype(np.int32) != k_gpu.astype(np.int32)
    nband = int(diff.sum())
    if nband:
        assert np.all(np.abs(k.astype(np.int32) - k_gpu.astype(np.int32))[diff] == 1), "a code is off by more than one level"
        lv = (1 << bits) - 1
        u = (np.abs(x_gpu[diff]) / s).astype(f32)
        up = np.nextafter(u, f32(2.0)).astype(f64)
        dn = np.nextafter(u, f32(-1.0)).astype(f64)
        t_up = np.floor(lv * np.log1p(alpha * up) / np.log1p(alpha) + 0.5)
        t_dn = np.floor(lv * np.log1p(alpha * dn) / np.log1p(alpha) + 0.5)
        kg = k_gpu[diff].astype(f64)
        assert np.all((t_up == kg) | (t_dn == kg)), "a differing code is not within 1 ulp of a bucket boundary"
    # the float32 threshold-table form of the same decision: no difference at all
    kt, sgt, _ = orc.log_quantize_threshold_form(x_gpu, bits, alpha)
    assert np.array_equal(kt, k_gpu), "%d codes differ from the float32 threshold form" % int((kt != k_gpu).sum())
    assert np.array_equal(sgt, s_gpu), "sign bits differ"
    # signs against the float64 rule: compared where the code is non-zero on both sides
    both = (k > 0) & (k_gpu > 0)
    assert np.array_equal(sg[both], s_gpu[both]), "sign bits differ"
    assert not np.any(s_gpu[k_gpu == 0]), "sign bit set on a zero code"
    tally = BAND_COUNTS.setdefault(os.environ.get("PYTEST_CURRENT_TEST", "?").split(" ")[0], [0, 0])
    tally[0] += nband
    tally[1] += int(k_gpu.size)
    return nband


class StageReport:
    def __init__(self):
        self.code_elems = 0
        self.code_flips = 0
        self.worst = {}

    def note(self, key, val):
        self.worst[key] = max(self.worst.get(key, 0.0), float(val))

    def __str__(self):
        parts = ["%s=%.2e" % kv for kv in sorted(self.worst.items())]
        return "codes: %d of %d at a bucket boundary (one level off the float64 rule, verified; budget %d), 0 elsewhere; " % (
            self.code_flips, self.code_elems, code_band_budget(self.code_elems)) + " ".join(parts)


def staged_iteration(comp: B.Compressor, G_host, G_dev, E_host, Q_host, matrix_layers, rep: StageReport,
                     layers_to_check=None, workers_to_check=None, aggregate_first=False):
    """One iteration through compress/decompress with every stage checked.

    G_host[w][l], E_host[w][l] (state before the iteration), Q_host[l]: numpy.
    matrix_layers: indices (in the compressor's layer list) of the 2-D layers;
    G_host / E_host / Q_host are indexed by position in that list.
    layers_to_check / workers_to_check restrict the comparison (and the copies
    to the host) to a sample; entries of G_host / E_host outside it may be None.
    aggregate_first: the compressor was created with FLAG_AGGREGATE_FIRST (the
    raw P_w is exchanged, the aggregate is orthonormalised once).
    Returns (E_new[w][l], Q_bar[l]) as read back from the device (None outside
    the sample).
    """
    W = comp.workers
    bp, bq, alpha = comp.bits_p, comp.bits_q, comp.alpha
    Ls = range(len(matrix_layers)) if layers_to_check is None else layers_to_check
    Ws = range(W) if workers_to_check is None else workers_to_check

    comp.compress(B.PHASE_P, G_dev)
    M = {}
    for li in Ls:
        l = matrix_layers[li]
        for w in Ws:
            m_gpu, _ = comp.get_state(l, w, want_q=False)
            M[(li, w)] = m_gpu
            # G' = G + E: one IEEE addition per element, must be bit-exact
            assert np.array_equal(m_gpu, (G_host[w][li].astype(f64) + E_host[w][li].astype(f64)).astype(f32))
            p_pre = comp.get_factor(B.FACTOR_P_PRE, l, w)
            want = m_gpu.astype(f64) @ Q_host[li].astype(f64)
            rep.note("P_pre", rel_fro(p_pre, want))
            assert rel_fro(p_pre, want) <= FP_TOL
            if aggregate_first:
                sent = p_pre              # the raw factor goes on the wire, Gram-Schmidt follows the exchange
            else:
                p_orth = comp.get_factor(B.FACTOR_P_ORTH, l, w)
                want = orc.orthonormalize(p_pre)
                # columns whose residual is rounding noise have no defined direction
                ok = _well_defined_columns(p_pre)
                rep.note("P_orth", rel_fro(p_orth[:, ok], want[:, ok]))
                assert rel_fro(p_orth[:, ok], want[:, ok]) <= FP_TOL
                sent = p_orth
            if bp:
                k, sg, sc = comp.get_packet(B.PHASE_P, l, w)
                rep.code_flips += check_codes(sent, k, sg, sc, bp, alpha)
                rep.code_elems += k.size
                mag, sgn = comp.get_packet_raw(B.PHASE_P, l, w)
                om, os_ = orc.pack_packet(k, sg, bp)
                assert np.array_equal(mag, om) and np.array_equal(sgn, os_)
    comp.decompress(B.PHASE_P)
    Pbar = {}
    for li in Ls:
        l = matrix_layers[li]
        pb = comp.get_factor(B.FACTOR_P_MEAN if aggregate_first else B.FACTOR_P_BAR, l)
        if bp:
            pk = [comp.get_packet(B.PHASE_P, l, w) for w in range(W)]
            want = orc.mean_of_packets(pk, bp, alpha)
        else:
            which = B.FACTOR_P_PRE if aggregate_first else B.FACTOR_P_ORTH
            want = np.mean(np.stack([comp.get_factor(which, l, w).astype(f64) for w in range(W)]), axis=0)
        rep.note("P_bar", rel_fro(pb, want))
        assert rel_fro(pb, want) <= MEAN_TOL
        if aggregate_first:
            p_hat = comp.get_factor(B.FACTOR_P_BAR, l)
            want = orc.orthonormalize(pb)
            ok = _well_defined_columns(pb)
            rep.note("P_hat", rel_fro(p_hat[:, ok], want[:, ok]))
            assert rel_fro(p_hat[:, ok], want[:, ok]) <= FP_TOL
            pb = p_hat
        Pbar[li] = pb
    comp.compress(B.PHASE_Q)
    for li in Ls:
        l = matrix_layers[li]
        for w in Ws:
            q_w = comp.get_factor(B.FACTOR_Q_W, l, w)
            want = M[(li, w)].astype(f64).T @ Pbar[li].astype(f64)
            rep.note("Q_w", rel_fro(q_w, want))
            assert rel_fro(q_w, want) <= FP_TOL
            if bq:
                k, sg, sc = comp.get_packet(B.PHASE_Q, l, w)
                rep.code_flips += check_codes(q_w, k, sg, sc, bq, alpha)
                rep.code_elems += k.size
                mag, sgn = comp.get_packet_raw(B.PHASE_Q, l, w)
                om, os_ = orc.pack_packet(k, sg, bq)
                assert np.array_equal(mag, om) and np.array_equal(sgn, os_)
    comp.decompress(B.PHASE_Q)
    E_new = [[None] * len(matrix_layers) for _ in range(W)]
    Q_bar = [None] * len(matrix_layers)
    for li in Ls:
        l = matrix_layers[li]
        qb = comp.get_factor(B.FACTOR_Q_BAR, l)
        Q_bar[li] = qb
        if bq:
            pk = [comp.get_packet(B.PHASE_Q, l, w) for w in range(W)]
            want = orc.mean_of_packets(pk, bq, alpha)
        else:
            want = np.mean(np.stack([comp.get_factor(B.FACTOR_Q_W, l, w).astype(f64) for w in range(W)]), axis=0)
        rep.note("Q_bar", rel_fro(qb, want))
        assert rel_fro(qb, want) <= MEAN_TOL
        ghat = (Pbar[li].astype(f64) @ qb.astype(f64).T).astype(f32)
        absterms = np.abs(Pbar[li]).astype(f64) @ np.abs(qb).astype(f64).T
        r_l = qb.shape[1]
        for w in Ws:
            e_gpu, q_state = comp.get_state(l, w)
            E_new[w][li] = e_gpu
            assert np.array_equal(q_state, qb)            # warm start = aggregated Q
            want = (M[(li, w)].astype(f64) - ghat.astype(f64)).astype(f32)
            rep.note("E", rel_fro(e_gpu, want))
            assert rel_fro(e_gpu, want) <= FP_TOL
            # Eq. (8) as an identity, element by element: the r-term fp32 sum
            # behind G-hat rounds r times, each relative to the size of its terms
            scale = np.abs(M[(li, w)]) + absterms
            assert np.all(np.abs(e_gpu.astype(f64) + ghat - M[(li, w)]) <= (r_l + 2) * 6e-8 * scale + 1e-30)
    assert rep.code_flips <= code_band_budget(rep.code_elems), str(rep)
    return E_new, Q_bar


def _well_defined_columns(p_pre):
    """Gram-Schmidt columns whose residual after removing the earlier columns is
    well above rounding noise (others have an arbitrary direction)."""
    v = np.array(p_pre, f64)
    ok = []
    for k in range(v.shape[1]):
        n0 = np.linalg.norm(v[:, k])
        for j in range(k):
            nj = np.linalg.norm(v[:, j])
            if nj > 0:
                v[:, k] -= (v[:, j] @ v[:, k]) / (nj * nj) * v[:, j]
        ok.append(bool(n0 > 0 and np.linalg.norm(v[:, k]) > 1e-3 * n0))
    return np.array(ok, bool)


def oracle_free_run(G_steps, layers, Q0, rank, bits_p, bits_q, alpha):
    return orc.run_steps(G_steps, layers, Q0, rank, bits_p, bits_q, alpha)
