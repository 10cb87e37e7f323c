"""CPU oracle for the LQ-SGD per-step gradient compressor.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain, obviously-correct
definition the HIP path is checked against.  Only tests, the smoke check and
the bench's cpu_baseline leg may import it; the product never does, and this
file imports nothing from the product.

Everything here is numpy in float64, with the tensors the method stores
(M, P, Q, P-bar, Q-bar, G-hat, E) rounded to float32 where the method stores
them.  No blocking, fusion or reordering: each function is the paper's step
written out.

Notation (the paper swaps the letters n and m between its Section 3.2 and
Section 4 / Algorithm 1, so neither is used here): a layer gradient is
``rows x cols``; P is ``rows x r``; Q is ``cols x r``; W workers.

Readings of the paper where it is silent or ambiguous:

* R1  per-worker: G_w, E_w, M_w = G_w + E_w, P_w, Q_w.  Shared by all
      workers: the warm-start Q, the aggregated P-bar, Q-bar and G-hat.
* R2  Algorithm 1 orthonormalises each worker's P *before* quantise /
      aggregate; P-bar is not re-orthonormalised.
* R3  "Orthonormalize" = one pass of modified Gram-Schmidt, columns left to
      right; a column whose squared norm is not above FLT_MIN becomes zero.
* R4  Eq. (5) needs |x| <= 1: every tensor is divided by its own absmax s
      (one float32 sent with the codes); s == 0 gives all-zero codes.
* R5  a code is one sign bit plus a b-bit magnitude index k in [0, 2^b - 1];
      levels are uniform in the q-domain with both endpoints,
      level_k = k / (2^b - 1); nearest level of |q(u)| (Eq. (5)), ties upward,
      decided in float64 on the float32 u = |x| / s.  (A second function gives
      the float32 threshold-table form of the same decision; the two differ
      only within a float32 rounding of a bucket boundary.)
* R6  the "All-Reduce" of quantised factors means: dequantise every worker's
      packet, then take the mean (Eq. (1)), summed in worker order.
* R7  effective rank of a layer is min(r, rows, cols).
* R8  b = 0 switches quantisation off (the PowerSGD baseline of Section 3.2).
* R9  ``layer_step_aggregate_first`` is the order Section 3.2 describes for
      PowerSGD (exchange P, orthonormalise the aggregate once, then Q); with
      bits > 0 the un-orthonormalised P_w is what gets quantised (R4's absmax
      scale brings it into range).
* R10 the model update is Algorithm 1's last statement / Eq. (2), plain SGD in
      float32 storage; eta is a float32 value.

Parity pins: see tests/test_oracle_pins.py.  Unpinned: the direction of a
Gram-Schmidt column whose residual is pure rounding noise (rank-deficient
input) -- "parity unpinned" for that direction; the paper prints no worked
numerical example, so no printed value is pinned either.
"""
from __future__ import annotations

import numpy as np

FLT_MIN = float(np.finfo(np.float32).tiny)

f32 = np.float32
f64 = np.float64


# ----------------------------------------------------------------------------
# Section 4.1: the logarithmic map and its inverse (continuous forms)
# ----------------------------------------------------------------------------
def compand(x, alpha):
    """Eq. (5): q(x) = sign(x) * log(1 + alpha |x|) / log(1 + alpha)."""
    x = np.asarray(x, dtype=f64)
    return np.sign(x) * np.log1p(alpha * np.abs(x)) / np.log1p(alpha)


def expand(q, alpha):
    """Eq. (6): x = sign(q) * ((1 + alpha)^|q| - 1) / alpha."""
    q = np.asarray(q, dtype=f64)
    return np.sign(q) * np.expm1(np.abs(q) * np.log1p(alpha)) / alpha


# ----------------------------------------------------------------------------
# Section 4.1, last paragraph: b-bit discretisation of |q| (readings R4, R5)
# ----------------------------------------------------------------------------
def log_quantize(x, bits, alpha):
    """LogQuantize of Algorithm 1 (statements "P_quant <- ..." / "Q_quant <- ...").

    x      float32 array, any shape
    returns (k, sign, s):
      k     uint8, magnitude index in [0, 2^bits - 1], same shape as x
      sign  uint8, 1 where x < 0 and k > 0 (the sign of a zero code carries
            nothing and is canonically 0)
      s     float32 absmax scale
    The normalised magnitude u = |x| / s is taken in float32 (the precision the
    stored factor has).  The map of Eq. (5) and the choice of the nearest of the
    2^bits levels k / (2^bits - 1) of |q| (Section 4.1, last paragraph; ties go
    up) run in float64: k = floor((2^bits - 1) q(u) + 1/2).
    """
    if not (1 <= bits <= 8):
        raise ValueError("bits must be in 1..8")
    x = np.asarray(x, dtype=f32)
    lv = (1 << bits) - 1
    s = f32(np.max(np.abs(x))) if x.size else f32(0.0)
    if not (s > 0):
        return (np.zeros(x.shape, np.uint8), np.zeros(x.shape, np.uint8), f32(0.0))
    u = (np.abs(x) / s).astype(f32)                       # float32 division
    t = lv * np.log1p(f64(alpha) * u.astype(f64)) / np.log1p(f64(alpha))
    k = np.floor(t + 0.5)
    k = np.clip(k, 0, lv).astype(np.uint8)
    sign = ((x < 0) & (k > 0)).astype(np.uint8)
    return k, sign, s


def level_thresholds(bits, alpha):
    """Decision thresholds of the same discretisation in the normalised magnitude u:
    T_j = Eq. (6) at the midpoint (j + 1/2) / (2^b - 1) between levels j and j + 1,
    j = 0 .. 2^b - 2, evaluated in float64 and stored as float32."""
    nlev = (1 << bits) - 1
    return expand((np.arange(nlev) + 0.5) / nlev, alpha).astype(f32)


def log_quantize_threshold_form(x, bits, alpha):
    """The same discretisation decided in float32: the code of u is the number of float32
    thresholds T_j <= u (Eq. (5) is increasing, so in exact arithmetic this is the nearest
    level with ties upward).  It can differ from ``log_quantize`` by one level, and only where
    u lies within a float32 rounding of a threshold; it is what an implementation that keeps
    u and a threshold table in float32 computes, and the tests use it to tell such boundary
    cases from real mistakes.  Returns (k, sign, s) like ``log_quantize``."""
    if not (1 <= bits <= 8):
        raise ValueError("bits must be in 1..8")
    x = np.asarray(x, dtype=f32)
    s = f32(np.max(np.abs(x))) if x.size else f32(0.0)
    if not (s > 0):
        return (np.zeros(x.shape, np.uint8), np.zeros(x.shape, np.uint8), f32(0.0))
    u = (np.abs(x) / s).astype(f32)
    kt = np.searchsorted(level_thresholds(bits, alpha), u, side="right").astype(np.uint8)
    sign_t = ((x < 0) & (kt > 0)).astype(np.uint8)
    return kt, sign_t, s


def log_dequantize(k, sign, s, bits, alpha):
    """LogDequantize of Algorithm 1: Eq. (6) at q = k / (2^bits - 1), times s.

    Returns float64 (the caller rounds where the method stores a tensor)."""
    lv = (1 << bits) - 1
    q = np.asarray(k, dtype=f64) / lv
    mag = np.expm1(q * np.log1p(f64(alpha))) / f64(alpha)
    sgn = np.where(np.asarray(sign) != 0, -1.0, 1.0)
    return sgn * f64(s) * mag


# ----------------------------------------------------------------------------
# Wire format of one quantised factor (reading R5: two separable planes)
# ----------------------------------------------------------------------------
def pack_packet(k, sign, bits):
    """Magnitude plane: element e (row-major order) occupies bits
    [e*bits, (e+1)*bits) of a little-endian bit stream, padded with zeros to
    whole groups of 8 elements.  Sign plane: 1 bit per element, LSB first.
    Returns (mag_bytes uint8[bits*ceil(n/8)], sign_bytes uint8[ceil(n/8)])."""
    k = np.asarray(k, np.uint8).ravel()
    sign = np.asarray(sign, np.uint8).ravel()
    n = k.size
    ngrp = (n + 7) // 8
    kp = np.zeros(ngrp * 8, np.uint8)
    kp[:n] = k
    sp = np.zeros(ngrp * 8, np.uint8)
    sp[:n] = sign
    # bit j of element e -> stream position e*bits + j
    bitmat = (kp[:, None] >> np.arange(bits, dtype=np.uint8)[None, :]) & 1
    mag_bytes = np.packbits(bitmat.ravel().astype(np.uint8), bitorder="little")
    sign_bytes = np.packbits(sp, bitorder="little")
    return mag_bytes, sign_bytes


def unpack_packet(mag_bytes, sign_bytes, n, bits):
    """Inverse of pack_packet for the first n elements."""
    mb = np.unpackbits(np.asarray(mag_bytes, np.uint8), bitorder="little")
    mb = mb[: ((n + 7) // 8) * 8 * bits].reshape(-1, bits)
    k = (mb.astype(np.uint16) << np.arange(bits, dtype=np.uint16)[None, :]).sum(axis=1)
    sb = np.unpackbits(np.asarray(sign_bytes, np.uint8), bitorder="little")
    return k[:n].astype(np.uint8), sb[:n].astype(np.uint8)


def wire_bytes(layers, rank, bits_p, bits_q):
    """Bytes one worker sends per step for the 2-D layers ``[(rows, cols), ...]``.

    Section 4.3 counts r(n+m)*b bits per layer; with the sign plane and one
    float32 scale per factor (readings R4, R5) a factor of n_el elements costs
    ceil(n_el*b/8) + ceil(n_el/8) + 4 bytes.  b = 0 sends raw float32."""
    total = 0
    for rows, cols in layers:
        r = min(rank, rows, cols)
        for n_el, b in ((rows * r, bits_p), (cols * r, bits_q)):
            if b == 0:
                total += 4 * n_el
            else:
                total += (n_el * b + 7) // 8 + (n_el + 7) // 8 + 4
    return total


# ----------------------------------------------------------------------------
# Algorithm 1, "Orthonormalize" (reading R3)
# ----------------------------------------------------------------------------
def orthonormalize(p):
    """Modified Gram-Schmidt, one pass, columns left to right, in float64."""
    v = np.array(p, dtype=f64, copy=True)
    r = v.shape[1]
    for k in range(r):
        for j in range(k):
            v[:, k] -= (v[:, j] @ v[:, k]) * v[:, j]
        n2 = v[:, k] @ v[:, k]
        if n2 > FLT_MIN:
            v[:, k] /= np.sqrt(n2)
        else:
            v[:, k] = 0.0
    return v


# ----------------------------------------------------------------------------
# One factor exchange: quantise per worker, dequantise, mean (reading R6)
# ----------------------------------------------------------------------------
def exchange(factors, bits, alpha):
    """factors: list over workers of float32 arrays (same shape).
    Returns (mean float32, packets) with packets[w] = (k, sign, s), or None
    entries when bits == 0."""
    W = len(factors)
    acc = np.zeros(factors[0].shape, f64)
    packets = []
    for w in range(W):
        if bits == 0:
            packets.append(None)
            acc += factors[w].astype(f64)
        else:
            k, sg, s = log_quantize(factors[w], bits, alpha)
            packets.append((k, sg, s))
            acc += log_dequantize(k, sg, s, bits, alpha)
    return (acc / W).astype(f32), packets


def mean_of_packets(packets, bits, alpha):
    """Dequantise-and-average only (the receiving side of the exchange)."""
    W = len(packets)
    acc = None
    for k, sg, s in packets:
        d = log_dequantize(k, sg, s, bits, alpha)
        acc = d if acc is None else acc + d
    return (acc / W).astype(f32)


# ----------------------------------------------------------------------------
# Algorithm 1, loop body, for one 2-D layer and W workers
# ----------------------------------------------------------------------------
def layer_step(G, E, Q, rank, bits_p, bits_q, alpha):
    """G, E: lists over workers of float32 (rows, cols); Q: float32 (cols, r_l)
    with r_l = min(rank, rows, cols).

    Returns a dict of every tensor the method materialises:
      M[w], P_pre[w], P_orth[w], pkt_P[w], P_bar, Q_w[w], pkt_Q[w], Q_bar,
      G_hat, E_new[w]
    """
    W = len(G)
    rows, cols = G[0].shape
    r = min(rank, rows, cols)
    Q = np.asarray(Q, f32)
    assert Q.shape == (cols, r)

    out = {"M": [], "P_pre": [], "P_orth": [], "Q_w": [], "E_new": []}
    for w in range(W):
        # G' <- G + E_{t-1}  (error-feedback compensation; Eq. (9))
        M = (G[w].astype(f64) + E[w].astype(f64)).astype(f32)
        # P <- G' Q
        P = (M.astype(f64) @ Q.astype(f64)).astype(f32)
        # P <- Orthonormalize(P)
        Po = orthonormalize(P).astype(f32)
        out["M"].append(M)
        out["P_pre"].append(P)
        out["P_orth"].append(Po)
    # LogQuantize, All-Reduce, LogDequantize of P
    out["P_bar"], out["pkt_P"] = exchange(out["P_orth"], bits_p, alpha)
    for w in range(W):
        # Q <- G'^T P
        Qw = (out["M"][w].astype(f64).T @ out["P_bar"].astype(f64)).astype(f32)
        out["Q_w"].append(Qw)
    # LogQuantize, All-Reduce, LogDequantize of Q
    out["Q_bar"], out["pkt_Q"] = exchange(out["Q_w"], bits_q, alpha)
    # G-hat <- P Q^T   (Eq. (7))
    G_hat = (out["P_bar"].astype(f64) @ out["Q_bar"].astype(f64).T).astype(f32)
    out["G_hat"] = G_hat
    for w in range(W):
        # E <- G' - G-hat   (Eq. (8))
        out["E_new"].append((out["M"][w].astype(f64) - G_hat.astype(f64)).astype(f32))
    return out


def layer_step_aggregate_first(G, E, Q, rank, bits_p, bits_q, alpha):
    """The PowerSGD order (Section 3.2: P = M Q is all-reduced, *then*
    orthonormalised, then Q = M^T P-hat is all-reduced), with the same
    quantised exchange as Algorithm 1 in place of the plain all-reduce.

    Returns M[w], P_pre[w], pkt_P[w], P_mean (aggregate before Gram-Schmidt),
    P_bar (the orthonormalised aggregate every worker then uses), Q_w[w],
    pkt_Q[w], Q_bar, G_hat, E_new[w]."""
    W = len(G)
    rows, cols = G[0].shape
    r = min(rank, rows, cols)
    Q = np.asarray(Q, f32)
    assert Q.shape == (cols, r)
    res = {"M": [], "P_pre": [], "Q_w": [], "E_new": []}
    for w in range(W):
        Mw = (G[w].astype(f64) + E[w].astype(f64)).astype(f32)          # Eq. (9)
        Pw = (Mw.astype(f64) @ Q.astype(f64)).astype(f32)               # P_w = M_w Q
        res["M"].append(Mw)
        res["P_pre"].append(Pw)
    # exchange the raw factors, then one Gram-Schmidt on the aggregate
    res["P_mean"], res["pkt_P"] = exchange(res["P_pre"], bits_p, alpha)
    P_hat = orthonormalize(res["P_mean"]).astype(f32)
    res["P_bar"] = P_hat
    for w in range(W):
        res["Q_w"].append((res["M"][w].astype(f64).T @ P_hat.astype(f64)).astype(f32))
    res["Q_bar"], res["pkt_Q"] = exchange(res["Q_w"], bits_q, alpha)
    Gh = (P_hat.astype(f64) @ res["Q_bar"].astype(f64).T).astype(f32)   # Eq. (7)
    res["G_hat"] = Gh
    for w in range(W):
        res["E_new"].append((res["M"][w].astype(f64) - Gh.astype(f64)).astype(f32))   # Eq. (8)
    return res


def model_update(weights, g_hat, eta):
    """w_{t+1} = w_t - eta G-hat_t (Algorithm 1, last statement; Eq. (2)).
    float32 storage, eta a float32 value; for a 1-D tensor g_hat is its mean."""
    step = f64(f32(eta)) * np.asarray(g_hat, f32).astype(f64)
    return (np.asarray(weights, f32).astype(f64) - step).astype(f32)


def vector_mean(vs):
    """Uncompressed 1-D tensors: plain mean over workers (Eq. (1))."""
    acc = np.zeros(vs[0].shape, f64)
    for v in vs:
        acc += v.astype(f64)
    return (acc / len(vs)).astype(f32)


def run_steps(grads_per_step, layers, Q0, rank, bits_p, bits_q, alpha):
    """Multi-step driver: error feedback and warm-start Q carried across steps.

    grads_per_step[t][w][l] float32 arrays (2-D layers only);
    layers = [(rows, cols), ...]; Q0[l] float32 (cols, r_l).
    Returns (list over steps of list over layers of layer_step dicts,
             final E[w][l], final Q[l])."""
    T = len(grads_per_step)
    W = len(grads_per_step[0])
    L = len(layers)
    E = [[np.zeros(layers[l], f32) for l in range(L)] for _ in range(W)]   # E_0 = 0
    Q = [np.asarray(Q0[l], f32) for l in range(L)]
    hist = []
    for t in range(T):
        outs = []
        for l in range(L):
            o = layer_step([grads_per_step[t][w][l] for w in range(W)],
                           [E[w][l] for w in range(W)], Q[l],
                           rank, bits_p, bits_q, alpha)
            for w in range(W):
                E[w][l] = o["E_new"][w]
            Q[l] = o["Q_bar"]                       # warm start for t + 1
            outs.append(o)
        hist.append(outs)
    return hist, E, Q
