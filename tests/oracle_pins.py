"""Pins for the CPU oracle: each check ties one part of oracle/lqsgd_oracle.py
to something fixed outside it -- a closed form, an invariant, a library
routine on a special case, brute force on a tiny input, or a value the paper
prints.  Every check takes the oracle module as an argument so that the
mutation test can run the same checks against deliberately broken copies.
"""
from __future__ import annotations

import math
import os
from fractions import Fraction

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
f32, f64 = np.float32, np.float64


def _golden_rows(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line)
    return rows


def _rng(seed):
    return np.random.default_rng(seed)


# --------------------------------------------------------------------------
# Section 4.1, Eq. (5) and Eq. (6)
# --------------------------------------------------------------------------
def check_map_closed_forms(o):
    for alpha in (1.0, 10.0, 255.0, 1000.0):
        x = np.concatenate([np.linspace(-1, 1, 2001), [1e-12, -1e-9, 0.3333]])
        q = o.compand(x, alpha)
        # mutual inverses
        assert np.allclose(o.expand(q, alpha), x, rtol=1e-13, atol=1e-16)
        # odd, fixed points, range
        assert np.array_equal(o.compand(-x, alpha), -q)
        assert o.compand(0.0, alpha) == 0.0
        assert abs(o.compand(1.0, alpha) - 1.0) < 1e-15 and abs(o.compand(-1.0, alpha) + 1.0) < 1e-15
        assert abs(o.expand(1.0, alpha) - 1.0) < 1e-13 and o.expand(0.0, alpha) == 0.0
        # strictly increasing
        xs = np.linspace(-1, 1, 4001)
        assert np.all(np.diff(o.compand(xs, alpha)) > 0)
        assert np.all(np.diff(o.expand(xs, alpha)) > 0)
        # independent evaluation with the math module, power form of Eq. (6)
        for xv in (0.001, 0.25, 0.9):
            qv = math.log(1 + alpha * xv) / math.log(1 + alpha)
            assert abs(float(o.compand(xv, alpha)) - qv) < 1e-14
            assert abs(float(o.expand(qv, alpha)) - ((1 + alpha) ** qv - 1) / alpha) < 1e-13


def check_mulaw_checkpoints(o):
    """alpha = 255: x = (2^j - 1)/255 maps to exactly j/8 (golden file)."""
    for row in _golden_rows("mulaw_checkpoints.txt"):
        j, xn, xd, qn, qd, code = row.split()
        x = Fraction(int(xn), int(xd))
        q = Fraction(int(qn), int(qd))
        assert abs(float(o.compand(float(x), 255.0)) - float(q)) < 1e-15
        assert abs(float(o.expand(float(q), 255.0)) - float(x)) < 1e-15
        if code != "tie":
            # a tensor holding x and the value 1 (so that the absmax scale is 1)
            k, sg, s = o.log_quantize(np.array([float(x), 1.0], f32), 8, 255.0)
            assert s == f32(1.0) and int(k[0]) == int(code) and int(k[1]) == 255
            k, sg, s = o.log_quantize(np.array([-float(x), 1.0], f32), 8, 255.0)
            assert int(k[0]) == int(code) and int(sg[0]) == (1 if int(code) > 0 else 0)


# --------------------------------------------------------------------------
# Section 4.1 last paragraph: 2^b uniform bins on |q|, nearest level
# --------------------------------------------------------------------------
def check_bin_rounding_bruteforce(o):
    rng = _rng(11)
    for alpha in (1.0, 255.0, 1000.0):
        for bits in (1, 2, 3, 4, 5, 8):
            lv = (1 << bits) - 1
            x = (rng.standard_t(3.0, size=4000) * 1e-3).astype(f32)
            k, sg, s = o.log_quantize(x, bits, alpha)
            u = (np.abs(x) / s).astype(f32).astype(f64)
            qabs = np.log(1.0 + alpha * u) / math.log(1.0 + alpha)
            levels = np.arange(lv + 1, dtype=f64) / lv
            dist = np.abs(qabs[:, None] - levels[None, :])
            best = np.argmin(dist, axis=1)
            srt = np.sort(dist, axis=1)
            clear = (srt[:, 1] - srt[:, 0]) > 1e-9          # leave exact ties aside
            assert np.array_equal(best[clear], k[clear].astype(np.int64))
            assert k.max() == lv                              # the absmax element
            assert np.array_equal(sg, ((x < 0) & (k > 0)).astype(np.uint8))


def check_two_bit_enumeration(o):
    """b = 2: levels 0, 1/3, 2/3, 1; decision thresholds in the x-domain are
    Eq. (6) at the midpoints 1/6, 1/2, 5/6."""
    alpha = 255.0
    thr = [((1 + alpha) ** m - 1) / alpha for m in (1 / 6, 1 / 2, 5 / 6)]
    for kexp, t in enumerate(thr):
        lo, hi = t * (1 - 1e-4), t * (1 + 1e-4)
        k, _, s = o.log_quantize(np.array([lo, hi, 1.0], f32), 2, alpha)
        assert s == f32(1.0)
        assert (int(k[0]), int(k[1]), int(k[2])) == (kexp, kexp + 1, 3)
    # dequantised levels: Eq. (6) at q = k/3
    d = o.log_dequantize(np.arange(4), np.zeros(4), f32(2.0), 2, alpha)
    want = [2.0 * ((1 + alpha) ** (k / 3) - 1) / alpha for k in range(4)]
    assert np.allclose(d, want, rtol=1e-13)


def check_threshold_ties(o):
    """The bin decision at and around the boundaries.
    (a) Exact ties: for b = 1 the boundary is |q| = 1/2, i.e. 1 + alpha u = sqrt(1 + alpha); with
        (alpha, u) = (8, 1/4), (48, 1/8), (224, 1/16) both sides are exact in binary (3^2 = 9,
        7^2 = 49, 15^2 = 225), the tie goes to the upper level and the float32 below it down.
    (b) Around every boundary (the midpoint between two levels mapped back by Eq. (6), written
        out here, not taken from the oracle): a few float32 steps above it the upper level,
        a few below it the lower one."""
    for alpha, u in ((8.0, 0.25), (48.0, 0.125), (224.0, 0.0625)):
        x = np.array([u, np.nextafter(f32(u), f32(0.0)), -u, 1.0], f32)
        k, sg, s = o.log_quantize(x, 1, alpha)
        assert s == 1.0 and k.tolist() == [1, 0, 1, 1] and sg.tolist() == [0, 0, 1, 0], (alpha, k, sg)
    for alpha in (1.0, 255.0):
        for bits in (1, 2, 4, 8):
            lv = (1 << bits) - 1
            mid = (np.arange(lv) + 0.5) / lv
            thr = ((1.0 + alpha) ** mid - 1.0) / alpha                        # Eq. (6), float64
            above = thr.astype(f32)
            below = thr.astype(f32)
            for _ in range(3):
                above = np.nextafter(above, f32(2.0)).astype(f32)
                below = np.nextafter(below, f32(0.0)).astype(f32)
            x = np.concatenate([above, below, [f32(1.0)]]).astype(f32)        # the 1 makes the scale exactly 1
            for fn in (o.log_quantize, o.log_quantize_threshold_form):
                k, sg, s = fn(x, bits, alpha)
                assert s == 1.0
                assert np.array_equal(k[:lv], np.arange(1, lv + 1)), (alpha, bits)
                assert np.array_equal(k[lv:2 * lv], np.arange(0, lv)), (alpha, bits)
                assert k[-1] == lv
                kn, sgn, _ = fn(-x, bits, alpha)
                assert np.array_equal(kn, k) and np.array_equal(sgn, (k > 0).astype(np.uint8))


def check_threshold_form(o):
    """The float32 threshold-table form against the float64 rule: equal everywhere except
    within one float32 step of a boundary, and there at most one level apart; a value equal
    to a float32 threshold counts as reached (goes up)."""
    rng = _rng(17)
    for alpha in (1.0, 255.0, 1000.0):
        for bits in (1, 2, 4, 8):
            lv = (1 << bits) - 1
            mid = (np.arange(lv) + 0.5) / lv
            thr32 = (((1.0 + alpha) ** mid - 1.0) / alpha).astype(f32)
            x = np.concatenate([thr32, [f32(1.0)]]).astype(f32)
            kt, _, s = o.log_quantize_threshold_form(x, bits, alpha)
            assert s == 1.0 and np.array_equal(kt[:lv], np.arange(1, lv + 1))
            # random values crowded around the boundaries, and plain ones
            near = thr32[rng.integers(0, lv, 20000)]
            steps = rng.integers(-3, 4, near.size)
            for _ in range(3):
                near = np.where(steps > 0, np.nextafter(near, f32(2.0)), np.where(steps < 0, np.nextafter(near, f32(0.0)), near)).astype(f32)
                steps = steps - np.sign(steps)
            x = np.concatenate([near, rng.random(20000).astype(f32), [f32(1.0)]]).astype(f32)
            k, sg, s = o.log_quantize(x, bits, alpha)
            kt, sgt, st = o.log_quantize_threshold_form(x, bits, alpha)
            assert s == st == 1.0
            d = k.astype(np.int64) - kt.astype(np.int64)
            assert np.abs(d).max() <= 1
            bad = np.nonzero(d)[0]
            u = x[bad]
            j = np.minimum(k[bad], kt[bad]).astype(np.int64)      # the boundary between the two codes
            t = thr32[j]
            assert np.all((u == t) | (np.nextafter(u, f32(2.0)) == t) | (np.nextafter(u, f32(0.0)) == t))
            assert bad.size < 0.5 * near.size                      # the crowd is +-3 steps wide
            assert np.array_equal(sgt, ((x < 0) & (kt > 0)).astype(np.uint8))


def check_quantiser_properties(o):
    rng = _rng(5)
    for alpha in (1.0, 10.0, 255.0, 1000.0):
        for bits in (1, 2, 4, 8):
            lv = (1 << bits) - 1
            # idempotence over every code, both signs
            s = f32(0.0371)
            codes = np.arange(lv + 1, dtype=np.uint8)
            for sign in (0, 1):
                sg = np.full(lv + 1, sign, np.uint8)
                x = o.log_dequantize(codes, sg, s, bits, alpha).astype(f32)
                k2, sg2, s2 = o.log_quantize(x, bits, alpha)
                assert s2 == s                      # top code dequantises to exactly s
                assert np.array_equal(k2, codes)
                assert np.array_equal(sg2, np.where(codes > 0, sign, 0))
            # sign preservation, monotone codes, absmax -> top code -> +-s
            x = (rng.standard_normal(3000) * 1e-2).astype(f32)
            k, sg, s = o.log_quantize(x, bits, alpha)
            xh = o.log_dequantize(k, sg, s, bits, alpha)
            assert np.all((np.sign(xh) == np.sign(x)) | (xh == 0))
            order = np.argsort(np.abs(x), kind="stable")
            assert np.all(np.diff(k[order].astype(np.int64)) >= 0)
            i = int(np.argmax(np.abs(x)))
            assert int(k[i]) == lv and f32(xh[i]) == f32(np.sign(x[i])) * s
            assert s == f32(np.abs(x).max())
            # exact error bound that follows from Eq. (5) with |t - k| <= 1/2
            u = (np.abs(x) / s).astype(f32).astype(f64)
            ratio = (np.abs(xh) / f64(s) + 1 / alpha) / (u + 1 / alpha)
            bound = (1 + alpha) ** (1 / (2 * lv))
            assert np.all(ratio <= bound * (1 + 1e-12)) and np.all(ratio >= 1 / bound * (1 - 1e-12))


def check_zero_and_shapes(o):
    k, sg, s = o.log_quantize(np.zeros((5, 3), f32), 8, 255.0)
    assert s == 0 and not k.any() and not sg.any() and k.shape == (5, 3)
    d = o.log_dequantize(k, sg, s, 8, 255.0)
    assert not d.any() and np.all(np.isfinite(d))


# --------------------------------------------------------------------------
# wire format and the Section 4.3 cost model
# --------------------------------------------------------------------------
def check_packing(o):
    for row in _golden_rows("packing_examples.txt"):
        bits, codes, mag_hex, signs, sign_hex = [c.strip() for c in row.split("|")]
        bits = int(bits)
        k = np.array([int(c) for c in codes.split(",")], np.uint8)
        sg = np.array([int(c) for c in signs.split(",")], np.uint8)
        mb, sb = o.pack_packet(k, sg, bits)
        assert bytes(mb) == bytes.fromhex(mag_hex.replace(" ", "")), (bits, bytes(mb).hex())
        assert bytes(sb) == bytes.fromhex(sign_hex.replace(" ", "")), (bits, bytes(sb).hex())
        k2, s2 = o.unpack_packet(mb, sb, k.size, bits)
        assert np.array_equal(k2, k) and np.array_equal(s2, sg)
    rng = _rng(3)
    for bits in range(1, 9):
        n = int(rng.integers(1, 300))
        k = rng.integers(0, 1 << bits, n).astype(np.uint8)
        sg = rng.integers(0, 2, n).astype(np.uint8)
        mb, sb = o.pack_packet(k, sg, bits)
        assert mb.size == bits * ((n + 7) // 8) and sb.size == (n + 7) // 8
        k2, s2 = o.unpack_packet(mb, sb, n, bits)
        assert np.array_equal(k2, k) and np.array_equal(s2, sg)


def check_wire_size(o, resnet_layers, resnet_vector_elems):
    # Section 4.3: r(n+m) b bits per layer, 32/b times fewer than fp32 factors.
    layers = [(256, 128), (64, 576)]
    for r in (1, 2, 4):
        for b in (2, 4, 8):
            n_el = sum(r * (n + m) for n, m in layers)
            planes_and_scales = sum(((n * r + 7) // 8 + (m * r + 7) // 8 + 8) for n, m in layers)
            assert o.wire_bytes(layers, r, b, b) == n_el * b // 8 + planes_and_scales
            assert o.wire_bytes(layers, r, 0, 0) == 4 * n_el
    # rank clipped to the smaller dimension
    assert o.wire_bytes([(10, 512)], 16, 0, 0) == 4 * 10 * (10 + 512)
    # Printed sizes (Tables 1-3, rank 1): the ratios they imply, with the
    # rounding of the printed integers taken into account.
    total = sum(n * m for n, m in resnet_layers) + resnet_vector_elems
    fac = sum(n + m for n, m in resnet_layers)
    for row in _golden_rows("table_sizes.txt"):
        name, sgd, psgd, topk, lq = row.split()
        sgd, psgd, lq = float(sgd), float(psgd), float(lq)
        # PowerSGD / SGD = (rank-1 factors + uncompressed vectors) / all parameters
        ours = (o.wire_bytes(resnet_layers, 1, 0, 0) + 4 * resnet_vector_elems) / (4 * total)
        if name == "cifar10":      # the layer set of the benchmark is the CIFAR-10 model
            assert (psgd - 0.5) / (sgd + 0.5) <= ours <= (psgd + 0.5) / (sgd - 0.5)
        # PowerSGD / LQ-SGD: the paper's nominal count is 32 / b = 4 at b = 8
        assert (psgd - 0.5) / (lq + 0.5) <= 32 / 8 <= (psgd + 0.5) / (lq - 0.5)
    assert fac == 36325


# --------------------------------------------------------------------------
# Algorithm 1, "Orthonormalize"
# --------------------------------------------------------------------------
def check_orthonormalize(o):
    rng = _rng(7)
    for rows, r in ((3, 1), (4, 2), (50, 4), (301, 8), (64, 32)):
        p = rng.standard_normal((rows, r))
        v = o.orthonormalize(p)
        assert np.abs(v.T @ v - np.eye(r)).max() < 1e-12
        # thin QR with positive diagonal is unique: v R = p, R upper triangular
        R = v.T @ p
        assert np.abs(np.tril(R, -1)).max() < 1e-12 * np.abs(R).max()
        assert np.all(np.diag(R) > 0)
        assert np.allclose(v @ np.triu(R), p, rtol=0, atol=1e-12 * np.abs(p).max() * rows)
        # library special case: Householder QR, signs fixed
        qn, rn = np.linalg.qr(p)
        qn = qn * np.sign(np.diag(rn))[None, :]
        assert np.allclose(v, qn, atol=1e-11)
    x = rng.standard_normal((9, 1))
    assert np.allclose(o.orthonormalize(x), x / np.linalg.norm(x), rtol=1e-15)
    # hand-worked 3-4-5 case
    v = o.orthonormalize(np.array([[3.0, 1.0], [4.0, 1.0], [0.0, 1.0]]))
    assert np.allclose(v[:, 0], [0.6, 0.8, 0.0], atol=1e-15)
    # second column: (1,1,1) - 1.4*(0.6,0.8,0) = (0.16,-0.12,1), norm sqrt(1.04)
    assert np.allclose(v[:, 1], np.array([0.16, -0.12, 1.0]) / math.sqrt(1.04), atol=1e-15)
    # zero and repeated columns: zero output, no NaN
    z = o.orthonormalize(np.zeros((6, 3)))
    assert not z.any()
    d = o.orthonormalize(np.array([[1.0, 2.0], [0.0, 0.0], [0.0, 0.0]]))
    assert np.allclose(d[:, 0], [1, 0, 0]) and not d[:, 1].any()


# --------------------------------------------------------------------------
# Algorithm 1 loop body with quantisation off: a PowerSGD power step
# --------------------------------------------------------------------------
def _lowrank(rng, rows, cols, r, scale=1.0):
    a = rng.standard_normal((rows, r))
    b = rng.standard_normal((cols, r))
    return (scale * a @ b.T).astype(f32)


def check_power_step_unquantised(o):
    rng = _rng(21)
    rows, cols, r = 37, 23, 3
    zeros = np.zeros((rows, cols), f32)
    q0 = rng.standard_normal((cols, r)).astype(f32)
    # (a) exact recovery of a rank-r matrix, single worker
    M = _lowrank(rng, rows, cols, r)
    out = o.layer_step([M], [zeros], q0, r, 0, 0, 255.0)
    assert np.linalg.norm(out["G_hat"] - M) <= 2e-6 * np.linalg.norm(M)
    assert np.linalg.norm(out["E_new"][0]) <= 2e-6 * np.linalg.norm(M)
    # ... and with identical workers
    out4 = o.layer_step([M] * 4, [zeros] * 4, q0, r, 0, 0, 255.0)
    assert np.array_equal(out4["G_hat"], out["G_hat"])
    # (b) general matrix: G_hat is the orthogonal projection of M on span(M Q0),
    #     computed here through LAPACK QR instead of Gram-Schmidt
    M = rng.standard_normal((rows, cols)).astype(f32)
    out = o.layer_step([M], [zeros], q0, r, 0, 0, 255.0)
    qn, _ = np.linalg.qr(M.astype(f64) @ q0.astype(f64))
    proj = qn @ (qn.T @ M.astype(f64))
    assert np.linalg.norm(out["G_hat"] - proj) <= 1e-5 * np.linalg.norm(M)
    P = out["P_orth"][0].astype(f64)
    assert np.abs(P.T @ out["E_new"][0].astype(f64)).max() <= 1e-5 * np.linalg.norm(M)
    nM, nG, nE = (np.linalg.norm(a.astype(f64)) ** 2 for a in (M, out["G_hat"], out["E_new"][0]))
    assert abs(nM - nG - nE) <= 1e-5 * nM
    assert np.array_equal(out["P_bar"], out["P_orth"][0])       # no quantisation, W = 1
    assert np.allclose(out["Q_bar"], M.astype(f64).T @ P, atol=1e-5)
    # (c) rank clipped: r >= rows  =>  projection on the whole space, G_hat = M
    Ms = rng.standard_normal((3, 11)).astype(f32)
    qs = rng.standard_normal((11, 3)).astype(f32)
    outs = o.layer_step([Ms], [np.zeros_like(Ms)], qs, 8, 0, 0, 255.0)
    assert outs["P_bar"].shape == (3, 3) and outs["Q_bar"].shape == (11, 3)
    assert np.linalg.norm(outs["G_hat"] - Ms) <= 1e-5 * np.linalg.norm(Ms)
    # (d) rank-1 closed form  M = sigma u v^T  =>  P = +-u, Q = +-sigma v
    u = rng.standard_normal(rows); u /= np.linalg.norm(u)
    v = rng.standard_normal(cols); v /= np.linalg.norm(v)
    M1 = (2.5 * np.outer(u, v)).astype(f32)
    o1 = o.layer_step([M1], [zeros], rng.standard_normal((cols, 1)).astype(f32), 1, 0, 0, 255.0)
    sgn = np.sign(o1["P_bar"][:, 0] @ u)
    assert np.allclose(o1["P_bar"][:, 0], sgn * u, atol=1e-6)
    assert np.allclose(o1["Q_bar"][:, 0], sgn * 2.5 * v, atol=1e-6)


def check_subspace_iteration_reaches_svd(o):
    """Repeating the step on a fixed M with the residual reset and Q warm-started
    is subspace iteration; its error tends to the truncated-SVD error."""
    rng = _rng(33)
    rows, cols, r = 40, 30, 3
    U, _ = np.linalg.qr(rng.standard_normal((rows, rows)))
    V, _ = np.linalg.qr(rng.standard_normal((cols, cols)))
    sv = np.array([10, 7, 5, 1.0, 0.8, 0.5] + [0.1] * (cols - 6))
    M = ((U[:, :cols] * sv[None, :]) @ V.T).astype(f32)
    svd = np.linalg.svd(M.astype(f64), compute_uv=False)
    best = math.sqrt(float((svd[r:] ** 2).sum()))
    q = rng.standard_normal((cols, r)).astype(f32)
    zeros = np.zeros_like(M)
    errs = []
    for _ in range(25):
        out = o.layer_step([M], [zeros], q, r, 0, 0, 255.0)
        q = out["Q_bar"]
        errs.append(float(np.linalg.norm(out["E_new"][0].astype(f64))))
    assert errs[-1] >= best * (1 - 1e-6)
    assert errs[-1] <= best * (1 + 1e-4)
    assert errs[-1] <= errs[0]


# --------------------------------------------------------------------------
# Section 4.2 error feedback, any b, any W
# --------------------------------------------------------------------------
def check_error_feedback_identities(o):
    rng = _rng(44)
    rows, cols, r, W = 29, 36, 2, 4
    layers = [(rows, cols), (12, 7)]
    T = 4
    grads = [[[(rng.standard_t(3.0, size=s) * 1e-3).astype(f32) for s in layers] for _ in range(W)] for _ in range(T)]
    Q0 = [rng.standard_normal((c, min(r, n, c))).astype(f32) for n, c in layers]
    for bits in (8, 4, 0):
        hist, E, Q = o.run_steps(grads, layers, Q0, r, bits, bits, 255.0)
        sumG = [np.zeros(s, f64) for s in layers]
        sumGhat = [np.zeros(s, f64) for s in layers]
        Eprev = [[np.zeros(s, f32) for s in layers] for _ in range(W)]
        for t in range(T):
            for l in range(len(layers)):
                out = hist[t][l]
                Mbar = np.zeros(layers[l], f64)
                for w in range(W):
                    M = out["M"][w]
                    # Eq. (9): G' = G + E_{t-1}, stored in fp32
                    assert np.array_equal(M, (grads[t][w][l].astype(f64) + Eprev[w][l].astype(f64)).astype(f32))
                    # Eq. (8): G' = G_hat + E to within the one rounding of E
                    En = out["E_new"][w]
                    recon = out["G_hat"].astype(f64) + En.astype(f64)
                    assert np.all(np.abs(recon - M) <= 0.5 * np.spacing(np.abs(En)).astype(f64))
                    Mbar += M
                    Eprev[w][l] = out["E_new"][w]
                Mbar /= W
                Ebar = sum(out["E_new"][w].astype(f64) for w in range(W)) / W
                assert np.allclose(Ebar, Mbar - out["G_hat"], atol=1e-9)
                sumG[l] += sum(grads[t][w][l].astype(f64) for w in range(W)) / W
                sumGhat[l] += out["G_hat"]
                # warm start: next step's Q is this step's aggregated Q
                if t + 1 < T:
                    nxt = hist[t + 1][l]
                    assert np.array_equal(
                        nxt["P_pre"][0],
                        (nxt["M"][0].astype(f64) @ out["Q_bar"].astype(f64)).astype(f32))
        # telescoping: what was applied plus what is still owed equals what came in
        for l in range(len(layers)):
            Ebar = sum(E[w][l].astype(f64) for w in range(W)) / W
            assert np.allclose(sumGhat[l] + Ebar, sumG[l], atol=2e-8)
            assert np.array_equal(Q[l], hist[-1][l]["Q_bar"])


def check_quantised_step_structure(o):
    """With quantisation on: every stage obeys what Algorithm 1 states about it."""
    rng = _rng(55)
    rows, cols, r, W, bits, alpha = 48, 20, 3, 4, 8, 255.0
    G = [(rng.standard_normal((rows, cols)) * 1e-3).astype(f32) for _ in range(W)]
    E = [(rng.standard_normal((rows, cols)) * 1e-4).astype(f32) for _ in range(W)]
    q0 = rng.standard_normal((cols, r)).astype(f32)
    out = o.layer_step(G, E, q0, r, bits, bits, alpha)
    lv = (1 << bits) - 1
    bound = (1 + alpha) ** (1 / (2 * lv))
    Pd = np.zeros((rows, r))
    for w in range(W):
        M = out["M"][w].astype(f64)
        assert np.allclose(out["P_pre"][w], M @ q0.astype(f64), rtol=1e-6, atol=1e-9)
        Po = out["P_orth"][w].astype(f64)
        assert np.abs(Po.T @ Po - np.eye(r)).max() < 1e-6
        R = Po.T @ out["P_pre"][w].astype(f64)
        assert np.all(np.diag(R) > 0) and np.abs(np.tril(R, -1)).max() < 1e-6 * np.abs(R).max()
        k, sg, s = out["pkt_P"][w]
        assert s == f32(np.abs(out["P_orth"][w]).max())
        d = o.log_dequantize(k, sg, s, bits, alpha)
        ratio = (np.abs(d) / f64(s) + 1 / alpha) / (np.abs(Po) / f64(s) + 1 / alpha)
        assert np.all(ratio < bound * (1 + 1e-6)) and np.all(ratio > 1 / bound * (1 - 1e-6))
        Pd += d
    assert np.allclose(out["P_bar"], Pd / W, rtol=1e-6, atol=1e-9)       # a mean, not a sum
    Qd = np.zeros((cols, r))
    for w in range(W):
        Qw = out["M"][w].astype(f64).T @ out["P_bar"].astype(f64)          # uses the aggregate
        assert np.allclose(out["Q_w"][w], Qw, rtol=1e-5, atol=1e-10)
        k, sg, s = out["pkt_Q"][w]
        assert s == f32(np.abs(out["Q_w"][w]).max())
        Qd += o.log_dequantize(k, sg, s, bits, alpha)
    assert np.allclose(out["Q_bar"], Qd / W, rtol=1e-6, atol=1e-12)
    assert np.allclose(out["G_hat"], out["P_bar"].astype(f64) @ out["Q_bar"].astype(f64).T, rtol=1e-6, atol=1e-12)
    for w in range(W):
        assert np.allclose(out["E_new"][w], out["M"][w].astype(f64) - out["G_hat"], rtol=1e-6, atol=1e-10)
    # mean_of_packets is the receiving half of exchange
    assert np.array_equal(o.mean_of_packets(out["pkt_P"], bits, alpha), out["P_bar"])


def check_aggregation(o):
    rng = _rng(66)
    rows, cols, r = 21, 34, 4
    G = (rng.standard_normal((rows, cols)) * 1e-3).astype(f32)
    E = (rng.standard_normal((rows, cols)) * 1e-4).astype(f32)
    q0 = rng.standard_normal((cols, r)).astype(f32)
    one = o.layer_step([G], [E], q0, r, 8, 8, 255.0)
    for W in (2, 8):
        many = o.layer_step([G] * W, [E] * W, q0, r, 8, 8, 255.0)
        for key in ("P_bar", "Q_bar", "G_hat"):
            assert np.array_equal(many[key], one[key])
        assert np.array_equal(many["E_new"][W - 1], one["E_new"][0])
    # permuting the workers changes the aggregate only by re-association
    Gs = [(rng.standard_normal((rows, cols)) * 1e-3).astype(f32) for _ in range(4)]
    Es = [np.zeros((rows, cols), f32)] * 4
    a = o.layer_step(Gs, Es, q0, r, 8, 8, 255.0)
    b = o.layer_step(Gs[::-1], Es, q0, r, 8, 8, 255.0)
    assert np.allclose(a["G_hat"], b["G_hat"], rtol=1e-5, atol=1e-9)
    assert np.array_equal(a["pkt_P"][0][0], b["pkt_P"][3][0])
    # 1-D tensors: a plain mean
    vs = [rng.standard_normal(13).astype(f32) for _ in range(4)]
    assert np.allclose(o.vector_mean(vs), np.mean(np.stack(vs).astype(f64), axis=0), rtol=1e-7)


def check_tiny_bruteforce(o):
    """4 x 3, r = 2, W = 2, small integers: the products in exact rationals,
    the quantiser by search over all levels, everything else by definition."""
    G = [np.array([[1, 2, 0], [0, 1, 1], [2, 0, 1], [1, 1, 1]], f32),
         np.array([[0, 1, 2], [1, 0, 1], [1, 1, 0], [2, 1, 0]], f32)]
    E = [np.array([[0, 0, 1], [0, 0, 0], [1, 0, 0], [0, 0, 0]], f32),
         np.zeros((4, 3), f32)]
    Q0 = np.array([[1, 0], [1, 1], [0, 2]], f32)
    bits, alpha = 4, 255.0
    lv = 15
    out = o.layer_step(G, E, Q0, 2, bits, bits, alpha)
    fr = lambda a: [[Fraction(float(v)) for v in row] for row in a]
    for w in range(2):
        M = [[fr(G[w])[i][j] + fr(E[w])[i][j] for j in range(3)] for i in range(4)]
        assert [[float(v) for v in row] for row in M] == out["M"][w].tolist()
        P = [[sum(M[i][c] * fr(Q0)[c][k] for c in range(3)) for k in range(2)] for i in range(4)]
        assert [[float(v) for v in row] for row in P] == out["P_pre"][w].tolist()
    # first Gram-Schmidt column of worker 0 by hand: M0 Q0[:,0] = (3, 1, 3, 2), norm sqrt(23)
    assert np.allclose(out["P_orth"][0][:, 0], np.array([3, 1, 3, 2]) / math.sqrt(23), atol=1e-7)
    levels_q = [k / lv for k in range(lv + 1)]
    levels_x = [((1 + alpha) ** q - 1) / alpha for q in levels_q]
    acc = np.zeros((4, 2))
    for w in range(2):
        Po = out["P_orth"][w]
        s = max(abs(float(v)) for v in Po.ravel())
        k, sg, sc = out["pkt_P"][w]
        assert float(sc) == s
        for i in range(4):
            for c in range(2):
                u = float(f32(abs(Po[i, c])) / f32(s))
                qv = math.log(1 + alpha * u) / math.log(1 + alpha)
                kb = min(range(lv + 1), key=lambda kk: abs(qv - levels_q[kk]))
                assert int(k[i, c]) == kb
                val = s * levels_x[kb] * (-1 if Po[i, c] < 0 and kb > 0 else 1)
                acc[i, c] += val
    assert np.allclose(out["P_bar"], acc / 2, rtol=1e-6)
    Pb = fr(out["P_bar"])
    for w in range(2):
        Mw = fr(out["M"][w])
        Qw = [[sum(Mw[i][c] * Pb[i][k] for i in range(4)) for k in range(2)] for c in range(3)]
        assert np.array_equal(out["Q_w"][w], np.array([[float(v) for v in row] for row in Qw], f32))
    Qb = fr(out["Q_bar"])
    Gh = [[sum(Pb[i][k] * Qb[c][k] for k in range(2)) for c in range(3)] for i in range(4)]
    assert np.array_equal(out["G_hat"], np.array([[float(v) for v in row] for row in Gh], f32))
    for w in range(2):
        Mw = fr(out["M"][w])
        Ew = [[Mw[i][c] - Fraction(float(out["G_hat"][i, c])) for c in range(3)] for i in range(4)]
        assert np.array_equal(out["E_new"][w], np.array([[float(v) for v in row] for row in Ew], f32))


def check_degenerate_inputs(o):
    z = np.zeros((6, 5), f32)
    q0 = np.ones((5, 2), f32)
    out = o.layer_step([z, z], [z, z], q0, 2, 8, 8, 255.0)
    for key in ("P_bar", "Q_bar", "G_hat"):
        assert not out[key].any() and np.all(np.isfinite(out[key]))
    for w in range(2):
        assert not out["E_new"][w].any()
        assert out["pkt_P"][w][2] == 0 and not out["pkt_P"][w][0].any()


def check_aggregate_first(o):
    """The PowerSGD order: with quantisation off the W workers act as one worker
    holding the mean gradient, a rank-r mean is recovered exactly for any W, and
    the aggregated P-hat is orthonormal; with quantisation on every stage still
    obeys its definition."""
    rng = _rng(77)
    rows, cols, r, W = 33, 26, 3, 5
    # distinct full-rank worker gradients whose MEAN has rank r
    A = rng.standard_normal((rows, r)); Bm = rng.standard_normal((r, cols))
    N = [rng.standard_normal((rows, cols)) for _ in range(W)]
    Nbar = sum(N) / W
    G = [(A @ Bm + (N[w] - Nbar)).astype(f32) for w in range(W)]
    E = [np.zeros((rows, cols), f32) for _ in range(W)]
    Q0 = rng.standard_normal((cols, r)).astype(f32)
    Mbar = sum(g.astype(f64) for g in G) / W
    out = o.layer_step_aggregate_first(G, E, Q0, r, 0, 0, 255.0)
    assert np.linalg.norm(out["G_hat"] - Mbar) <= 2e-5 * np.linalg.norm(Mbar)        # exact recovery, any W
    std = o.layer_step(G, E, Q0, r, 0, 0, 255.0)
    assert np.linalg.norm(std["G_hat"] - Mbar) > 1e-2 * np.linalg.norm(Mbar)         # ... which Algorithm 1's order lacks
    P = out["P_bar"].astype(f64)
    assert np.allclose(P.T @ P, np.eye(r), atol=1e-5)
    # the same as one worker holding the mean gradient (LAPACK projection of that mean)
    qr, _ = np.linalg.qr(Mbar @ Q0.astype(f64))
    assert np.linalg.norm(out["G_hat"] - qr @ (qr.T @ Mbar)) <= 2e-5 * np.linalg.norm(Mbar)
    one = o.layer_step([Mbar.astype(f32)], [E[0]], Q0, r, 0, 0, 255.0)
    assert np.linalg.norm(out["Q_bar"] - one["Q_bar"]) <= 1e-5 * np.linalg.norm(one["Q_bar"])
    assert np.linalg.norm(out["P_bar"] - one["P_bar"]) <= 1e-5 * np.linalg.norm(one["P_bar"])
    # Eq. (8) per worker and in the mean; W = 1 coincides with Algorithm 1's order
    for w in range(W):
        assert np.array_equal(out["M"][w], G[w])
        assert np.allclose(out["E_new"][w].astype(f64) + out["G_hat"], out["M"][w], rtol=0, atol=1e-6)
    G1 = [rng.standard_normal((rows, cols)).astype(f32)]
    E1 = [(rng.standard_normal((rows, cols)) * 0.1).astype(f32)]
    a1 = o.layer_step_aggregate_first(G1, E1, Q0, r, 0, 0, 255.0)
    s1 = o.layer_step(G1, E1, Q0, r, 0, 0, 255.0)
    for key in ("P_bar", "Q_bar", "G_hat"):
        assert np.array_equal(a1[key], s1[key])
    assert np.array_equal(a1["E_new"][0], s1["E_new"][0])
    # quantisation on: stages against their definitions
    bits, alpha = 8, 255.0
    Gq = [rng.standard_normal((rows, cols)).astype(f32) for _ in range(W)]
    Eq = [(rng.standard_normal((rows, cols)) * 0.05).astype(f32) for _ in range(W)]
    oq = o.layer_step_aggregate_first(Gq, Eq, Q0, r, bits, 4, alpha)
    lv = (1 << bits) - 1
    acc = np.zeros((rows, r))
    for w in range(W):
        Mw = Gq[w].astype(f64) + Eq[w].astype(f64)
        assert np.allclose(oq["M"][w], Mw, rtol=1e-7, atol=0)
        assert np.allclose(oq["P_pre"][w], Mw @ Q0.astype(f64), rtol=0, atol=1e-5)
        k, sg, s = oq["pkt_P"][w]
        assert s == np.max(np.abs(oq["P_pre"][w]))          # the raw factor is what gets quantised
        d = o.log_dequantize(k, sg, s, bits, alpha)
        # Eq. (5)/(6): half a level in the q-domain bounds the error
        half = 0.5 / lv
        qx = np.log1p(alpha * np.abs(oq["P_pre"][w].astype(f64)) / s) / np.log1p(alpha)
        hi = np.expm1(np.minimum(qx + half, 1.0) * np.log1p(alpha)) / alpha * s
        lo = np.expm1(np.maximum(qx - half, 0.0) * np.log1p(alpha)) / alpha * s
        assert np.all(np.abs(d) <= hi * (1 + 1e-6) + 1e-12) and np.all(np.abs(d) >= lo * (1 - 1e-6) - 1e-12)
        acc += d
        assert np.allclose(oq["Q_w"][w], Mw.T @ oq["P_bar"].astype(f64), rtol=0, atol=1e-5)
        assert oq["pkt_Q"][w][0].max() <= 15
    assert np.allclose(oq["P_mean"], acc / W, rtol=0, atol=1e-6)
    Pq = oq["P_bar"].astype(f64)
    assert np.allclose(Pq.T @ Pq, np.eye(r), atol=1e-5)
    qr, rr = np.linalg.qr(oq["P_mean"].astype(f64))
    assert np.allclose(Pq, qr * np.sign(np.diag(rr)), atol=1e-5)
    assert np.allclose(oq["G_hat"], Pq @ oq["Q_bar"].astype(f64).T, rtol=0, atol=1e-5)
    Ebar = sum(e.astype(f64) for e in oq["E_new"]) / W
    Mq = sum(m.astype(f64) for m in oq["M"]) / W
    assert np.allclose(Ebar, Mq - oq["G_hat"], rtol=0, atol=1e-6)


def check_model_update(o):
    """Algorithm 1's last statement.  With quantisation off, one worker and
    rank(G) <= r the reconstruction is G itself, so the step is plain SGD, Eq. (2)."""
    rng = _rng(88)
    rows, cols, r = 19, 14, 2
    G = (rng.standard_normal((rows, r)) @ rng.standard_normal((r, cols))).astype(f32)
    w0 = rng.standard_normal((rows, cols)).astype(f32)
    out = o.layer_step([G], [np.zeros_like(G)], rng.standard_normal((cols, r)).astype(f32), r, 0, 0, 255.0)
    eta = 0.125                                        # a power of two: eta * g is exact
    w1 = o.model_update(w0, out["G_hat"], eta)
    assert w1.dtype == f32 and w1.shape == w0.shape
    assert np.allclose(w1, w0.astype(f64) - eta * G.astype(f64), rtol=0, atol=2e-5 * np.abs(G).max())
    # exact cases: small integers and a power-of-two eta leave no rounding at all
    wi = np.array([[4.0, -2.0], [1.0, 8.0]], f32); gi = np.array([[2.0, 4.0], [-6.0, 0.0]], f32)
    assert np.array_equal(o.model_update(wi, gi, 0.5), np.array([[3.0, -4.0], [4.0, 8.0]], f32))
    assert np.array_equal(o.model_update(wi, np.zeros_like(gi), 0.3), wi)
    assert np.array_equal(o.model_update(wi, gi, 0.0), wi)
    # linear in eta and in g
    a = o.model_update(wi, gi, 0.25).astype(f64); b = o.model_update(wi, gi, 0.75).astype(f64)
    assert np.array_equal(b - a, -0.5 * gi)
    # eta is taken as a float32 value
    gv = rng.standard_normal(4000).astype(f32)
    assert np.array_equal(o.model_update(np.zeros_like(gv), gv, 0.1), (-(f64(f32(0.1)) * gv.astype(f64))).astype(f32))


def all_checks(resnet_layers, resnet_vector_elems):
    return [
        ("map_closed_forms", check_map_closed_forms),
        ("mulaw_checkpoints", check_mulaw_checkpoints),
        ("bin_rounding_bruteforce", check_bin_rounding_bruteforce),
        ("two_bit_enumeration", check_two_bit_enumeration),
        ("threshold_ties", check_threshold_ties),
        ("threshold_form", check_threshold_form),
        ("quantiser_properties", check_quantiser_properties),
        ("zero_and_shapes", check_zero_and_shapes),
        ("packing", check_packing),
        ("wire_size", lambda o: check_wire_size(o, resnet_layers, resnet_vector_elems)),
        ("orthonormalize", check_orthonormalize),
        ("power_step_unquantised", check_power_step_unquantised),
        ("subspace_iteration_reaches_svd", check_subspace_iteration_reaches_svd),
        ("error_feedback_identities", check_error_feedback_identities),
        ("quantised_step_structure", check_quantised_step_structure),
        ("aggregation", check_aggregation),
        ("tiny_bruteforce", check_tiny_bruteforce),
        ("degenerate_inputs", check_degenerate_inputs),
        ("aggregate_first", check_aggregate_first),
        ("model_update", check_model_update),
    ]
