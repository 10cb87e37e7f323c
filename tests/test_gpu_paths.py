"""GPU parity for the code paths and API calls that the other files do not reach:
the in-memory Gram-Schmidt kernel (factors of 513..2048 rows at rank pads >= 16),
factor injection through lqsgd_set_factor, the checkpoint round trip through
lqsgd_get_state / lqsgd_set_state, and what lqsgd_get_state returns in the middle of
a staged iteration.  Everything here needs a real MI355X."""
import numpy as np
import pytest

import oracle.lqsgd_oracle as orc
from paper_2506_17974_amd import binding as B
from paper_2506_17974_amd import workloads as wl
from tests import parity_utils as pu
from tests.test_gpu_parity import _make, _random_inputs, _run_staged, _say, _vector_mean_ok

pytestmark = pytest.mark.gpu
f32, f64 = np.float32, np.float64


# ---------------------------------------------------------------------------
# Gram-Schmidt in memory: one workgroup per (layer, worker), rows beyond what the
# register-resident form holds at that rank
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("layers,rank,W", [
    ([(1024, 260)], 16, 2),                       # 1024 rows at rank pad 16
    ([(1024, 3136), (10, 1024)], 16, 4),          # the small CNN's fc1 / fc2 at rank 16
    ([(1024, 260), (600, 128)], 32, 2),           # rank pad 32
    ([(1500, 68)], 50, 2),                        # rank pad 64
    ([(1024, 132)], 20, 3),                       # rank below its pad
])
def test_in_memory_gram_schmidt(layers, rank, W):
    _say("case: in-memory Gram-Schmidt", layers, rank, W)
    rep = _run_staged(layers, rank, 8, 8, W, steps=2, seed=rank + W, e0_scale=3e-4)
    _say("  ", rep)


# ---------------------------------------------------------------------------
# lqsgd_set_factor: another implementation's aggregated factors take the place of
# the device's own (Algorithm 1, "Q <- G'^T P" with the injected P; the warm start
# with the injected Q)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("layers,rank,W", [([(64, 576), (33, 70)], 4, 4), ([(200, 1100)], 32, 2)])
def test_set_factor_injects_the_oracles_factors(layers, rank, W):
    _say("case: set_factor", layers, rank, W)
    rng = np.random.default_rng(rank)
    comp, ml = _make(layers, (), rank, 8, 8, W)
    Q0 = [rng.standard_normal((c, min(rank, r, c))).astype(f32) for r, c in layers]
    for l in ml:
        comp.set_q(l, Q0[l])
    G = _random_inputs(rng, layers, W)
    Gd = pu.to_device(G)
    zeros = [[np.zeros(s, f32) for s in layers] for _ in range(W)]
    # the oracle's own iteration on the same inputs
    outs = [orc.layer_step([G[k][l] for k in range(W)], [zeros[k][l] for k in range(W)], Q0[l], rank, 8, 8, 255.0)
            for l in ml]
    comp.compress(B.PHASE_P, Gd)
    comp.decompress(B.PHASE_P)
    for l in ml:
        assert pu.rel_fro(comp.get_factor(B.FACTOR_P_BAR, l), outs[l]["P_bar"]) < 0.1    # same thing, up to code flips
        comp.set_factor(B.FACTOR_P_BAR, l, outs[l]["P_bar"])
        assert np.array_equal(comp.get_factor(B.FACTOR_P_BAR, l), outs[l]["P_bar"])
    comp.compress(B.PHASE_Q)
    for l in ml:
        for k in range(W):
            # M is one IEEE addition on both sides, so the oracle's Q_w is M^T P-bar of the same operands
            err = pu.rel_fro(comp.get_factor(B.FACTOR_Q_W, l, k), outs[l]["Q_w"][k])
            assert err <= pu.FP_TOL, (l, k, err)
    comp.decompress(B.PHASE_Q)
    for l in ml:
        pb = outs[l]["P_bar"]
        qb_dev = comp.get_factor(B.FACTOR_Q_BAR, l)
        # injecting Q-bar after the iteration: the residual keeps the value the device's own Q-bar gave it
        # (a deferred update is applied before the factor is overwritten), the warm start changes
        comp.set_factor(B.FACTOR_Q_BAR, l, outs[l]["Q_bar"])
        for k in range(W):
            e, q = comp.get_state(l, k)
            assert np.array_equal(q, outs[l]["Q_bar"])
            m = (G[k][l].astype(f64) + zeros[k][l]).astype(f32)
            want = (m.astype(f64) - (pb.astype(f64) @ qb_dev.astype(f64).T).astype(f32)).astype(f32)
            assert pu.rel_fro(e, want) <= pu.FP_TOL
    # the next iteration starts from the injected Q-bar
    G2 = _random_inputs(rng, layers, W)
    comp.compress(B.PHASE_P, pu.to_device(G2))
    for l in ml:
        for k in range(W):
            m, _ = comp.get_state(l, k, want_q=False)
            want = m.astype(f64) @ outs[l]["Q_bar"].astype(f64)
            assert pu.rel_fro(comp.get_factor(B.FACTOR_P_PRE, l, k), want) <= pu.FP_TOL
    with pytest.raises(B.LqsgdError) as ei:
        comp.set_factor(B.FACTOR_Q_W, 0, outs[0]["Q_w"][0])
    assert ei.value.code == B.EINVAL
    comp.close()


# ---------------------------------------------------------------------------
# what lqsgd_get_state returns between the calls of a staged iteration
# ---------------------------------------------------------------------------
def test_get_state_in_the_middle_of_an_iteration():
    _say("case: get_state mid-iteration")
    layers, rank, W = [(64, 576), (17, 100)], 4, 2
    rng = np.random.default_rng(3)
    comp, ml = _make(layers, (), rank, 8, 8, W)
    Q0 = [rng.standard_normal((c, min(rank, r, c))).astype(f32) for r, c in layers]
    E0 = [[(rng.standard_normal(s) * 1e-4).astype(f32) for s in layers] for _ in range(W)]
    for l in ml:
        comp.set_q(l, Q0[l])
        for k in range(W):
            comp.set_state(l, k, e=E0[k][l])
    G = _random_inputs(rng, layers, W)
    comp.compress(B.PHASE_P, pu.to_device(G))
    for stage in ("after compress(P)", "after decompress(P)", "after compress(Q)"):
        for l in ml:
            for k in range(W):
                m, q = comp.get_state(l, k)
                assert np.array_equal(m, (G[k][l].astype(f64) + E0[k][l]).astype(f32)), stage   # G' = G + E (Eq. (9))
                assert np.array_equal(q, Q0[l]), stage                                          # still this iteration's Q
        if stage == "after compress(P)":
            comp.decompress(B.PHASE_P)
        elif stage == "after decompress(P)":
            comp.compress(B.PHASE_Q)
    comp.decompress(B.PHASE_Q)
    for l in ml:
        qb = comp.get_factor(B.FACTOR_Q_BAR, l)
        gh = (comp.get_factor(B.FACTOR_P_BAR, l).astype(f64) @ qb.astype(f64).T).astype(f32)
        for k in range(W):
            e, q = comp.get_state(l, k)
            assert np.array_equal(q, qb)
            m = (G[k][l].astype(f64) + E0[k][l]).astype(f32)
            assert pu.rel_fro(e, (m.astype(f64) - gh).astype(f32)) <= pu.FP_TOL                 # Eq. (8)
    comp.close()


# ---------------------------------------------------------------------------
# checkpoint / resume: the state the method carries between iterations is E of every
# worker (Section 4.2) and the warm-start Q of every layer (Algorithm 1)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("name,rank,flags", [("small_cnn", 4, 0), ("small_cnn", 16, 0), ("mixed", 32, 0),
                                             ("small_cnn", 4, B.FLAG_AGGREGATE_FIRST)])
def test_resume_from_saved_state_is_bit_identical(name, rank, flags):
    import torch
    _say("case: resume", name, rank, flags)
    if name == "small_cnn":
        w = wl.small_cnn()
        layers, vectors, W = list(w.layers), list(w.vectors), w.workers
    else:
        layers, vectors, W = [(200, 1100), (10, 512), (64, 27), (1024, 260)], [33], 2
    L, V = len(layers), len(vectors)
    rng = np.random.default_rng(41)
    Q0 = [rng.standard_normal((c, min(rank, r, c))).astype(f32) for r, c in layers]
    steps = [pu.to_device([g + [(rng.standard_normal(n) * 1e-3).astype(f32) for n in vectors]
                           for g in _random_inputs(rng, layers, W)]) for _ in range(10)]

    def outputs():
        return [torch.empty(s, device="cuda") for s in layers] + [torch.empty(n, device="cuda") for n in vectors]

    def run(comp, ghat, ts):
        for t in ts:
            comp.step(steps[t], ghat)
        comp.synchronize()

    ref, ml = _make(layers, vectors, rank, 8, 8, W, flags=flags)
    for l in ml:
        ref.set_q(l, Q0[l])
    g_ref = outputs()
    run(ref, g_ref, range(10))

    first, _ = _make(layers, vectors, rank, 8, 8, W, flags=flags)
    for l in ml:
        first.set_q(l, Q0[l])
    g_a = outputs()
    run(first, g_a, range(5))
    saved = [[first.get_state(l, k) for l in ml] for k in range(W)]      # (E, Q) per worker and layer
    first.close()

    second, _ = _make(layers, vectors, rank, 8, 8, W, flags=flags)
    for l in ml:
        for k in range(W):
            second.set_state(l, k, e=saved[k][l][0], q=saved[k][l][1] if k == 0 else None)
    g_b = outputs()
    run(second, g_b, range(5, 10))
    for i in range(L + V):
        assert torch.equal(g_ref[i], g_b[i]), "output %d differs after the resume" % i
    for l in ml:
        for k in range(W):
            e1, q1 = ref.get_state(l, k)
            e2, q2 = second.get_state(l, k)
            assert np.array_equal(e1, e2) and np.array_equal(q1, q2), (l, k)
    ref.close(); second.close()


# ---------------------------------------------------------------------------
# Gram-Schmidt on nearly dependent columns (here: a warm-start Q with two almost equal columns, so
# that two columns of P = M Q are almost parallel): the result must still be the oracle's within
# the fp32 tolerance on every column that is well defined, and orthonormal there
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("layers,rank,eps", [
    ([(300, 260)], 16, 4e-3), ([(512, 1100), (64, 576)], 32, 4e-3), ([(200, 520)], 50, 4e-3),
    ([(512, 1100)], 32, 3e-2),
])
def test_gram_schmidt_with_nearly_dependent_columns(layers, rank, eps):
    _say("case: nearly dependent columns", layers, rank, eps)
    rng = np.random.default_rng(int(rank + 1000 * eps))
    W = 2
    comp, ml = _make(layers, (), rank, 8, 8, W)
    Q = []
    for rows, cols in layers:
        q = rng.standard_normal((cols, min(rank, rows, cols))).astype(f32)
        q[:, 3] = q[:, 1] + eps * rng.standard_normal(cols).astype(f32)
        Q.append(q)
    E = [[np.zeros(s, f32) for s in layers] for _ in range(W)]
    for l in ml:
        comp.set_q(l, Q[l])
    rep = pu.StageReport()
    G = _random_inputs(rng, layers, W)
    E, Q = pu.staged_iteration(comp, G, pu.to_device(G), E, Q, ml, rep)
    for l in ml:
        for k in range(W):
            p = comp.get_factor(B.FACTOR_P_ORTH, l, k).astype(f64)
            ok = pu._well_defined_columns(comp.get_factor(B.FACTOR_P_PRE, l, k))
            gram = p[:, ok].T @ p[:, ok]
            assert np.abs(gram - np.eye(int(ok.sum()))).max() <= 2e-4, "columns not orthonormal"
            assert np.all(np.isfinite(p))
    _say("  ", rep)
    comp.close()


# ---------------------------------------------------------------------------
# Tall factors at rank pads >= 8: Orthogonalize (Algorithm 1) through two passes of Cholesky-QR
# instead of column by column.  Every stage is held against the oracle's Gram-Schmidt; the one
# cooperative launch and the form of three launches must agree bit for bit; pairs whose pivots fall
# below the floor (nearly dependent columns, an all-zero gradient) are done column by column, again
# with the same bits in both forms.
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("layers,rank,W,special", [
    ([(4096, 300)], 16, 4, None),
    ([(4096, 300)], 8, 3, None),                      # rank pad 8
    ([(2304, 200)], 7, 2, 4e-3),
    ([(2600, 36), (3000, 64)], 32, 2, None),
    ([(8192, 128)], 50, 2, None),
    ([(2304, 200), (300, 40)], 20, 3, None),          # rank below its pad; a short layer in the same launch
    ([(4096, 300), (2600, 12), (2305, 9)], 16, 2, None),   # layers whose own rank is clipped by their width (12, 9); a ragged last slice
    ([(4096, 300)], 16, 2, 4e-3),                     # two nearly parallel columns: a pivot below the floor
    ([(5000, 96)], 50, 2, 4e-3),
    ([(2600, 72)], 32, 2, 0.3),                       # columns at an angle the factorisation still takes
    ([(8192, 96)], 32, 2, 0.03),                      # ... and close to its pivot floor (ratio about 5e-4)
    ([(4096, 300)], 50, 2, 0.03),
    ([(4096, 300)], 16, 3, "zero"),                   # one worker's gradient is zero: P_w = 0
])
def test_tall_gram_schmidt_by_cholesky_qr(layers, rank, W, special):
    _say("case: tall Gram-Schmidt, Cholesky-QR", layers, rank, W, special)
    rng = np.random.default_rng(rank + W)
    Q0 = []
    for rows, cols in layers:
        q = rng.standard_normal((cols, min(rank, rows, cols))).astype(f32)
        if isinstance(special, float):
            q[:, 3] = q[:, 1] + special * rng.standard_normal(cols).astype(f32)
        Q0.append(q)
    G = _random_inputs(rng, layers, W)
    if special == "zero":
        G[W - 1][0][:] = 0.0
    Gd = pu.to_device(G)
    rp = 8 if rank <= 8 else 16 if rank <= 16 else 32 if rank <= 32 else 64
    got = {}
    for flags, name in ((0, "orth_chol_kernel<%d>" % rp), (B.FLAG_NO_COOPERATIVE_LAUNCH, "orth_chol_kernel<%d> x 3 launches" % rp)):
        comp, ml = _make(layers, (), rank, 8, 8, W, flags=flags)
        for l in ml:
            comp.set_q(l, Q0[l])
        E = [[np.zeros(s, f32) for s in layers] for _ in range(W)]
        rep = pu.StageReport()
        pu.staged_iteration(comp, G, Gd, E, Q0, ml, rep)
        assert comp.launched_kernel(B.KERNEL_ORTH) == name, comp.launched_kernel(B.KERNEL_ORTH)
        facs = []
        for l in ml:
            for k in range(W):
                p = comp.get_factor(B.FACTOR_P_ORTH, l, k)
                assert np.all(np.isfinite(p))
                ok = pu._well_defined_columns(comp.get_factor(B.FACTOR_P_PRE, l, k))
                if special == "zero" and l == 0 and k == W - 1:
                    assert not p.any()
                else:
                    p64 = p[:, ok].astype(f64)
                    assert np.abs(p64.T @ p64 - np.eye(int(ok.sum()))).max() <= 2e-4, "columns not orthonormal"
                facs.append(p)
            facs.append(comp.get_factor(B.FACTOR_Q_BAR, l))
        got[flags] = facs
        _say("  ", name, rep)
        comp.close()
    for x, y in zip(got[0], got[B.FLAG_NO_COOPERATIVE_LAUNCH]):
        assert np.array_equal(x, y), "the one-launch and the three-launch form differ"


def test_more_tall_factors_than_one_launch_can_hold():
    """100 (layer, worker) pairs of 16 slices each are more workgroups than fit the chip at once: the
    Cholesky-QR Gram-Schmidt has to take its three-launch form by itself (no flag), and the sampled
    layers and workers must still agree with the oracle at every stage."""
    _say("case: tall factors, one-launch form does not fit")
    layers, rank, W = [(4096, 256)] * 20, 16, 5
    rng = np.random.default_rng(5)
    comp, ml = _make(layers, (), rank, 8, 8, W)
    Q = [rng.standard_normal((c, rank)).astype(f32) for r, c in layers]
    for l in ml:
        comp.set_q(l, Q[l])
    G = _random_inputs(rng, layers, W)
    E = [[np.zeros(s, f32) for s in layers] for _ in range(W)]
    rep = pu.StageReport()
    pu.staged_iteration(comp, G, pu.to_device(G), E, Q, ml, rep, layers_to_check=[0, 7, 13, 19], workers_to_check=[0, 2, 4])
    assert comp.launched_kernel(B.KERNEL_ORTH) == "orth_chol_kernel<16> x 3 launches", comp.launched_kernel(B.KERNEL_ORTH)
    _say("  ", rep)
    comp.close()
