"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Everything here needs a real MI355X."""
import zlib

import numpy as np
import pytest

import oracle.lqsgd_oracle as orc
from paper_2506_17974_amd import binding as B
from paper_2506_17974_amd import workloads as wl
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu
f32, f64 = np.float32, np.float64


def _say(*a):
    print(*a, flush=True)


def _vector_mean_ok(got, vs):
    """fp32 sum of W values in worker order, then one division: W + 1 roundings,
    each relative to the running magnitude."""
    want = orc.vector_mean(vs)
    bound = (len(vs) + 1) * 6e-8 * sum(np.abs(v).astype(f64) for v in vs) + 1e-30
    return bool(np.all(np.abs(got.astype(f64) - want) <= bound))


def _make(layers, vectors, rank, bits_p, bits_q, W, alpha=255.0, flags=0):
    ll = B.layer_list(layers, vectors)
    return B.Compressor(ll, rank, bits_p, bits_q, W, alpha, flags), list(range(len(layers)))


def _random_inputs(rng, layers, W, dist="normal", scale=1e-3):
    def draw(shape):
        if dist == "student_t3":
            return (rng.standard_t(3.0, size=shape) * scale).astype(f32)
        return (rng.standard_normal(shape) * scale).astype(f32)
    return [[draw(s) for s in layers] for _ in range(W)]


def _run_staged(layers, rank, bits_p, bits_q, W, alpha=255.0, steps=2, seed=0, dist="normal", e0_scale=0.0):
    """`steps` staged iterations, error feedback carried on the device, each
    stage checked against the oracle."""
    rng = np.random.default_rng(seed)
    comp, ml = _make(layers, (), rank, bits_p, bits_q, W, alpha)
    Q = [rng.standard_normal((c, min(rank, r, c))).astype(f32) for r, c in layers]
    E = [[(rng.standard_normal(s) * e0_scale).astype(f32) for s in layers] for _ in range(W)]
    for l in ml:
        comp.set_q(l, Q[l])
        if e0_scale:
            for w in range(W):
                comp.set_state(l, w, e=E[w][l])
    rep = pu.StageReport()
    for t in range(steps):
        G = _random_inputs(rng, layers, W, dist)
        Gd = pu.to_device(G)
        E, Q = pu.staged_iteration(comp, G, Gd, E, Q, ml, rep)
    comp.close()
    return rep


# ---------------------------------------------------------------------------
# benchmark config 0: one 256 x 128 layer, r = 2, b = 8, W = 2
# ---------------------------------------------------------------------------
def test_fc_256x128_staged_and_free_run():
    w = wl.fc_256x128()
    _say("case: fc_256x128 staged")
    comp, ml = _make(w.layers, (), w.rank, w.bits, w.bits, w.workers, w.alpha)
    Q0 = [wl.initial_q(w, 0)]
    comp.set_q(0, Q0[0])
    G = wl.host_step_inputs(w, 0)
    E0 = [[np.zeros(w.layers[0], f32)] for _ in range(w.workers)]
    rep = pu.StageReport()
    E1, Q1 = pu.staged_iteration(comp, G, pu.to_device(G), E0, Q0, ml, rep)
    _say("  ", rep)
    # the same step free-running through lqsgd_step on a fresh context: same bits
    comp2, _ = _make(w.layers, (), w.rank, w.bits, w.bits, w.workers, w.alpha)
    comp2.set_q(0, Q0[0])
    import torch
    ghat = [torch.empty(w.layers[0], device="cuda", dtype=torch.float32)]
    comp2.step(pu.to_device(G), ghat)
    for k in range(w.workers):
        e2, q2 = comp2.get_state(0, k)
        assert np.array_equal(e2, E1[k][0]) and np.array_equal(q2, Q1[0])
    # and against the oracle's own free run (insensitive tensors only)
    out = orc.layer_step([G[k][0] for k in range(w.workers)], [E0[k][0] for k in range(w.workers)],
                         Q0[0], w.rank, w.bits, w.bits, w.alpha)
    gh = ghat[0].cpu().numpy()
    _say("   free run: G_hat %.2e  E %.2e" % (pu.rel_fro(gh, out["G_hat"]), pu.rel_fro(E1[0][0], out["E_new"][0])))
    assert pu.rel_fro(E1[0][0], out["E_new"][0]) <= pu.FP_TOL
    for k in range(w.workers):   # Eq. (8) on the device's own outputs
        m = (G[k][0].astype(f64) + E0[k][0]).astype(f32)
        assert np.all(np.abs(gh.astype(f64) + E1[k][0] - m) <= 5e-7 * (np.abs(gh) + np.abs(m)) + 1e-9)
    comp.close(); comp2.close()


# ---------------------------------------------------------------------------
# shapes, ranks, bit widths, worker counts: tails, odd sizes, degenerate cases
# ---------------------------------------------------------------------------
EDGE_CASES = [
    # layers, rank, bits_p, bits_q, W, alpha
    ([(1, 1)], 1, 8, 8, 1, 255.0),
    ([(1, 7), (7, 1)], 4, 8, 8, 2, 255.0),
    ([(5, 3), (64, 27), (32, 25)], 4, 8, 8, 4, 255.0),
    ([(10, 512), (3, 1024)], 16, 8, 8, 2, 255.0),          # rank clipped to rows: 10, 3
    ([(300, 260)], 3, 8, 8, 3, 255.0),                     # odd rank, odd W
    ([(300, 260)], 7, 4, 4, 5, 255.0),
    ([(17, 4100)], 4, 8, 8, 2, 255.0),                     # several column segments + tail
    ([(1000, 68)], 8, 8, 8, 2, 255.0),
    ([(129, 1028)], 1, 8, 8, 2, 255.0),
    ([(129, 1028)], 2, 2, 2, 2, 255.0),
    ([(129, 1028)], 16, 8, 4, 2, 255.0),                   # b_p != b_q
    ([(96, 520)], 32, 8, 8, 2, 255.0),
    ([(200, 1100), (10, 512), (64, 27)], 32, 8, 8, 2, 255.0),  # full, clipped (padded operand copies) and unaligned layers together
    ([(100, 1100), (33, 64)], 20, 8, 8, 2, 255.0),         # rank 20 in a rank pad of 32
    ([(70, 200)], 12, 8, 8, 2, 255.0),                     # rank 12 in a rank pad of 16
    ([(40, 36)], 32, 8, 8, 2, 255.0),                      # rank 32 clipped to 36 cols / 40 rows
    ([(100, 1100), (70, 200)], 50, 8, 8, 2, 255.0),        # rank 50 in a rank pad of 64 (two blocks of 32 ranks)
    ([(96, 520)], 64, 8, 8, 2, 255.0),
    ([(129, 131), (300, 64)], 40, 8, 4, 2, 255.0),         # pad 64 with unaligned rows (plain fallback) and a clipped rank
    ([(257, 513)], 4, 1, 1, 2, 255.0),
    ([(257, 513)], 4, 3, 5, 2, 255.0),
    ([(257, 513)], 4, 6, 7, 2, 255.0),                     # bit widths that are not whole bytes or nibbles
    ([(257, 513), (64, 27)], 8, 7, 6, 3, 255.0),
    ([(257, 513)], 4, 0, 0, 4, 255.0),                     # quantisation off
    ([(257, 513)], 4, 0, 8, 2, 255.0),
    ([(64, 576), (128, 64)], 4, 8, 8, 8, 1.0),
    ([(64, 576), (128, 64)], 4, 8, 8, 8, 10.0),
    ([(64, 576), (128, 64)], 4, 8, 8, 8, 1000.0),
    ([(2100, 132)], 4, 8, 8, 2, 255.0),                    # several row blocks
    ([(33, 70)], 4, 8, 8, 64, 255.0),                      # the largest worker count: eight passes of eight worker slots
    ([(33, 70)], 4, 8, 4, 9, 255.0),                       # a ragged last pass of worker slots
    ([(3, 70000)], 2, 8, 8, 2, 255.0),                     # very wide: 69 column segments
    ([(70000, 12)], 4, 8, 8, 2, 255.0),                    # very tall: 274 slices, Gram-Schmidt one launch per column
    ([(20000, 16)], 16, 8, 8, 3, 255.0),                   # tall, rank 16, 79 slices: Cholesky-QR in its form of three launches
    ([(17000, 40)], 32, 8, 8, 2, 255.0),                   # the same at rank pad 32 (67 slices)
]


@pytest.mark.parametrize("case", EDGE_CASES, ids=lambda c: "%s-r%d-b%d%d-W%d-a%g" % (
    "+".join("%dx%d" % s for s in c[0]), c[1], c[2], c[3], c[4], c[5]))
def test_edge_cases_staged(case):
    layers, rank, bp, bq, W, alpha = case
    _say("case:", case)
    rep = _run_staged(layers, rank, bp, bq, W, alpha, steps=2, seed=zlib.crc32(str(case).encode()) % 1000, e0_scale=3e-4)
    _say("  ", rep)


def test_heavy_tailed_inputs():
    _say("case: student-t inputs")
    rep = _run_staged([(128, 1152), (64, 27)], 4, 8, 8, 8, steps=2, seed=5, dist="student_t3")
    _say("  ", rep)


def test_zero_gradients():
    _say("case: zero gradients")
    import torch
    layers = [(64, 128), (9, 5)]
    comp, ml = _make(layers, (7,), 4, 8, 8, 2)
    for l in ml:
        comp.set_q(l, np.ones((layers[l][1], min(4, *layers[l])), f32))
    G = [[torch.zeros(s, device="cuda") for s in layers] + [torch.zeros(7, device="cuda")] for _ in range(2)]
    ghat = [torch.full(s, 7.0, device="cuda") for s in layers] + [torch.full((7,), 7.0, device="cuda")]
    comp.step(G, ghat)
    for l in ml:
        for w in range(2):
            e, q = comp.get_state(l, w)
            assert not e.any() and not q.any() and np.all(np.isfinite(q))
            k, sg, sc = comp.get_packet(B.PHASE_P, l, w)
            assert sc == 0 and not k.any() and not sg.any()
        assert not ghat[l].cpu().numpy().any()
    assert not ghat[2].cpu().numpy().any()
    comp.close()


# ---------------------------------------------------------------------------
# benchmark config 1: small CNN, 10 steps, error feedback carried, W = 4
# ---------------------------------------------------------------------------
def test_small_cnn_ten_steps():
    import torch
    w = wl.small_cnn()
    L, V = len(w.layers), len(w.vectors)
    _say("case: small_cnn 10 steps")
    staged, ml = _make(w.layers, w.vectors, w.rank, w.bits, w.bits, w.workers, w.alpha)
    free, _ = _make(w.layers, w.vectors, w.rank, w.bits, w.bits, w.workers, w.alpha)
    Q = [wl.initial_q(w, l) for l in range(L)]
    for l in range(L):
        staged.set_q(l, Q[l]); free.set_q(l, Q[l])
    G_steps = [wl.host_step_inputs(w, t) for t in range(w.steps)]
    # the oracle's own free run of the ten steps
    hist, Eo, Qo = orc.run_steps(G_steps, list(w.layers), Q, w.rank, w.bits, w.bits, w.alpha)
    E = [[np.zeros(s, f32) for s in w.layers] for _ in range(w.workers)]
    rep = pu.StageReport()
    sumG = [np.zeros(s, f64) for s in w.layers]
    sumGhat = [np.zeros(s, f64) for s in w.layers]
    ghat = [torch.empty(s, device="cuda") for s in w.layers] + [torch.empty(n, device="cuda") for n in w.vectors]
    same_codes = [True] * L          # the device's packets have matched the oracle's free run so far
    agreed_steps = [0] * L
    for t in range(w.steps):
        G = G_steps[t]
        Vg = [[wl.vector_gradient(w, t, v, k) for v in range(V)] for k in range(w.workers)]
        Gd = pu.to_device([G[k] + Vg[k] for k in range(w.workers)])
        # every stage against the oracle fed the device's own upstream tensors
        E, Q = pu.staged_iteration(staged, G, Gd, E, Q, ml, rep)
        free.step(Gd, ghat)
        for l in range(L):
            for k in range(w.workers):
                e2, q2 = free.get_state(l, k)
                assert np.array_equal(e2, E[k][l]), "fused step differs from the staged path"
                assert np.array_equal(q2, Q[l])
            sumG[l] += sum(G[k][l].astype(f64) for k in range(w.workers)) / w.workers
            sumGhat[l] += ghat[l].cpu().numpy()
            # Free-running comparison.  Summation order differs between the two
            # sides, so a value on a bucket boundary may take the neighbouring code;
            # from that step on the two runs are different (equally valid)
            # trajectories.  While all packets agree, the residuals must agree to
            # the fp32 tolerance.
            for k in range(w.workers):
                for ph, key in ((B.PHASE_P, "pkt_P"), (B.PHASE_Q, "pkt_Q")):
                    kg, sg, sc = staged.get_packet(ph, l, k)
                    ko, so, sco = hist[t][l][key][k]
                    if not (np.array_equal(kg, ko) and abs(float(sc) - float(sco)) <= 1e-5 * float(sco)):
                        same_codes[l] = False
            if same_codes[l]:
                agreed_steps[l] = t + 1
                for k in range(w.workers):
                    assert pu.rel_fro(E[k][l], hist[t][l]["E_new"][k]) <= pu.FP_TOL
                assert pu.rel_fro(ghat[l].cpu().numpy(), hist[t][l]["G_hat"]) <= pu.FP_TOL
        for v in range(V):
            got = ghat[L + v].cpu().numpy()
            assert _vector_mean_ok(got, [Vg[k][v] for k in range(w.workers)])
            assert np.array_equal(free.get_factor(B.FACTOR_VMEAN, L + v), got)
    _say("  ", rep)
    _say("   steps over which the free-running packets equal the oracle's, per layer:", agreed_steps)
    assert max(agreed_steps) >= 1
    # telescoping: applied updates + residual still owed = gradients that came in
    for l in range(L):
        Ebar = sum(E[k][l].astype(f64) for k in range(w.workers)) / w.workers
        err = np.abs(sumGhat[l] + Ebar - sumG[l]).max()
        assert err <= 5e-6 * np.abs(sumG[l]).max() + 1e-9, (l, err)
        worst = max(pu.rel_fro(E[k][l], Eo[k][l]) for k in range(w.workers))
        _say("   layer %d free-run residual difference after %d steps: %.2e" % (l, w.steps, worst))
    staged.close(); free.close()


# ---------------------------------------------------------------------------
# benchmark config 2: the ResNet-18-shaped set at full size
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("rank,bits", [(4, 8), (2, 8), (4, 4), (2, 4)])
def test_resnet18_full_size(rank, bits):
    w = wl.resnet18(rank, bits)
    L = len(w.layers)
    _say("case: resnet18 r=%d b=%d W=%d (full size)" % (rank, bits, w.workers))
    comp, ml = _make(w.layers, (), rank, bits, bits, w.workers, w.alpha)
    Q = [wl.initial_q(w, l) for l in range(L)]
    for l in range(L):
        comp.set_q(l, Q[l])
    E = [[np.zeros(s, f32) for s in w.layers] for _ in range(w.workers)]
    rep = pu.StageReport()
    # the (4, 8) point carries the residual into a second iteration
    for t in range(2 if (rank, bits) == (4, 8) else 1):
        G = wl.host_step_inputs(w, t)
        E, Q = pu.staged_iteration(comp, G, pu.to_device(G), E, Q, ml, rep)
        _say("   step %d: %s" % (t, rep))
    comp.close()


def test_resnet18_free_run_matches_oracle_and_is_deterministic():
    import torch
    w = wl.resnet18(4, 8)
    L, V = len(w.layers), len(w.vectors)
    _say("case: resnet18 free run + determinism")
    G = wl.host_step_inputs(w, 0)
    Vg = [[wl.vector_gradient(w, 0, v, k) for v in range(V)] for k in range(w.workers)]
    Gd = pu.to_device([G[k] + Vg[k] for k in range(w.workers)])
    Q0 = [wl.initial_q(w, l) for l in range(L)]
    results = []
    for rep_i in range(2):
        comp, ml = _make(w.layers, w.vectors, 4, 8, 8, w.workers, w.alpha)
        for l in range(L):
            comp.set_q(l, Q0[l])
        ghat = [torch.empty(s, device="cuda") for s in w.layers] + [torch.empty(n, device="cuda") for n in w.vectors]
        comp.step(Gd, ghat)
        packets1 = {(ph, l, k): comp.get_packet(ph, l, k) for ph in (B.PHASE_P, B.PHASE_Q)
                    for l in range(L) for k in range(w.workers)}
        comp.step(Gd, ghat)     # second step exercises the carried residual and warm start
        comp.synchronize()
        res = {"E": [[comp.get_state(l, k, want_q=False)[0] for l in range(L)] for k in range(w.workers)],
               "Q": [comp.get_factor(B.FACTOR_Q_BAR, l) for l in range(L)],
               "G": [g.cpu().numpy() for g in ghat], "packets1": packets1,
               "packets": {(ph, l, k): comp.get_packet(ph, l, k) for ph in (B.PHASE_P, B.PHASE_Q)
                           for l in range(L) for k in range(w.workers)}}
        results.append(res)
        comp.close()
    a, b = results
    for l in range(L):
        assert np.array_equal(a["Q"][l], b["Q"][l]) and np.array_equal(a["G"][l], b["G"][l])
        for k in range(w.workers):
            assert np.array_equal(a["E"][k][l], b["E"][k][l])
    # The oracle's own free run.  Summation order differs, so a factor value that
    # sits on a bucket boundary may take the neighbouring code on one side; that
    # moves one entry of P-bar or Q-bar by one quantisation step and everything
    # after it.  Layers whose packets all agree must match to the fp32 tolerance;
    # the others are reported and held to the size of such a step.
    hist, Eo, Qo = orc.run_steps([G, G], list(w.layers), Q0, 4, 8, 8, w.alpha)
    pk = results[1]["packets"]
    n_codes = n_flips = 0
    for l in range(L):
        flips = 0
        for k in range(w.workers):
            for ph, key in ((B.PHASE_P, "pkt_P"), (B.PHASE_Q, "pkt_Q")):
                kg = pk[(ph, l, k)][0]
                ko = hist[1][l][key][k][0]
                flips += int((kg != ko).sum())
                n_codes += kg.size
        n_flips += flips
        err_e = max(pu.rel_fro(a["E"][k][l], Eo[k][l]) for k in range(w.workers))
        err_g = pu.rel_fro(a["G"][l], hist[1][l]["G_hat"])
        _say("   layer %2d %4dx%-4d: code diffs in step 2: %3d, E %.2e, G_hat %.2e" % (
            l, w.layers[l][0], w.layers[l][1], flips, err_e, err_g))
        clean = all(np.array_equal(results[1]["packets1"][(ph, l, k)][0], hist[0][l][key][k][0])
                    for k in range(w.workers) for ph, key in ((B.PHASE_P, "pkt_P"), (B.PHASE_Q, "pkt_Q")))
        if flips == 0 and clean:
            assert err_e <= pu.FP_TOL and err_g <= pu.FP_TOL
        else:
            assert err_e <= 5e-3 and err_g <= 5e-2
    _say("   free run: %d of %d codes differ from the oracle's free run in step 2" % (n_flips, n_codes))
    # Step 1 starts from identical state on both sides.  A P code can then differ only where a
    # value sits on a bucket boundary (summation order): by one level, and rarely.  Q_w = M^T P-bar
    # inherits every such flip (one entry of P-bar moves by one quantisation step, times a row of a
    # heavy-tailed M), so its codes differ more often and by more than one level; reported, and
    # held to a small fraction.
    st = {B.PHASE_P: [0, 0, 0], B.PHASE_Q: [0, 0, 0]}       # codes, differing, largest difference
    for (ph, l, k), (kg, _, _) in results[1]["packets1"].items():
        ko = hist[0][l]["pkt_P" if ph == B.PHASE_P else "pkt_Q"][k][0]
        diff = np.abs(kg.astype(np.int32) - ko.astype(np.int32))
        st[ph][0] += kg.size
        st[ph][1] += int((diff != 0).sum())
        st[ph][2] = max(st[ph][2], int(diff.max()))
    _say("   free run, step 1: P codes %d of %d differ (largest %d level), Q codes %d of %d differ (largest %d levels)" % (
        st[B.PHASE_P][1], st[B.PHASE_P][0], st[B.PHASE_P][2], st[B.PHASE_Q][1], st[B.PHASE_Q][0], st[B.PHASE_Q][2]))
    assert st[B.PHASE_P][2] <= 1 and st[B.PHASE_P][1] <= 1e-4 * st[B.PHASE_P][0]
    assert st[B.PHASE_Q][1] <= 5e-3 * st[B.PHASE_Q][0]
    for v in range(V):
        assert _vector_mean_ok(a["G"][L + v], [Vg[k][v] for k in range(w.workers)])


# ---------------------------------------------------------------------------
# run-to-run determinism of the paths that add partial results across work items
# (matrix-core sweeps, the one-launch Gram-Schmidt with its slice tables)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("layers,rank,W", [
    ([(200, 1100), (10, 512), (64, 27)], 32, 3),      # narrow matrix-core sweep 0, padded operand copies
    ([(129, 1028), (70, 27)], 16, 2),
    ([(100, 1100), (70, 200)], 50, 2),                 # rank pad 64
    ([(20000, 16)], 16, 3),                            # tall factor: Gram-Schmidt in 79 slices (Cholesky-QR, three launches)
    ([(8192, 96)], 32, 2),                             # tall factor, 32 slices: the one-launch form
])
def test_three_steps_twice_give_the_same_bits(layers, rank, W):
    import torch
    _say("case: determinism", layers, rank, W)
    rng = np.random.default_rng(11)
    Q0 = [rng.standard_normal((c, min(rank, r, c))).astype(f32) for r, c in layers]
    Gs = [pu.to_device(_random_inputs(rng, layers, W)) for _ in range(3)]
    runs = []
    for rep in range(2):
        # the second run must not launch cooperatively: the tall factor's Gram-Schmidt then takes its
        # one-launch-per-column form, which has to give the same bits as the one-launch form
        comp, ml = _make(layers, (), rank, 8, 8, W, flags=B.FLAG_NO_COOPERATIVE_LAUNCH if rep else 0)
        for l in ml:
            comp.set_q(l, Q0[l])
        ghat = [torch.empty(s, device="cuda") for s in layers]
        for G in Gs:
            comp.step(G, ghat)
        comp.synchronize()
        runs.append(([g.cpu().numpy() for g in ghat],
                     [[comp.get_state(l, w) for l in ml] for w in range(W)]))
        comp.close()
    (ga, sa), (gb, sb) = runs
    for l in range(len(layers)):
        assert np.array_equal(ga[l], gb[l])
        for w in range(W):
            assert np.array_equal(sa[w][l][0], sb[w][l][0]) and np.array_equal(sa[w][l][1], sb[w][l][1])


# ---------------------------------------------------------------------------
# deferred residual update (the default) against the eager one: same bits
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("layers,rank,bits,W", [
    ([(64, 576), (128, 64), (64, 27), (10, 512)], 4, 8, 4),
    ([(300, 260), (17, 4100)], 3, 4, 3),
    ([(96, 520)], 16, 8, 2),
    ([(96, 520), (40, 36), (70, 27), (200, 1100), (10, 512)], 32, 8, 2),   # matrix-core path, clipped ranks, unaligned rows
    ([(130, 260)], 20, 4, 3),                                      # rank pad 32 with rank 20
    ([(200, 1100), (70, 27), (96, 520)], 50, 8, 2),                # rank pad 64
])
def test_deferred_residual_is_bit_identical_to_eager(layers, rank, bits, W):
    import torch
    _say("case: deferred vs eager residual", layers, rank, bits, W)
    rng = np.random.default_rng(17)
    vectors = (33,)
    lazy, ml = _make(layers, vectors, rank, bits, bits, W)
    eager, _ = _make(layers, vectors, rank, bits, bits, W, flags=B.FLAG_EAGER_RESIDUAL)
    for l in ml:
        q0 = rng.standard_normal((layers[l][1], min(rank, *layers[l]))).astype(f32)
        lazy.set_q(l, q0); eager.set_q(l, q0)
    n = len(layers)
    gl = [torch.empty(s, device="cuda") for s in layers] + [torch.empty(33, device="cuda")]
    ge = [torch.empty(s, device="cuda") for s in layers] + [torch.empty(33, device="cuda")]
    for t in range(5):
        G = _random_inputs(rng, layers, W)
        Gd = pu.to_device([G[k] + [rng.standard_normal(33).astype(f32)] for k in range(W)])
        lazy.step(Gd, gl if t != 2 else None)       # one step without G-hat
        eager.step(Gd, ge if t != 2 else None)
        for l in range(n + 1):
            if t != 2:
                assert torch.equal(gl[l], ge[l]), (t, l)
        for l in ml:
            assert np.array_equal(lazy.get_factor(B.FACTOR_Q_BAR, l), eager.get_factor(B.FACTOR_Q_BAR, l))
            assert np.array_equal(lazy.get_factor(B.FACTOR_P_BAR, l), eager.get_factor(B.FACTOR_P_BAR, l))
        if t in (1, 3):          # reading the state applies the deferred update; the run must not notice
            for l in ml:
                for k in range(W):
                    assert np.array_equal(lazy.get_state(l, k)[0], eager.get_state(l, k)[0]), (t, l, k)
        if t == 3:               # overwriting one residual while an update is deferred
            e_new = (rng.standard_normal(layers[0]) * 1e-4).astype(f32)
            lazy.set_state(0, W - 1, e=e_new); eager.set_state(0, W - 1, e=e_new)
    for l in ml:
        for k in range(W):
            el, ql = lazy.get_state(l, k)
            ee, qe = eager.get_state(l, k)
            assert np.array_equal(el, ee) and np.array_equal(ql, qe)
    lazy.close(); eager.close()


# ---------------------------------------------------------------------------
# the C ABI's error behaviour on a live context
# ---------------------------------------------------------------------------
def test_abi_errors():
    import torch
    _say("case: ABI errors")
    layers = [(16, 8)]
    comp, ml = _make(layers, (4,), 2, 8, 8, 2)
    G = [[torch.zeros(16, 8, device="cuda"), torch.zeros(4, device="cuda")] for _ in range(2)]
    with pytest.raises(B.LqsgdError) as ei:
        comp.decompress(B.PHASE_P)
    assert ei.value.code == B.ESTATE
    with pytest.raises(B.LqsgdError) as ei:
        comp.compress(B.PHASE_Q)
    assert ei.value.code == B.ESTATE
    comp.compress(B.PHASE_P, G)
    with pytest.raises(B.LqsgdError) as ei:
        comp.step(G)
    assert ei.value.code == B.ESTATE
    comp.decompress(B.PHASE_P); comp.compress(B.PHASE_Q); comp.decompress(B.PHASE_Q)
    with pytest.raises(B.LqsgdError) as ei:
        comp.get_state(5, 0)
    assert ei.value.code == B.ESHAPE
    with pytest.raises(B.LqsgdError) as ei:
        comp.get_state(1, 0)            # a VECTOR layer has no residual
    assert ei.value.code == B.ESHAPE
    with pytest.raises(B.LqsgdError) as ei:
        comp.get_state(0, 2)
    assert ei.value.code == B.ESHAPE
    with pytest.raises(B.LqsgdError) as ei:
        comp.get_factor(99, 0)
    assert ei.value.code == B.EINVAL
    # misaligned gradient pointer
    base = torch.zeros(16 * 8 + 1, device="cuda")
    bad = [[base[1:].view(16, 8), G[0][1]], G[1]]
    with pytest.raises(B.LqsgdError) as ei:
        comp.step(bad)
    assert ei.value.code == B.EINVAL
    # G-hat aliasing a gradient
    with pytest.raises(B.LqsgdError) as ei:
        comp.step(G, [G[0][0], None])
    assert ei.value.code == B.EINVAL
    comp.step(G)                        # still usable afterwards
    comp.close()
    comp.close()                        # double close is safe
    off, _ = _make(layers, (), 2, 0, 0, 2)
    off.step([[G[0][0]], [G[1][0]]])
    with pytest.raises(B.LqsgdError) as ei:
        off.get_packet(B.PHASE_P, 0, 0)
    assert ei.value.code == B.EUNSUPPORTED
    off.close()


def test_packet_injection_round_trip():
    """set_packet followed by decompress gives the oracle's mean of those packets."""
    _say("case: packet injection")
    rng = np.random.default_rng(9)
    layers = [(70, 36)]
    W, r, bits = 3, 4, 5
    comp, ml = _make(layers, (), r, bits, bits, W)
    comp.set_q(0, rng.standard_normal((36, r)).astype(f32))
    G = _random_inputs(rng, layers, W)
    comp.compress(B.PHASE_P, pu.to_device(G))
    pk = []
    for w in range(W):
        k = rng.integers(0, 1 << bits, (70, r)).astype(np.uint8)
        sg = (rng.integers(0, 2, (70, r)) & (k > 0)).astype(np.uint8)
        sc = f32(rng.uniform(0.1, 2.0))
        comp.set_packet(B.PHASE_P, 0, w, k, sg, sc)
        k2, s2, sc2 = comp.get_packet(B.PHASE_P, 0, w)
        assert np.array_equal(k, k2) and np.array_equal(sg, s2) and sc == sc2
        pk.append((k, sg, sc))
    comp.decompress(B.PHASE_P)
    got = comp.get_factor(B.FACTOR_P_BAR, 0)
    assert pu.rel_fro(got, orc.mean_of_packets(pk, bits, 255.0)) <= pu.MEAN_TOL
    comp.close()


def test_two_contexts_on_their_own_streams():
    """Contexts are independent: two of them, each on a stream of its own, stepping
    in turn without host synchronisation in between, give bit for bit what a context
    on the default stream gives when run alone."""
    import torch
    _say("case: two contexts on two streams")
    layers, vectors, W, rank = [(128, 1152), (64, 27), (2304, 96)], (33,), 4, 4
    rng = np.random.default_rng(17)
    ll = B.layer_list(layers, vectors)
    shapes = list(layers) + [(v,) for v in vectors]
    q0 = [rng.standard_normal((c, min(rank, r, c))).astype(f32) for r, c in layers]
    steps = [[[torch.from_numpy((rng.standard_normal(s) * 1e-3).astype(f32)).cuda() for s in shapes] for _ in range(W)]
             for _ in range(3)]
    torch.cuda.synchronize()

    def make(stream):
        c = B.Compressor(ll, rank, 8, 8, W, 255.0, 0, stream=stream)
        for l in range(len(layers)):
            c.set_q(l, q0[l])
        return c

    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    a, b = make(s1.cuda_stream), make(s2.cuda_stream)
    ga = [torch.zeros(s, device="cuda") for s in shapes]
    gb = [torch.zeros(s, device="cuda") for s in shapes]
    for t in range(3):
        a.step(steps[t], ga)
        b.step(steps[2 - t], gb)          # a different order of inputs on the second context
    a.synchronize(); b.synchronize()
    ref = make(None)
    gr = [torch.zeros(s, device="cuda") for s in shapes]
    for t in range(3):
        ref.step(steps[t], gr)
    ref.synchronize()
    for l in range(len(layers)):
        assert torch.equal(ga[l], gr[l])
        for w in range(W):
            ea, qa = a.get_state(l, w)
            er, qr = ref.get_state(l, w)
            assert np.array_equal(ea, er) and np.array_equal(qa, qr)
    ref2 = make(None)
    for t in range(3):
        ref2.step(steps[2 - t], gr)
    ref2.synchronize()
    for l in range(len(layers)):
        assert torch.equal(gb[l], gr[l])
    for c in (a, b, ref, ref2):
        c.close()


def test_vector_only_context():
    """No matrix layer at all: the step is the plain mean of the 1-D tensors, the staged
    calls are empty iterations, and nothing is launched on empty work lists."""
    import torch
    _say("case: vector layers only")
    W, lens = 3, (7, 1000, 1)
    rng = np.random.default_rng(4)
    comp = B.Compressor(B.layer_list((), lens), 4, 8, 8, W)
    G = [[torch.from_numpy(rng.standard_normal(n).astype(f32)).cuda() for n in lens] for _ in range(W)]
    out = [torch.zeros(n, device="cuda") for n in lens]
    comp.step(G, out)
    comp.synchronize()
    for i, n in enumerate(lens):
        assert _vector_mean_ok(out[i].cpu().numpy(), [G[w][i].cpu().numpy() for w in range(W)])
        assert np.array_equal(comp.get_factor(B.FACTOR_VMEAN, i), out[i].cpu().numpy())
    comp.compress(B.PHASE_P, G); comp.decompress(B.PHASE_P); comp.compress(B.PHASE_Q); comp.decompress(B.PHASE_Q)
    comp.step(G)
    assert comp.wire_bytes() == 0
    comp.close()
