"""GPU parity of the two variants around Algorithm 1: the PowerSGD order of
Section 3.2 (aggregate, then orthonormalise) and the fused model update
w <- w - eta G-hat (Algorithm 1, last statement).  Needs a real MI355X."""
import zlib

import numpy as np
import pytest

import oracle.lqsgd_oracle as orc
from paper_2506_17974_amd import binding as B
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu
f32, f64 = np.float32, np.float64


def _say(*a):
    print(*a, flush=True)


def _inputs(rng, layers, W, scale=1e-3):
    return [[(rng.standard_normal(s) * scale).astype(f32) for s in layers] for _ in range(W)]


AGG_CASES = [
    # layers, rank, bits_p, bits_q, W
    ([(256, 128)], 2, 8, 8, 2),
    ([(5, 3), (64, 27), (32, 25)], 4, 8, 8, 4),
    ([(300, 260)], 3, 0, 0, 3),                      # PowerSGD itself
    ([(300, 260)], 7, 4, 4, 5),
    ([(17, 4100)], 4, 8, 8, 2),
    ([(2100, 132), (1000, 68)], 8, 8, 4, 2),
    ([(129, 1028)], 16, 8, 8, 2),                    # matrix-core sweeps 0 / 2
    ([(100, 1100), (33, 64)], 20, 8, 8, 2),          # rank pad 32
    ([(2304, 96)], 4, 8, 8, 1),                      # one worker, tall: one-launch many-workgroup Gram-Schmidt
    ([(4608, 64)], 32, 8, 8, 2),                     # tall + rank 32: the same on the aggregate, 18 slices
    ([(2304, 72), (70, 200)], 50, 8, 8, 2),          # rank pad 64
]


@pytest.mark.parametrize("case", AGG_CASES, ids=lambda c: "%s-r%d-b%d%d-W%d" % (
    "+".join("%dx%d" % s for s in c[0]), c[1], c[2], c[3], c[4]))
def test_aggregate_first_staged(case):
    layers, rank, bp, bq, W = case
    _say("case: aggregate-first", case)
    rng = np.random.default_rng(zlib.crc32(str(case).encode()) % 1000)
    comp = B.Compressor(B.layer_list(layers, ()), rank, bp, bq, W, 255.0, B.FLAG_AGGREGATE_FIRST)
    ml = list(range(len(layers)))
    Q = [rng.standard_normal((c, min(rank, r, c))).astype(f32) for r, c in layers]
    E = [[(rng.standard_normal(s) * 3e-4).astype(f32) for s in layers] for _ in range(W)]
    for l in ml:
        comp.set_q(l, Q[l])
        for w in range(W):
            comp.set_state(l, w, e=E[w][l])
    rep = pu.StageReport()
    for t in range(2):
        G = _inputs(rng, layers, W)
        E, Q = pu.staged_iteration(comp, G, pu.to_device(G), E, Q, ml, rep, aggregate_first=True)
    with pytest.raises(B.LqsgdError) as ei:
        comp.get_factor(B.FACTOR_P_ORTH, 0, 0)
    assert ei.value.code == B.EINVAL
    comp.close()
    _say("  ", rep)


# Aggregate-first on a tall factor at rank pad >= 16: Gram-Schmidt of the aggregate runs in place on
# P-bar, through Cholesky-QR; with two nearly parallel columns its pivot test fails and the factor is
# done column by column from the copy of the aggregate kept aside.  Both launch forms, same bits.
@pytest.mark.parametrize("layers,rank,eps", [([(4608, 64)], 32, 4e-3), ([(2560, 200)], 16, 4e-3), ([(2560, 200)], 16, None)])
def test_aggregate_first_tall_factor_with_nearly_dependent_columns(layers, rank, eps):
    _say("case: aggregate-first, tall, Cholesky-QR", layers, rank, eps)
    W = 2
    rng = np.random.default_rng(rank)
    ml = list(range(len(layers)))
    Q = []
    for r_, c_ in layers:
        q = rng.standard_normal((c_, min(rank, r_, c_))).astype(f32)
        if eps:
            q[:, 3] = q[:, 1] + eps * rng.standard_normal(c_).astype(f32)
        Q.append(q)
    G = _inputs(rng, layers, W)
    Gd = pu.to_device(G)
    got = {}
    for flags in (0, B.FLAG_NO_COOPERATIVE_LAUNCH):
        comp = B.Compressor(B.layer_list(layers, ()), rank, 8, 8, W, 255.0, B.FLAG_AGGREGATE_FIRST | flags)
        for l in ml:
            comp.set_q(l, Q[l])
        E = [[np.zeros(s, f32) for s in layers] for _ in range(W)]
        rep = pu.StageReport()
        pu.staged_iteration(comp, G, Gd, E, Q, ml, rep, aggregate_first=True)
        got[flags] = [comp.get_factor(B.FACTOR_P_BAR, l) for l in ml] + [comp.get_factor(B.FACTOR_Q_BAR, l) for l in ml]
        _say("  ", comp.launched_kernel(B.KERNEL_ORTH), rep)
        comp.close()
    for x, y in zip(got[0], got[B.FLAG_NO_COOPERATIVE_LAUNCH]):
        assert np.array_equal(x, y), "the one-launch and the three-launch form differ"


def test_p_mean_needs_the_flag():
    comp = B.Compressor(B.layer_list([(16, 8)], ()), 2, 8, 8, 2)
    with pytest.raises(B.LqsgdError) as ei:
        comp.get_factor(B.FACTOR_P_MEAN, 0, 0)
    assert ei.value.code == B.EINVAL
    comp.close()


@pytest.mark.parametrize("rank,bits,flags", [(4, 8, 0), (4, 0, 0), (16, 8, 0), (4, 8, B.FLAG_EAGER_RESIDUAL)])
def test_aggregate_first_fused_step_equals_staged(rank, bits, flags):
    """lqsgd_step, the staged calls, and the deferred / eager residual schedules
    give bit-identical state and G-hat in the aggregate-first order too."""
    import torch
    _say("case: aggregate-first fused vs staged", rank, bits, flags)
    layers, vectors, W = [(128, 1152), (64, 27), (70, 200)], (33,), 4
    rng = np.random.default_rng(rank * 10 + bits)
    ll = B.layer_list(layers, vectors)
    a = B.Compressor(ll, rank, bits, bits, W, 255.0, B.FLAG_AGGREGATE_FIRST | flags)
    b = B.Compressor(ll, rank, bits, bits, W, 255.0, B.FLAG_AGGREGATE_FIRST)
    for l, (r, c) in enumerate(layers):
        q = rng.standard_normal((c, min(rank, r, c))).astype(f32)
        a.set_q(l, q); b.set_q(l, q)
    for t in range(3):
        G = [[(rng.standard_normal(s) * 1e-3).astype(f32) for s in layers] +
             [(rng.standard_normal(v) * 1e-3).astype(f32) for v in vectors] for _ in range(W)]
        Gd = pu.to_device(G)
        ghat = [torch.zeros(s, device="cuda") for s in layers] + [torch.zeros(v, device="cuda") for v in vectors]
        a.step(Gd, ghat)
        b.compress(B.PHASE_P, Gd); b.decompress(B.PHASE_P); b.compress(B.PHASE_Q); b.decompress(B.PHASE_Q)
        for l in range(len(layers)):
            pa, qa = a.get_factor(B.FACTOR_P_BAR, l), a.get_factor(B.FACTOR_Q_BAR, l)
            assert np.array_equal(pa, b.get_factor(B.FACTOR_P_BAR, l))
            assert np.array_equal(qa, b.get_factor(B.FACTOR_Q_BAR, l))
            assert np.array_equal(a.get_factor(B.FACTOR_P_MEAN, l), b.get_factor(B.FACTOR_P_MEAN, l))
            want = (pa.astype(f64) @ qa.astype(f64).T)
            got = ghat[l].cpu().numpy()
            assert pu.rel_fro(got, want) <= pu.FP_TOL
            for w in range(W):
                ea, _ = a.get_state(l, w)
                eb, _ = b.get_state(l, w)
                assert np.array_equal(ea, eb)
    a.close(); b.close()


def test_powersgd_recovers_a_low_rank_mean_for_any_w():
    """bits = 0, aggregate-first: distinct full-rank worker gradients whose mean has
    rank r are reconstructed exactly (the property Algorithm 1's own order gives
    up), and the result matches the oracle run on the same inputs."""
    import torch
    _say("case: PowerSGD exact recovery")
    rng = np.random.default_rng(99)
    rows, cols, r, W = 192, 320, 4, 6
    base = rng.standard_normal((rows, r)) @ rng.standard_normal((r, cols))
    N = [rng.standard_normal((rows, cols)) for _ in range(W)]
    Nbar = sum(N) / W
    G = [[(base + N[w] - Nbar).astype(f32)] for w in range(W)]
    Mbar = sum(g[0].astype(f64) for g in G) / W
    q0 = rng.standard_normal((cols, r)).astype(f32)
    comp = B.Compressor(B.layer_list([(rows, cols)], ()), r, 0, 0, W, 255.0, B.FLAG_AGGREGATE_FIRST)
    comp.set_q(0, q0)
    ghat = [torch.zeros((rows, cols), device="cuda")]
    comp.step(pu.to_device(G), ghat)
    got = ghat[0].cpu().numpy()
    assert np.linalg.norm(got - Mbar) <= 1e-5 * np.linalg.norm(Mbar)
    want = orc.layer_step_aggregate_first([g[0] for g in G], [np.zeros((rows, cols), f32)] * W, q0, r, 0, 0, 255.0)
    assert pu.rel_fro(got, want["G_hat"]) <= pu.FP_TOL
    for w in range(W):
        e, qb = comp.get_state(0, w)
        assert pu.rel_fro(e, want["E_new"][w]) <= pu.FP_TOL
        assert pu.rel_fro(qb, want["Q_bar"]) <= pu.FP_TOL
    comp.close()


def _ulp_close(got, want, frac=1e-5):
    """Equal up to one float32 ulp, on at most `frac` of the elements (the oracle
    rounds a float64 result to float32, the kernel rounds a fused multiply-add once)."""
    got = np.asarray(got, f32); want = np.asarray(want, f32)
    diff = got != want
    if not diff.any():
        return True
    ok = np.abs(got[diff].astype(f64) - want[diff].astype(f64)) <= np.spacing(np.abs(want[diff])).astype(f64)
    return bool(ok.all() and diff.mean() <= frac)


@pytest.mark.parametrize("layers,rank,bits,W,flags", [
    ([(256, 128)], 2, 8, 2, 0),
    ([(64, 576), (128, 64), (10, 512), (33, 65)], 4, 8, 4, 0),
    ([(64, 576), (128, 64)], 4, 8, 4, B.FLAG_EAGER_RESIDUAL),
    ([(129, 1028), (70, 200)], 16, 8, 2, 0),                       # matrix-core G-hat pass
    ([(96, 520)], 32, 4, 2, B.FLAG_EAGER_RESIDUAL),
    ([(96, 520), (129, 131)], 50, 8, 2, 0),                        # rank pad 64, with an unaligned layer
    ([(300, 260)], 3, 0, 3, B.FLAG_AGGREGATE_FIRST),
])
def test_model_update(layers, rank, bits, W, flags):
    """lqsgd_step_update applies w <- w - eta G-hat with the very G-hat lqsgd_step
    writes, leaves the compressor state identical, updates 1-D tensors with their
    mean, and skips tensors whose parameter pointer is NULL."""
    import torch
    _say("case: model update", layers, rank, bits, W, flags)
    vectors = (40, 7)
    rng = np.random.default_rng(rank + bits + W)
    ll = B.layer_list(layers, vectors)
    a = B.Compressor(ll, rank, bits, bits, W, 255.0, flags)
    b = B.Compressor(ll, rank, bits, bits, W, 255.0, flags)
    for l, (r, c) in enumerate(layers):
        q = rng.standard_normal((c, min(rank, r, c))).astype(f32)
        a.set_q(l, q); b.set_q(l, q)
    shapes = list(layers) + [(v,) for v in vectors]
    w_host = [rng.standard_normal(s).astype(f32) for s in shapes]
    params = [torch.from_numpy(w.copy()).cuda() for w in w_host]
    skipped = len(layers) - 1                      # this matrix keeps its parameters
    plist = list(params)
    plist[skipped] = None
    for t, eta in enumerate((0.1, 0.25, 3e-2)):
        G = [[(rng.standard_normal(s) * 1e-1).astype(f32) for s in shapes] for _ in range(W)]
        Gd = pu.to_device(G)
        ghat = [torch.zeros(s, device="cuda") for s in shapes]
        b.step(Gd, ghat)
        a.step_update(Gd, plist, eta)
        for i, s in enumerate(shapes):
            got = params[i].cpu().numpy()
            if i == skipped:
                assert np.array_equal(got, w_host[i])
                continue
            want = orc.model_update(w_host[i], ghat[i].cpu().numpy(), eta)
            assert _ulp_close(got, want), "tensor %d step %d" % (i, t)
            w_host[i] = got
        for l in range(len(layers)):
            for w in range(W):
                ea, qa = a.get_state(l, w)
                eb, qb = b.get_state(l, w)
                assert np.array_equal(ea, eb) and np.array_equal(qa, qb)
        for vi, v in enumerate(vectors):
            i = len(layers) + vi
            assert np.array_equal(a.get_factor(B.FACTOR_VMEAN, i), b.get_factor(B.FACTOR_VMEAN, i))
    # argument errors
    with pytest.raises(B.LqsgdError) as ei:
        a.step_update(Gd, plist, float("nan"))
    assert ei.value.code == B.EINVAL
    bad = list(plist)
    bad[0] = Gd[0][0]
    with pytest.raises(B.LqsgdError) as ei:
        a.step_update(Gd, bad, 0.1)
    assert ei.value.code == B.EINVAL
    a.close(); b.close()


@pytest.mark.parametrize("rank", [4, 32])     # column by column (orth_coop_kernel) / Cholesky-QR (orth_chol_kernel)
def test_expired_device_wait_is_reported(monkeypatch, rank):
    """The one-launch Gram-Schmidt kernels for tall factors wait for other workgroups with
    a bounded number of polls.  With the bound forced to one poll from the host the
    waits expire (the kernel still runs to its end), the context raises its status
    word, and every synchronising call reports it instead of returning bad data."""
    import torch
    _say("case: expired device-side wait, rank", rank)
    rows, cols, W = 8192, 64, 4
    rng = np.random.default_rng(3)
    G = [[torch.from_numpy((rng.standard_normal((rows, cols)) * 1e-3).astype(f32)).cuda()] for _ in range(W)]
    q0 = rng.standard_normal((cols, rank)).astype(f32)
    # healthy run first: same shape, default bound
    ok = B.Compressor(B.layer_list([(rows, cols)], ()), rank, 8, 8, W)
    ok.set_q(0, q0)
    ok.step(G)
    ok.synchronize()
    p = ok.get_factor(B.FACTOR_P_ORTH, 0, 0).astype(f64)
    assert np.allclose(p.T @ p, np.eye(rank), atol=1e-4)
    ok.close()
    monkeypatch.setenv("LQSGD_TABLE_POLLS", "1")
    bad = B.Compressor(B.layer_list([(rows, cols)], ()), rank, 8, 8, W)
    bad.set_q(0, q0)
    raised = False
    for _ in range(3):
        bad.step(G)
        try:
            bad.synchronize()
        except B.LqsgdError as e:
            assert e.code == B.EHIP and "wait expired" in str(e)
            raised = True
            break
    assert raised
    with pytest.raises(B.LqsgdError):
        bad.get_factor(B.FACTOR_P_ORTH, 0, 0)
    bad.close()


BF16_CASES = [
    # layers, vectors, rank, bits, W, flags
    ([(256, 128)], (), 2, 8, 2, 0),
    ([(64, 576), (128, 64), (64, 27), (33, 65)], (40,), 4, 8, 4, 0),          # aligned and unaligned rows
    ([(300, 260)], (), 7, 4, 3, B.FLAG_EAGER_RESIDUAL),
    ([(129, 1028), (70, 27)], (9,), 16, 8, 2, 0),                             # matrix-core sweep 0
    ([(200, 1100), (96, 520)], (), 32, 8, 2, 0),
    ([(100, 1100), (129, 131)], (), 50, 8, 2, B.FLAG_AGGREGATE_FIRST),        # rank pad 64 and its plain fallback
]


@pytest.mark.parametrize("layers,vectors,rank,bits,W,flags", BF16_CASES)
def test_bf16_gradients(layers, vectors, rank, bits, W, flags):
    """Gradients handed over in bfloat16: the HIP path widens each value exactly,
    so every stage must agree with the oracle fed the widened values (G' = G + E
    bit-exact), over three steps with the error feedback carried."""
    import torch
    _say("case: bf16 gradients", layers, vectors, rank, bits, W, flags)
    rng = np.random.default_rng(rank * 7 + W)
    comp = B.Compressor(B.layer_list(layers, vectors), rank, bits, bits, W, 255.0, flags | B.FLAG_BF16_GRADIENTS)
    ml = list(range(len(layers)))
    Q = [rng.standard_normal((c, min(rank, r, c))).astype(f32) for r, c in layers]
    E = [[np.zeros(s, f32) for s in layers] for _ in range(W)]
    for l in ml:
        comp.set_q(l, Q[l])
    rep = pu.StageReport()
    shapes = list(layers) + [(v,) for v in vectors]
    for t in range(3):
        raw = [[torch.from_numpy((rng.standard_normal(s) * 1e-3).astype(f32)) for s in shapes] for _ in range(W)]
        Gd = [[x.to(torch.bfloat16).cuda() for x in row] for row in raw]          # what the library is given
        Gh = [[x.float().cpu().numpy() for x in row] for row in Gd]               # the same values, widened
        assert any(not np.array_equal(Gh[0][i], raw[0][i].numpy()) for i in range(len(shapes)))
        if t < 2:
            E, Q = pu.staged_iteration(comp, Gh, Gd, E, Q, ml, rep, aggregate_first=bool(flags & B.FLAG_AGGREGATE_FIRST))
        else:
            # fused step with G-hat and the 1-D means; compared with the oracle on the device's own state
            ghat = [torch.zeros(s, device="cuda") for s in shapes]
            comp.step(Gd, ghat)
            step = orc.layer_step_aggregate_first if flags & B.FLAG_AGGREGATE_FIRST else orc.layer_step
            for l in ml:
                want = step([Gh[w][l] for w in range(W)], [E[w][l] for w in range(W)], Q[l], rank, bits, bits, 255.0)
                got = ghat[l].cpu().numpy()
                assert pu.rel_fro(got, want["G_hat"]) <= 5e-2 if bits else pu.rel_fro(got, want["G_hat"]) <= pu.FP_TOL
                m0, _ = comp.get_state(l, 0, want_q=False)
                pb, qb = comp.get_factor(B.FACTOR_P_BAR, l), comp.get_factor(B.FACTOR_Q_BAR, l)
                mine = (Gh[0][l].astype(f64) + E[0][l].astype(f64)).astype(f32).astype(f64) - pb.astype(f64) @ qb.astype(f64).T
                assert pu.rel_fro(m0, mine) <= pu.FP_TOL
            for vi, v in enumerate(vectors):
                i = len(layers) + vi
                want = orc.vector_mean([Gh[w][i] for w in range(W)])
                assert np.allclose(ghat[i].cpu().numpy(), want, rtol=1e-6, atol=1e-9)
    comp.close()
    _say("  ", rep)


@pytest.mark.parametrize("layers,rank,W", [
    ([(32, 25), (64, 800), (1024, 3136), (10, 1024)], 4, 4),        # the small-CNN set: launch-bound
    ([(2304, 96), (129, 1028)], 16, 2),                             # tall factor: Gram-Schmidt must not take its one-launch form
    ([(129, 1028), (10, 512)], 16, 2),                              # a clipped rank: the padded operand copies are refreshed in every replay
])
def test_step_recorded_into_a_graph(layers, rank, W):
    """lqsgd_step recorded into a HIP graph on the context's stream: every replay,
    with fresh gradient values in the recorded buffers and eager work and
    synchronisation in between, gives bit for bit what an eager context gives."""
    import torch
    _say("case: step in a HIP graph", layers, rank, W)
    vectors = (32, 10)
    rng = np.random.default_rng(23)
    ll = B.layer_list(layers, vectors)
    shapes = list(layers) + [(v,) for v in vectors]
    q0 = [rng.standard_normal((c, min(rank, r, c))).astype(f32) for r, c in layers]

    def fresh():
        return [[torch.from_numpy((rng.standard_normal(s) * 1e-3).astype(f32)).cuda() for s in shapes] for _ in range(W)]

    s = torch.cuda.Stream()
    rec = B.Compressor(ll, rank, 8, 8, W, 255.0, 0, stream=s.cuda_stream)
    ref = B.Compressor(ll, rank, 8, 8, W, 255.0, 0)
    for l in range(len(layers)):
        rec.set_q(l, q0[l]); ref.set_q(l, q0[l])
    buf = fresh()                                   # the buffers the graph will read
    out_rec = [torch.zeros(sh, device="cuda") for sh in shapes]
    out_ref = [torch.zeros(sh, device="cuda") for sh in shapes]
    torch.cuda.synchronize()
    # two ordinary iterations: pointer lists bound, deferred residual in its steady state
    for _ in range(2):
        vals = fresh()
        torch.cuda.synchronize()
        for w in range(W):
            for i in range(len(shapes)):
                buf[w][i].copy_(vals[w][i])
        torch.cuda.synchronize()
        rec.step(buf, out_rec); ref.step(buf, out_ref)
        rec.synchronize(); ref.synchronize()
    tab = rec.pointer_table(buf)
    import ctypes as C
    gt = (C.c_void_p * len(shapes))()
    for i, t in enumerate(out_rec):
        gt[i] = t.data_ptr()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        rec.step_raw(tab, gt)
    torch.cuda.synchronize()
    # the recording itself ran nothing: bring the reference to the same point by replaying once first
    for rep_i in range(4):
        vals = fresh()
        torch.cuda.synchronize()
        for w in range(W):
            for i in range(len(shapes)):
                buf[w][i].copy_(vals[w][i])
        scratch = torch.randn(1 << 16, device="cuda").sum()          # unrelated eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        ref.step(buf, out_ref)
        torch.cuda.synchronize()
        for i in range(len(shapes)):
            assert torch.equal(out_rec[i], out_ref[i]), "replay %d tensor %d" % (rep_i, i)
        del scratch
    # the context's host-side bookkeeping did not see the replays; its device state did: compare it
    for l in range(len(layers)):
        for w in range(W):
            ea, qa = rec.get_state(l, w)
            eb, qb = ref.get_state(l, w)
            assert np.array_equal(qa, qb) and np.array_equal(ea, eb)
    rec.close(); ref.close()


def test_packets_move_between_contexts_on_the_device():
    """lqsgd_packet_device: the packets one context compressed are copied, device to device, into
    the slots of a second context, whose decompress then gives the first one's aggregate bit for bit
    (what a collective between GPUs would do with the same pointers)."""
    import ctypes as C
    import torch
    _say("case: packets handed over through device pointers")
    hip = C.CDLL("libamdhip64.so")
    hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
    layers, rank, bp, bq, W = [(300, 260), (64, 27)], 4, 8, 5, 3
    rng = np.random.default_rng(31)
    q0 = [rng.standard_normal((c, min(rank, r, c))).astype(f32) for r, c in layers]
    G = [[torch.from_numpy((rng.standard_normal(s) * 1e-3).astype(f32)).cuda() for s in layers] for _ in range(W)]
    Z = [[torch.zeros(s, device="cuda") for s in layers] for _ in range(W)]
    ll = B.layer_list(layers, ())
    src = B.Compressor(ll, rank, bp, bq, W, 255.0, 0)
    dst = B.Compressor(ll, rank, bp, bq, W, 255.0, 0)
    for l in range(len(layers)):
        src.set_q(l, q0[l]); dst.set_q(l, q0[l])
    src.compress(B.PHASE_P, G)
    dst.compress(B.PHASE_P, Z)          # brings dst to the same phase; its own packets are all zero
    src.synchronize(); dst.synchronize()
    for l in range(len(layers)):
        for w in range(W):
            mp, ml, sp, sl, cp = src.packet_device(B.PHASE_P, l, w)
            mp2, ml2, sp2, sl2, cp2 = dst.packet_device(B.PHASE_P, l, w)
            assert (ml, sl) == (ml2, sl2) and ml == bp * sl
            raw_m, raw_s = src.get_packet_raw(B.PHASE_P, l, w)
            t = torch.empty(ml, dtype=torch.uint8, device="cuda")
            assert hip.hipMemcpy(t.data_ptr(), mp, ml, 3) == 0        # 3 = device to device
            assert np.array_equal(t.cpu().numpy(), raw_m)
            for a, b, n in ((mp2, mp, ml), (sp2, sp, sl), (cp2, cp, 4)):
                assert hip.hipMemcpy(a, b, n, 3) == 0
    torch.cuda.synchronize()
    src.decompress(B.PHASE_P); dst.decompress(B.PHASE_P)
    for l in range(len(layers)):
        assert np.array_equal(src.get_factor(B.FACTOR_P_BAR, l), dst.get_factor(B.FACTOR_P_BAR, l))
    off = B.Compressor(ll, rank, 0, 0, W, 255.0, 0)
    with pytest.raises(B.LqsgdError):
        off.packet_device(B.PHASE_P, 0, 0)      # quantisation off: there is no packet
    src.close(); dst.close(); off.close()
