"""GPU test of lqsgd_step_static, the entry point that allocates nothing: called through
the C ABI on caller-held state, its outputs must equal, bit for bit, those of lqsgd_step
on a context loaded with the same state -- on calls in a row that change the
configuration (a larger set, then a smaller one, then the smaller one again, so that
the shared scratch block is laid out anew, reused, and keeps the last call's contents)."""
import numpy as np
import pytest

from paper_2506_17974_amd import binding as B
from paper_2506_17974_amd import workloads as wl

pytestmark = pytest.mark.gpu
f32 = np.float32


def _round_up(x, m):
    return (x + m - 1) // m * m


def _layout(matrices, rank):
    e_off, q_off, ea, qa = [], [], 0, 0
    for rows, cols in matrices:
        e_off.append(ea)
        q_off.append(qa)
        ea += _round_up(rows * cols, 64)
        qa += _round_up(cols * min(rank, rows, cols), 64)
    return e_off, q_off


def _one_call(matrices, vectors, rank, bits, W, flags, rng, E, Q, tag):
    """One iteration both ways from the state (E[w][l], Q[l]); returns the new state as the
    static entry point left it."""
    import torch
    print("case: lqsgd_step_static", tag, matrices, vectors, "r=%d b=%d W=%d flags=%d" % (rank, bits, W, flags), flush=True)
    layers = B.layer_list(matrices, vectors)
    L, V = len(matrices), len(vectors)
    info = B.plan_query(layers, rank, bits, bits, W, 255.0, flags)
    e_off, q_off = _layout(matrices, rank)
    G = [[(rng.standard_normal(s) * 1e-3).astype(f32) for s in matrices] +
         [(rng.standard_normal(n) * 1e-3).astype(f32) for n in vectors] for _ in range(W)]
    Gd = [[torch.from_numpy(g).cuda() for g in row] for row in G]
    if flags & B.FLAG_BF16_GRADIENTS:
        Gd = [[t.to(torch.bfloat16) for t in row] for row in Gd]

    # reference: the existing entry point on a context that holds the same state
    ref = B.Compressor(layers, rank, bits, bits, W, 255.0, flags)
    for l in range(L):
        for k in range(W):
            ref.set_state(l, k, e=E[k][l], q=Q[l] if k == 0 else None)
    g_ref = [torch.full(s, 3.0, device="cuda") for s in matrices] + [torch.full((n,), 3.0, device="cuda") for n in vectors]
    ref.step(Gd, g_ref)
    ref.synchronize()

    # the static entry point on caller-held buffers (filled with a pattern where no tensor lies)
    res = np.full((W, info.residual_stride), 7.0, f32)
    wq = np.full(info.warm_q_floats, 7.0, f32)
    for l, (rows, cols) in enumerate(matrices):
        r = min(rank, rows, cols)
        for k in range(W):
            res[k, e_off[l]:e_off[l] + rows * cols] = E[k][l].ravel()
        wq[q_off[l]:q_off[l] + cols * r] = Q[l].ravel()
    res_d = torch.from_numpy(res).cuda() if L else None
    wq_d = torch.from_numpy(wq).cuda() if L else None
    g_st = [torch.full(s, 5.0, device="cuda") for s in matrices] + [torch.full((n,), 5.0, device="cuda") for n in vectors]
    B.step_static(layers, rank, bits, bits, W, 255.0, flags, Gd, res_d, wq_d, g_st)
    torch.cuda.synchronize()

    for i in range(L + V):
        assert torch.equal(g_ref[i], g_st[i]), "%s: output %d differs" % (tag, i)
    E_new = [[None] * L for _ in range(W)]
    Q_new = [None] * L
    if L:
        res_h, wq_h = res_d.cpu().numpy(), wq_d.cpu().numpy()
    for l, (rows, cols) in enumerate(matrices):
        r = min(rank, rows, cols)
        Q_new[l] = wq_h[q_off[l]:q_off[l] + cols * r].reshape(cols, r).copy()
        for k in range(W):
            e_ref, q_ref = ref.get_state(l, k)
            E_new[k][l] = res_h[k, e_off[l]:e_off[l] + rows * cols].reshape(rows, cols).copy()
            assert np.array_equal(E_new[k][l], e_ref), "%s: residual of layer %d, worker %d differs" % (tag, l, k)
            assert np.array_equal(Q_new[l], q_ref), "%s: warm-start Q of layer %d differs" % (tag, l)
            # nothing is written between the tensors of the caller's buffers
            end = e_off[l + 1] if l + 1 < L else info.residual_stride
            assert np.all(res_h[k, e_off[l] + rows * cols:end] == 7.0)
    ref.close()
    return E_new, Q_new


def _fresh_state(matrices, rank, W, rng):
    E = [[(rng.standard_normal(s) * 3e-4).astype(f32) for s in matrices] for _ in range(W)]
    Q = [rng.standard_normal((c, min(rank, r, c))).astype(f32) for r, c in matrices]
    return E, Q


def test_step_static_matches_step_on_calls_in_a_row():
    rng = np.random.default_rng(2506)
    cnn = wl.small_cnn()
    big, big_v = list(cnn.layers), list(cnn.vectors)
    small, small_v = [(256, 128)], []
    E, Q = _fresh_state(big, 4, 4, rng)
    _one_call(big, big_v, 4, 8, 4, 0, rng, E, Q, "first call, small CNN set")
    E, Q = _fresh_state(small, 2, 2, rng)
    E, Q = _one_call(small, small_v, 2, 8, 2, 0, rng, E, Q, "second call, a smaller set")
    E, Q = _one_call(small, small_v, 2, 8, 2, 0, rng, E, Q, "third call, same set, state carried on")
    # other paths through the same block: matrix-core sweeps with padded operand copies and a tall
    # factor (per-column Gram-Schmidt), then the aggregate-first order on bfloat16 gradients
    mixed = [(200, 1100), (10, 512), (64, 27), (2600, 36)]
    E, Q = _fresh_state(mixed, 32, 2, rng)
    E, Q = _one_call(mixed, [33], 32, 8, 2, 0, rng, E, Q, "rank 32")
    _one_call(mixed, [33], 32, 8, 2, 0, rng, E, Q, "rank 32 again")
    E, Q = _fresh_state(small, 2, 3, rng)
    _one_call(small, [5], 2, 4, 3, B.FLAG_AGGREGATE_FIRST | B.FLAG_BF16_GRADIENTS, rng, E, Q, "aggregate-first, bf16")


def test_step_static_rejects_what_does_not_fit():
    import torch
    w = wl.resnet18(rank=32)
    layers = B.layer_list(w.layers, w.vectors)
    info = B.plan_query(layers, w.rank, w.bits, w.bits, w.workers)
    assert info.device_bytes - 4 * w.workers * info.residual_stride > (32 << 20)
    dummy = torch.zeros(16, device="cuda")
    grads = [[dummy] * len(layers) for _ in range(w.workers)]
    with pytest.raises(B.LqsgdError) as ei:
        B.step_static(layers, w.rank, w.bits, w.bits, w.workers, 255.0, 0, grads, dummy, dummy, None)
    assert ei.value.code == B.EUNSUPPORTED and "scratch" in str(ei.value)
    with pytest.raises(B.LqsgdError) as ei:
        B.step_static(layers, 0, 8, 8, 2, 255.0, 0, grads, dummy, dummy, None)
    assert ei.value.code == B.EINVAL
    # and the block still serves a configuration that fits
    rng = np.random.default_rng(1)
    E, Q = _fresh_state([(64, 27)], 4, 2, rng)
    _one_call([(64, 27)], [], 4, 8, 2, 0, rng, E, Q, "after a rejected call")
