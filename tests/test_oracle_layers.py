"""Pins for the floating-point half of the CPU oracle: gather, mean aggregation, layer
forward/backward, loss, the whole step, and the cache semantics. Checked against dense
linear algebra, PyTorch-CPU autograd (a library, independent code), finite differences and
the special cases the method fixes (S = 0, frozen weights)."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import oracle as ora


def _small_problem(V=150, E=1200, F=7, dims=(7, 6, 5, 4), fanouts=(3, 3, 2), B=9, seed=3):
    src, dst = si.rmat_edges(V, E, seed=seed)
    g = ora.build_csr(src, dst, V)
    feat = si.features(V, F, seed)
    lab = si.labels(V, dims[-1], seed)
    train = si.train_split(V, 0.65, seed)
    weights = si.init_weights(list(dims), seed)
    return src, dst, g, feat, lab, train, weights, fanouts, B


def _dense_mean_matrix(blk):
    a = np.zeros((blk.n_dst, blk.n_src))
    for v in range(blk.n_dst):
        for e in range(blk.indptr[v], blk.indptr[v + 1]):
            a[v, blk.indices[e]] += 1.0
    deg = a.sum(axis=1, keepdims=True)
    return np.divide(a, deg, out=np.zeros_like(a), where=deg > 0)


def test_gather_is_row_copy():
    t = si.features(500, 13, 1)
    ids = np.array([4, 4, 499, 0, 17], dtype=np.int32)
    assert np.array_equal(ora.gather_features(t, ids), t[ids])
    tb = si.features(500, 6, 1, "bf16")
    assert np.array_equal(ora.gather_features(tb, ids), tb[ids])
    assert ora.gather_features(t, np.zeros(0, np.int32)).shape == (0, 13)


def test_mean_over_all_neighbours_is_normalised_adjacency_product():
    """With fanout >= max degree the mean aggregate is D^-1 A X on the raw edge list (Eq. 1)."""
    V = 90
    src, dst = si.random_graph_small(V, 500, seed=2)
    g = ora.build_csr(src, dst, V)
    x = si.features(V, 5, 2).astype(np.float64)
    kmax = int(np.diff(g.rowptr).max())
    all_v = np.arange(V, dtype=np.int32)
    blk = ora.sample_blocks(g, all_v, [kmax], 0, 0).blocks[0]
    assert np.array_equal(blk.src_global, all_v)       # every vertex is a destination already
    a = np.zeros((V, V))
    np.add.at(a, (dst, src), 1.0)
    deg = a.sum(1, keepdims=True)
    expect = np.divide(a, deg, out=np.zeros_like(a), where=deg > 0) @ x
    got = ora.mean_aggregate(x, blk.indptr, blk.indices, V)
    assert np.allclose(got, expect, rtol=1e-13, atol=1e-13)
    assert (got[deg[:, 0] == 0] == 0).all()


def test_adjoint_is_transpose_of_mean():
    *_, g, feat, lab, train, weights, fanouts, B = _small_problem()
    blk = ora.sample_blocks(g, train[:B], [3, 3], 0, 0).blocks[1]
    a = _dense_mean_matrix(blk)
    gm = np.random.default_rng(0).standard_normal((blk.n_dst, 4))
    assert np.allclose(ora.mean_aggregate_adjoint(gm, blk.indptr, blk.indices, blk.n_dst, blk.n_src), a.T @ gm,
                       rtol=1e-13, atol=1e-13)


def test_softmax_xent_against_torch():
    rng = np.random.default_rng(0)
    z = rng.standard_normal((11, 6)) * 4
    y = rng.integers(0, 6, 11)
    loss, g = ora.softmax_xent(z, y)
    zt = torch.tensor(z, requires_grad=True)
    lt = torch.nn.functional.cross_entropy(zt, torch.tensor(y))
    lt.backward()
    assert abs(loss - lt.item()) < 1e-12
    assert np.allclose(g, zt.grad.numpy(), atol=1e-14)
    # large logits do not overflow
    loss2, _ = ora.softmax_xent(z + 1e4, y)
    assert abs(loss2 - loss) < 1e-9


def _torch_step(sb, x0, weights, labels_of_seeds, cache_emb_rows=None):
    """The same step written as dense matrices with autograd doing the backward."""
    L = len(sb.blocks)
    ws = [tuple(torch.tensor(np.asarray(t, np.float64), requires_grad=True) for t in w) for w in weights]
    x = torch.tensor(x0.astype(np.float64))
    hs = []
    for l in range(1, L + 1):
        blk = sb.blocks[L - l]
        a = torch.tensor(_dense_mean_matrix(blk))
        z = x[: blk.n_dst] @ ws[l - 1][0] + (a @ x) @ ws[l - 1][1] + ws[l - 1][2]
        h = torch.relu(z) if l < L else z
        if l == 1 and cache_emb_rows is not None:
            n_v1 = len(sb.compute_pos) + len(sb.hit_pos)
            full = torch.zeros((n_v1, h.shape[1]), dtype=torch.float64)
            full = full.index_put((torch.tensor(sb.compute_pos.astype(np.int64)),), h)
            full = full.index_put((torch.tensor(sb.hit_pos.astype(np.int64)),), torch.tensor(cache_emb_rows))
            h = full
        hs.append(h)
        x = h
    loss = torch.nn.functional.cross_entropy(x, torch.tensor(labels_of_seeds.astype(np.int64)))
    loss.backward()
    return loss.item(), [tuple(t.grad.numpy() for t in w) for w in ws], [h.detach().numpy() for h in hs]


@pytest.mark.parametrize("n_layers", [1, 2, 3])
def test_step_against_torch_autograd(n_layers):
    *_, g, feat, lab, train, weights, fanouts, B = _small_problem()
    dims = [7, 6, 5, 4]
    dims = [dims[0]] + dims[1:n_layers] + [dims[-1]]
    weights = si.init_weights(dims, 5)
    fan = fanouts[:n_layers]
    seeds = train[:B]
    res = ora.train_step(g, feat, lab, seeds, fan, weights, lr=0.05, seed=1, step=2)
    loss, grads, hs = _torch_step(res.batch, res.x0, weights, lab[seeds])
    assert abs(res.loss - loss) < 1e-12
    for l in range(n_layers):
        assert np.allclose(res.h[l], hs[l], atol=1e-12)
        for a, b in zip(res.grads[l], grads[l]):
            assert np.allclose(a, b, rtol=1e-10, atol=1e-13)
        for k in range(3):      # SGD closed form
            assert np.allclose(res.new_weights[l][k], np.asarray(weights[l][k], np.float64) - 0.05 * grads[l][k],
                               rtol=1e-12, atol=1e-15)


def test_step_with_cache_against_torch_autograd():
    """Reused rows enter layer 2 as constants: no gradient reaches layer 1 through them."""
    *_, g, feat, lab, train, weights, fanouts, B = _small_problem(V=150, E=2500)
    cache = ora.select_hot(g, train, B, fanouts, 2, 0.3, 5, 6, 0)
    rng = np.random.default_rng(4)
    cache.emb[:] = rng.standard_normal(cache.emb.shape)
    cache.version[::2] = 1
    seeds = train[:B]
    before = cache.copy()
    res = ora.train_step(g, feat, lab, seeds, fanouts, weights, lr=0.01, seed=1, step=3, cache=cache)
    assert res.n_hit > 0 and len(res.batch.compute_pos) > 0
    loss, grads, hs = _torch_step(res.batch, res.x0, weights, lab[seeds], before.emb[res.batch.hit_slot])
    assert abs(res.loss - loss) < 1e-12
    for l in range(3):
        for a, b in zip(res.grads[l], grads[l]):
            assert np.allclose(a, b, rtol=1e-10, atol=1e-13)
    # refresh: every computed hot vertex now holds its fresh row with version = step
    v1c = res.batch.blocks[-1].dst_global
    slots = cache.slot_of_vertex[v1c]
    sel = slots >= 0
    assert sel.any()
    assert np.array_equal(cache.emb[slots[sel]], res.h[0][res.batch.compute_pos][sel])
    assert (cache.version[slots[sel]] == 3).all()
    untouched = np.setdiff1d(np.arange(cache.n_hot), slots[sel])
    assert np.array_equal(cache.emb[untouched], before.emb[untouched])
    assert np.array_equal(cache.version[untouched], before.version[untouched])


def test_loss_gradient_by_finite_differences():
    *_, g, feat, lab, train, weights, fanouts, B = _small_problem(F=4, dims=(4, 3, 3))
    fan = (3, 2)
    seeds = train[:6]
    w64 = [tuple(np.asarray(t, np.float64) for t in w) for w in weights]
    res = ora.train_step(g, feat, lab, seeds, fan, w64, 0.0, 9, 0)
    eps = 1e-6
    for l in range(2):
        for k in range(3):
            it = np.nditer(w64[l][k], flags=["multi_index"])
            for _ in it:
                idx = it.multi_index
                orig = w64[l][k][idx]
                w64[l][k][idx] = orig + eps
                lp = ora.train_step(g, feat, lab, seeds, fan, w64, 0.0, 9, 0).loss
                w64[l][k][idx] = orig - eps
                lm = ora.train_step(g, feat, lab, seeds, fan, w64, 0.0, 9, 0).loss
                w64[l][k][idx] = orig
                fd = (lp - lm) / (2 * eps)
                assert abs(fd - res.grads[l][k][idx]) < 1e-6 * max(1.0, abs(fd)), (l, k, idx)


def _run_steps(g, feat, lab, train, weights, fanouts, B, n, lr, cache):
    ws = [tuple(np.asarray(t, np.float64) for t in w) for w in weights]
    out = []
    for t in range(n):
        r = ora.train_step(g, feat, lab, si.batch_seeds(train, B, t), fanouts, ws, lr, 0, t, cache)
        ws = r.new_weights
        out.append(r)
    return out, ws


def test_staleness_zero_is_exact_training():
    """S = 0 means nothing may be reused: bit-identical to training with no cache."""
    *_, g, feat, lab, train, weights, fanouts, B = _small_problem(E=2500)
    cache = ora.select_hot(g, train, B, fanouts, 2, 0.3, 0, 6, 0)
    a, wa = _run_steps(g, feat, lab, train, weights, fanouts, B, 4, 0.05, cache)
    b, wb = _run_steps(g, feat, lab, train, weights, fanouts, B, 4, 0.05, None)
    for ra, rb in zip(a, b):
        assert ra.n_hit == 0 and ra.loss == rb.loss
        assert np.array_equal(ra.h[-1], rb.h[-1])
    for x, y in zip(wa, wb):
        for p, q in zip(x, y):
            assert np.array_equal(p, q)
    empty = ora.select_hot(g, train, B, fanouts, 1, 0.0, 3, 6, 0)
    c, _ = _run_steps(g, feat, lab, train, weights, fanouts, B, 2, 0.05, empty)
    assert c[0].loss == b[0].loss and c[1].loss == b[1].loss


def test_frozen_weights_make_reuse_exact_and_ages_bounded():
    """With lr = 0 and the full neighbourhood sampled, a reused row equals a freshly computed
    one, so any staleness bound gives the exact loss; every hit is at most S steps old."""
    *_, g, feat, lab, train, weights, fanouts, B = _small_problem(E=900)
    kmax = int(np.diff(g.rowptr).max())
    fan = (kmax, kmax, kmax)
    S = 2
    cache = ora.select_hot(g, train, B, fan, 1, 0.4, S, 6, 0)
    ws = [tuple(np.asarray(t, np.float64) for t in w) for w in weights]
    hits = 0
    for t in range(6):
        seeds = si.batch_seeds(train, B, t)
        ver_before = cache.version.copy()
        r = ora.train_step(g, feat, lab, seeds, fan, ws, 0.0, 0, t, cache)
        exact = ora.train_step(g, feat, lab, seeds, fan, ws, 0.0, 0, t, None)
        assert abs(r.loss - exact.loss) < 1e-12
        age = t - ver_before[r.batch.hit_slot]
        assert (age <= S).all() and (age >= 1).all() and (ver_before[r.batch.hit_slot] >= 0).all()
        hits += r.n_hit
    assert hits > 0


def test_stale_gap_shrinks_with_learning_rate():
    """Lemma 1's shape: the gap between a reused embedding and the exact one is bounded by the
    weight drift. With the full neighbourhood sampled (so only the weights differ) it is zero
    for frozen weights and shrinks with the learning rate."""
    *_, g, feat, lab, train, weights, _, B = _small_problem(E=900)
    kmax = int(np.diff(g.rowptr).max())
    fan = (kmax, kmax, kmax)

    def gap(lr):
        cache = ora.select_hot(g, train, B, fan, 2, 0.5, 3, 6, 0)
        runs, ws = _run_steps(g, feat, lab, train, weights, fan, B, 3, lr, cache)
        seeds = si.batch_seeds(train, B, 3)
        snap = cache.copy()
        r = ora.train_step(g, feat, lab, seeds, fan, ws, lr, 0, 3, cache)
        e = ora.train_step(g, feat, lab, seeds, fan, ws, lr, 0, 3, None)
        assert r.n_hit > 0
        fresh = e.h[0][r.batch.hit_pos]
        return np.abs(snap.emb[r.batch.hit_slot] - fresh).max()

    g1, g2, g3 = gap(0.1), gap(0.01), gap(0.0)
    assert g3 < 1e-12
    assert 0 < g2 < g1


def test_bf16_features_are_upcast_exactly():
    *_, g, feat, lab, train, weights, fanouts, B = _small_problem()
    fb = si.f32_to_bf16_bits(feat)
    r1 = ora.train_step(g, fb, lab, train[:B], fanouts, weights, 0.1, 0, 0, None, feat_is_bf16=True)
    r2 = ora.train_step(g, si.bf16_bits_to_f32(fb), lab, train[:B], fanouts, weights, 0.1, 0, 0)
    assert r1.loss == r2.loss
    assert r1.x0.dtype == np.uint16
