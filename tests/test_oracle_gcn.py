"""Pins for the oracle's GCN-style layers (Eq. 1 as printed: the aggregate runs over N_in(v) U {v};
Eq. 2 with one weight matrix): closed form on the raw edge list, dense matrices with PyTorch-CPU
autograd (independent code), the transpose identity and finite differences."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import oracle as ora


def _problem(V=150, E=1200, F=7, dims=(7, 6, 5, 4), fanouts=(3, 3, 2), B=9, seed=3):
    src, dst = si.rmat_edges(V, E, seed=seed)
    g = ora.build_csr(src, dst, V)
    feat = si.features(V, F, seed)
    lab = si.labels(V, dims[-1], seed)
    train = si.train_split(V, 0.65, seed)
    weights = [(np.asarray(w[0], np.float64), np.asarray(w[2], np.float64)) for w in si.init_weights(list(dims), seed)]
    return src, dst, g, feat, lab, train, weights, fanouts, B


def _dense_self_mean_matrix(blk):
    """Row v: 1/(len+1) on column v and on every sampled source (with multiplicity)."""
    a = np.zeros((blk.n_dst, blk.n_src))
    for v in range(blk.n_dst):
        a[v, v] += 1.0
        for e in range(blk.indptr[v], blk.indptr[v + 1]):
            a[v, blk.indices[e]] += 1.0
    return a / a.sum(axis=1, keepdims=True)


def test_full_neighbourhood_aggregate_is_normalised_adjacency_plus_identity():
    """Fanout >= max degree on all vertices: a = (D + I)^-1 (A + I) X on the raw edge list."""
    V = 90
    src, dst = si.random_graph_small(V, 500, seed=2)
    g = ora.build_csr(src, dst, V)
    x = si.features(V, 5, 2).astype(np.float64)
    kmax = int(np.diff(g.rowptr).max())
    all_v = np.arange(V, dtype=np.int32)
    blk = ora.sample_blocks(g, all_v, [kmax], 0, 0).blocks[0]
    a = np.zeros((V, V))
    np.add.at(a, (dst, src), 1.0)
    a += np.eye(V)
    expect = (a / a.sum(1, keepdims=True)) @ x
    got = ora.gcn_aggregate(x, blk.indptr, blk.indices, V)
    assert np.allclose(got, expect, rtol=1e-13, atol=1e-13)
    iso = np.diff(g.rowptr) == 0
    assert iso.any() and np.array_equal(got[iso], x[iso])          # no in-neighbours: the vertex itself


def test_adjoint_is_transpose():
    *_, g, feat, lab, train, weights, fanouts, B = _problem()
    blk = ora.sample_blocks(g, train[:B], [3, 3], 0, 0).blocks[1]
    a = _dense_self_mean_matrix(blk)
    x = np.random.default_rng(1).standard_normal((blk.n_src, 4))
    ga = np.random.default_rng(0).standard_normal((blk.n_dst, 4))
    assert np.allclose(ora.gcn_aggregate(x, blk.indptr, blk.indices, blk.n_dst), a @ x, rtol=1e-13, atol=1e-13)
    assert np.allclose(ora.gcn_aggregate_adjoint(ga, blk.indptr, blk.indices, blk.n_dst, blk.n_src), a.T @ ga,
                       rtol=1e-13, atol=1e-13)


def _torch_step(sb, x0, weights, labels_of_seeds, cache_emb_rows=None):
    L = len(sb.blocks)
    ws = [tuple(torch.tensor(np.asarray(t, np.float64), requires_grad=True) for t in w) for w in weights]
    x = torch.tensor(x0.astype(np.float64))
    hs = []
    for l in range(1, L + 1):
        blk = sb.blocks[L - l]
        a = torch.tensor(_dense_self_mean_matrix(blk))
        z = (a @ x) @ ws[l - 1][0] + ws[l - 1][1]
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
    *_, g, feat, lab, train, weights, fanouts, B = _problem()
    dims = [7, 6, 5, 4]
    dims = [dims[0]] + dims[1:n_layers] + [dims[-1]]
    weights = [(np.asarray(w[0], np.float64), np.asarray(w[2], np.float64)) for w in si.init_weights(dims, 5)]
    fan = fanouts[:n_layers]
    seeds = train[:B]
    res = ora.train_step(g, feat, lab, seeds, fan, weights, lr=0.05, seed=1, step=2, arch="gcn")
    loss, grads, hs = _torch_step(res.batch, res.x0, weights, lab[seeds])
    assert abs(res.loss - loss) < 1e-12
    for l in range(n_layers):
        assert np.allclose(res.h[l], hs[l], atol=1e-12)
        assert len(res.grads[l]) == 2
        for a, b in zip(res.grads[l], grads[l]):
            assert np.allclose(a, b, rtol=1e-10, atol=1e-13)
        for k in range(2):      # SGD closed form
            assert np.allclose(res.new_weights[l][k], weights[l][k] - 0.05 * grads[l][k], rtol=1e-12, atol=1e-15)


def test_step_with_cache_against_torch_autograd():
    *_, g, feat, lab, train, weights, fanouts, B = _problem(V=150, E=2500)
    cache = ora.select_hot(g, train, B, fanouts, 2, 0.3, 5, 6, 0)
    rng = np.random.default_rng(4)
    cache.emb[:] = rng.standard_normal(cache.emb.shape)
    cache.version[::2] = 1
    seeds = train[:B]
    before = cache.copy()
    res = ora.train_step(g, feat, lab, seeds, fanouts, weights, lr=0.01, seed=1, step=3, cache=cache, arch="gcn")
    assert res.n_hit > 0 and len(res.batch.compute_pos) > 0
    loss, grads, hs = _torch_step(res.batch, res.x0, weights, lab[seeds], before.emb[res.batch.hit_slot])
    assert abs(res.loss - loss) < 1e-12
    for l in range(3):
        for a, b in zip(res.grads[l], grads[l]):
            assert np.allclose(a, b, rtol=1e-10, atol=1e-13)


def test_weight_gradient_by_finite_differences():
    *_, g, feat, lab, train, weights, fanouts, B = _problem()
    seeds = train[:B]
    res = ora.train_step(g, feat, lab, seeds, fanouts, weights, lr=0.0, seed=1, step=0, arch="gcn")
    eps = 1e-6
    rng = np.random.default_rng(0)
    for l in (0, 2):
        for _ in range(3):
            i, j = rng.integers(0, weights[l][0].shape[0]), rng.integers(0, weights[l][0].shape[1])
            wp = [tuple(t.copy() for t in w) for w in weights]
            wm = [tuple(t.copy() for t in w) for w in weights]
            wp[l][0][i, j] += eps
            wm[l][0][i, j] -= eps
            lp = ora.train_step(g, feat, lab, seeds, fanouts, wp, 0.0, 1, 0, arch="gcn").loss
            lm = ora.train_step(g, feat, lab, seeds, fanouts, wm, 0.0, 1, 0, arch="gcn").loss
            assert abs((lp - lm) / (2 * eps) - res.grads[l][0][i, j]) < 1e-7


def test_bulk_refresh_of_gcn_rows_is_the_exact_embedding():
    """Full neighbourhood: refreshed row = relu(W^T (x_v + sum_{u in N_in(v)} x_u) / (deg + 1) + b), loops."""
    src, dst, g, feat, lab, train, weights, fanouts, B = _problem(V=140, E=900, dims=(7, 5, 4), fanouts=(3, 2))
    kmax = int(np.diff(g.rowptr).max())
    cache = ora.select_hot(g, train, B, (kmax, kmax), 1, 0.25, 3, 5, 0)
    emb, ver = ora.refresh_hot(g, feat, cache, weights[0], kmax, 2, 11)
    x = feat.astype(np.float64)
    for i, v in enumerate(cache.hot_ids):
        nb = [int(s) for s, d in zip(src, dst) if d == v]
        a = (x[v] + sum((x[u] for u in nb), np.zeros(x.shape[1]))) / (len(nb) + 1)
        assert np.allclose(emb[i], np.maximum(a @ weights[0][0] + weights[0][1], 0.0), rtol=1e-12, atol=1e-12)
    assert (ver == 2).all()


# ------------------------------------------------------------------ sum and symmetric normalisation
# (Eq. 1 lists sum among the AGGREGATE functions; Table 1 names A^, the adjacency matrix after symmetric
# normalisation. For a sampled block the reading is A^ = D_r^-1/2 (A_i + I) D_c^-1/2 with the row and column sums of
# the block's own adjacency with self loops.)

def _dense_block_with_self_loops(blk):
    a = np.zeros((blk.n_dst, blk.n_src))
    for v in range(blk.n_dst):
        a[v, v] += 1.0
        for e in range(blk.indptr[v], blk.indptr[v + 1]):
            a[v, blk.indices[e]] += 1.0
    return a


def _dense_normalised(blk, norm):
    a = _dense_block_with_self_loops(blk)
    if norm == "sum":
        return a
    if norm == "mean":
        return a / a.sum(axis=1, keepdims=True)
    col = a.sum(axis=0)
    return a / np.sqrt(a.sum(axis=1, keepdims=True)) / np.sqrt(np.where(col > 0, col, 1.0))[None, :]


@pytest.mark.parametrize("norm", ["sum", "sym", "mean"])
def test_aggregate_and_adjoint_are_the_dense_normalised_products(norm):
    *_, g, feat, lab, train, weights, fanouts, B = _problem()
    blk = ora.sample_blocks(g, train[:B], [3, 3], 0, 0).blocks[1]
    assert blk.n_src > blk.n_dst and (np.bincount(blk.indices, minlength=blk.n_src) > 1).any()
    a = _dense_normalised(blk, norm)
    x = np.random.default_rng(1).standard_normal((blk.n_src, 4))
    ga = np.random.default_rng(0).standard_normal((blk.n_dst, 4))
    assert np.allclose(ora.gcn_aggregate(x, blk.indptr, blk.indices, blk.n_dst, norm), a @ x, rtol=1e-13, atol=1e-13)
    assert np.allclose(ora.gcn_aggregate_adjoint(ga, blk.indptr, blk.indices, blk.n_dst, blk.n_src, norm), a.T @ ga,
                       rtol=1e-13, atol=1e-13)


def test_symmetric_normalisation_on_a_full_undirected_graph_is_the_textbook_gcn_matrix():
    """Every vertex a destination, every neighbour taken, edges in both directions and no multi-edges: the block is
    the whole graph and the aggregate is D~^-1/2 (A + I) D~^-1/2 X with D~ = D + I, the propagation rule of GCN;
    the sum form is (A + I) X."""
    V = 60
    rng = np.random.default_rng(5)
    pairs = {(int(a), int(b)) for a, b in rng.integers(0, V, (200, 2)) if a != b}
    pairs |= {(b, a) for a, b in pairs}
    src = np.array([p[0] for p in pairs], np.int32)
    dst = np.array([p[1] for p in pairs], np.int32)
    g = ora.build_csr(src, dst, V)
    kmax = int(np.diff(g.rowptr).max())
    all_v = np.arange(V, dtype=np.int32)
    blk = ora.sample_blocks(g, all_v, [kmax], 0, 0).blocks[0]
    x = si.features(V, 5, 2).astype(np.float64)
    a = np.zeros((V, V))
    a[dst, src] = 1.0
    a_tilde = a + np.eye(V)
    d = a_tilde.sum(1)
    assert np.array_equal(d, a_tilde.sum(0))
    expect = (a_tilde / np.sqrt(d)[:, None] / np.sqrt(d)[None, :]) @ x
    assert np.allclose(ora.gcn_aggregate(x, blk.indptr, blk.indices, V, "sym"), expect, rtol=1e-13, atol=1e-13)
    assert np.allclose(ora.gcn_aggregate(x, blk.indptr, blk.indices, V, "sum"), a_tilde @ x, rtol=1e-13, atol=1e-13)


def _torch_step_norm(sb, x0, weights, labels_of_seeds, norm, cache_emb_rows=None):
    L = len(sb.blocks)
    ws = [tuple(torch.tensor(np.asarray(t, np.float64), requires_grad=True) for t in w) for w in weights]
    x = torch.tensor(x0.astype(np.float64))
    for l in range(1, L + 1):
        blk = sb.blocks[L - l]
        z = (torch.tensor(_dense_normalised(blk, norm)) @ x) @ ws[l - 1][0] + ws[l - 1][1]
        h = torch.relu(z) if l < L else z
        if l == 1 and cache_emb_rows is not None:
            n_v1 = len(sb.compute_pos) + len(sb.hit_pos)
            full = torch.zeros((n_v1, h.shape[1]), dtype=torch.float64)
            full = full.index_put((torch.tensor(sb.compute_pos.astype(np.int64)),), h)
            full = full.index_put((torch.tensor(sb.hit_pos.astype(np.int64)),), torch.tensor(cache_emb_rows))
            h = full
        x = h
    loss = torch.nn.functional.cross_entropy(x, torch.tensor(labels_of_seeds.astype(np.int64)))
    loss.backward()
    return loss.item(), [tuple(t.grad.numpy() for t in w) for w in ws]


@pytest.mark.parametrize("arch,norm", [("gcn_sum", "sum"), ("gcn_sym", "sym")])
def test_sum_and_sym_steps_against_torch_autograd(arch, norm):
    *_, g, feat, lab, train, weights, fanouts, B = _problem(V=150, E=2500)
    seeds = train[:B]
    res = ora.train_step(g, feat, lab, seeds, fanouts, weights, lr=0.05, seed=1, step=2, arch=arch)
    loss, grads = _torch_step_norm(res.batch, res.x0, weights, lab[seeds], norm)
    assert abs(res.loss - loss) < 1e-11
    for l in range(3):
        for a, b in zip(res.grads[l], grads[l]):
            assert np.allclose(a, b, rtol=1e-10, atol=1e-12)
    # with reuse: cached rows enter layer 2 as constants
    cache = ora.select_hot(g, train, B, fanouts, 2, 0.3, 5, 6, 0)
    cache.emb[:] = np.random.default_rng(4).standard_normal(cache.emb.shape)
    cache.version[::2] = 1
    before = cache.copy()
    res = ora.train_step(g, feat, lab, seeds, fanouts, weights, lr=0.01, seed=1, step=3, cache=cache, arch=arch)
    assert res.n_hit > 0
    loss, grads = _torch_step_norm(res.batch, res.x0, weights, lab[seeds], norm, before.emb[res.batch.hit_slot])
    assert abs(res.loss - loss) < 1e-11
    for l in range(3):
        for a, b in zip(res.grads[l], grads[l]):
            assert np.allclose(a, b, rtol=1e-10, atol=1e-12)


def test_bulk_refresh_of_sum_and_sym_rows():
    """Full neighbourhood: a refreshed sum row is relu(W^T (x_v + sum of in-neighbours) + b); the sym row weighs
    every term by the block's own degrees (one-hop block over the hot vertices)."""
    src, dst, g, feat, lab, train, weights, fanouts, B = _problem(V=140, E=900, dims=(7, 5, 4), fanouts=(3, 2))
    kmax = int(np.diff(g.rowptr).max())
    cache = ora.select_hot(g, train, B, (kmax, kmax), 1, 0.25, 3, 5, 0)
    x = feat.astype(np.float64)
    emb, _ = ora.refresh_hot(g, feat, cache, weights[0], kmax, 2, 11, norm="sum")
    for i, v in enumerate(cache.hot_ids):
        nbrs = [int(s) for s, d in zip(src, dst) if d == v]
        a = x[v] + sum((x[u] for u in nbrs), np.zeros(x.shape[1]))
        assert np.allclose(emb[i], np.maximum(a @ weights[0][0] + weights[0][1], 0.0), rtol=1e-12, atol=1e-12)
    emb, _ = ora.refresh_hot(g, feat, cache, weights[0], kmax, 2, 11, norm="sym")
    blk = ora.sample_hop(g, cache.hot_ids, kmax, 2 + 11, ora.DOMAIN_REFRESH, 0)
    a = _dense_normalised(blk, "sym") @ x[blk.src_global]
    assert np.allclose(emb, np.maximum(a @ weights[0][0] + weights[0][1], 0.0), rtol=1e-12, atol=1e-12)
