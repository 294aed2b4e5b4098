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
    r1 = ora.train_step(g, fb, lab, train[:B], fanouts, weights, 0.1, 0, 0, None, feat_is_bf16=True, bf16_products=False)
    r2 = ora.train_step(g, si.bf16_bits_to_f32(fb), lab, train[:B], fanouts, weights, 0.1, 0, 0)
    assert r1.loss == r2.loss
    assert r1.x0.dtype == np.uint16


# ------------------------------------------------------------------ the ReLU-decision hook of the backward pass
# (Eq. 2's activation inside the backward loop of Algorithm 1: the derivative of ReLU is a float deciding a bit.
# The GPU parity tests may hand the oracle the decisions taken in fp32 for pre-activations that are zero to within
# rounding; these pins fix what the hook does so that it cannot hide anything else.)

def test_relu_decision_hook_defaults_to_the_sign_of_the_pre_activation():
    *_, g, feat, lab, train, weights, fanouts, B = _small_problem()
    blk = ora.sample_blocks(g, train[:B], [3, 3], 0, 0).blocks[1]
    rng = np.random.default_rng(1)
    x = rng.standard_normal((blk.n_src, 7))
    (ws, wn, bias), = si.init_weights([7, 5], 2)
    mean, z, h = ora.sage_layer_fwd_z(blk, x, ws, wn, bias, relu=True)
    assert np.array_equal(h > 0, z > 0) and (z > 0).any() and (z < 0).any()
    gh = rng.standard_normal(h.shape)
    ref = ora.sage_layer_bwd(blk, x, mean, h, gh, ws, wn, True, True)
    same = ora.sage_layer_bwd(blk, x, mean, h, gh, ws, wn, True, True, active=(z > 0))
    for a, b in zip(ref, same):
        assert np.array_equal(a, b)
    # without an activation the hook is ignored
    lin = ora.sage_layer_bwd(blk, x, mean, z, gh, ws, wn, False, True)
    lin2 = ora.sage_layer_bwd(blk, x, mean, z, gh, ws, wn, False, True, active=np.zeros(z.shape, bool))
    for a, b in zip(lin, lin2):
        assert np.array_equal(a, b)
    # GCN-style layer: same contract
    a, zg, hg = ora.gcn_layer_fwd_z(blk, x, ws, bias, relu=True)
    refg = ora.gcn_layer_bwd(blk, a, hg, gh, ws, True, True)
    sameg = ora.gcn_layer_bwd(blk, a, hg, gh, ws, True, True, active=(zg > 0))
    for p, q in zip(refg, sameg):
        assert np.array_equal(p, q)


def test_flipping_one_relu_decision_moves_every_gradient_by_its_rank_one_term():
    """Decision (r, c) flipped from 'off' to 'on' adds grad_h[r, c] to gz[r, c] and nothing else, so
    gw_self += outer(x_dst[r], e_c) g, gw_neigh += outer(mean[r], e_c) g, gbias[c] += g, and the input gradient
    gains g * w_self[:, c] on row r plus g * w_neigh[:, c] / len(row r) on each sampled source of r."""
    *_, g, feat, lab, train, weights, fanouts, B = _small_problem()
    blk = ora.sample_blocks(g, train[:B], [3, 3], 0, 0).blocks[1]
    rng = np.random.default_rng(2)
    x = rng.standard_normal((blk.n_src, 7))
    (ws, wn, bias), = si.init_weights([7, 5], 3)
    ws, wn = ws.astype(np.float64), wn.astype(np.float64)
    mean, z, h = ora.sage_layer_fwd_z(blk, x, ws, wn, bias, relu=True)
    gh = rng.standard_normal(h.shape)
    off = np.argwhere(z < 0)
    rows_with_edges = np.flatnonzero(np.diff(blk.indptr) > 0)
    r, c = next((int(a), int(b)) for a, b in off if a in rows_with_edges)
    act = z > 0
    base = ora.sage_layer_bwd(blk, x, mean, h, gh, ws, wn, True, True, active=act)
    act2 = act.copy()
    act2[r, c] = True
    flip = ora.sage_layer_bwd(blk, x, mean, h, gh, ws, wn, True, True, active=act2)
    gval = gh[r, c]
    e_c = np.zeros(5)
    e_c[c] = 1.0
    assert np.allclose(flip[0] - base[0], gval * np.outer(x[r], e_c), rtol=1e-12, atol=1e-14)
    assert np.allclose(flip[1] - base[1], gval * np.outer(mean[r], e_c), rtol=1e-12, atol=1e-14)
    assert np.allclose(flip[2] - base[2], gval * e_c, rtol=1e-12, atol=1e-14)
    dgx = np.zeros_like(x)
    dgx[r] += gval * ws[:, c]
    seg = blk.indices[blk.indptr[r]:blk.indptr[r + 1]]
    for u in seg:
        dgx[u] += gval * wn[:, c] / len(seg)
    assert np.allclose(flip[3] - base[3], dgx, rtol=1e-12, atol=1e-14)
    assert np.abs(flip[0] - base[0]).max() > 0


@pytest.mark.parametrize("arch", ["sage", "gcn"])
def test_step_hook_is_consulted_for_hidden_layers_only_and_none_means_default(arch):
    *_, g, feat, lab, train, weights, fanouts, B = _small_problem(V=150, E=2500)
    ws = [((w[0], w[2]) if arch == "gcn" else w) for w in weights]
    cache = ora.select_hot(g, train, B, fanouts, 2, 0.3, 5, 6, 0)
    cache.emb[:] = np.random.default_rng(4).standard_normal(cache.emb.shape)
    cache.version[::2] = 1
    seeds = train[:B]
    ref = ora.train_step(g, feat, lab, seeds, fanouts, ws, 0.01, 1, 3, cache.copy(), arch=arch)
    seen = []

    def hook_none(layer, z):
        seen.append((layer, z.shape))
        return None

    r1 = ora.train_step(g, feat, lab, seeds, fanouts, ws, 0.01, 1, 3, cache.copy(), relu_decisions=hook_none, arch=arch)
    r2 = ora.train_step(g, feat, lab, seeds, fanouts, ws, 0.01, 1, 3, cache.copy(),
                        relu_decisions=lambda layer, z: z > 0, arch=arch)
    L = len(fanouts)
    assert [s[0] for s in seen] == list(range(L - 1, 0, -1))           # layers with a ReLU, top down; never layer L
    # layer 1's pre-activations cover the computed rows only (reused rows take no gradient)
    assert seen[-1][1][0] == len(ref.batch.compute_pos) and ref.n_hit > 0
    for r in (r1, r2):
        assert r.loss == ref.loss
        for ga, gb in zip(r.grads, ref.grads):
            for a, b in zip(ga, gb):
                assert np.array_equal(a, b)
    # a hook that switches everything off zeroes every gradient below the classifier layer
    r0 = ora.train_step(g, feat, lab, seeds, fanouts, ws, 0.01, 1, 3, cache.copy(),
                        relu_decisions=lambda layer, z: np.zeros(z.shape, bool), arch=arch)
    assert all(not np.any(a) for ga in r0.grads[:-1] for a in ga)
    assert any(np.any(a) for a in r0.grads[-1])


# ------------------------------------------------------------------ bf16 operands for a bf16 feature table

def test_round_to_bf16_matches_the_library_conversion_and_ties_go_to_even():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(5000) * 10.0 ** rng.integers(-20, 20, 5000), [0.0, -0.0, 1.0, -1.0]]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(ora.round_to_bf16(x).astype(np.float32), ref)
    # exactly half-way cases: 1 + 2^-8 lies between 1 and 1 + 2^-7 and goes to the even one (1.0); 1 + 3 * 2^-8 goes up
    assert ora.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert ora.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    # values that are bf16 already are unchanged
    b = si.bf16_bits_to_f32(si.f32_to_bf16_bits(x))
    assert np.array_equal(ora.round_to_bf16(b).astype(np.float32), b)


def test_bf16_products_stay_within_the_rounding_bound_of_the_exact_layer():
    """Rounding an operand to bf16 (8 significant bits, nearest) moves it by at most 2^-9 of its size. A product with
    one rounded operand (bf16 features x rounded weights) is off by at most 2^-9 of its size, with two rounded operands
    (mean x weights) by 2 * 2^-9 + 2^-18: elementwise bounds on the pre-activations and on the weight gradients."""
    *_, g, feat, lab, train, weights, fanouts, B = _small_problem(F=16, dims=(16, 12, 5), fanouts=(4, 3))
    fb = si.f32_to_bf16_bits(feat)
    x_tab = si.bf16_bits_to_f32(fb).astype(np.float64)
    blk = ora.sample_blocks(g, train[:40], [4, 3], 0, 0).blocks[1]
    x = x_tab[blk.src_global]
    (ws, wn, bias) = weights[0]
    u = 2.0 ** -9
    mean, z, h = ora.sage_layer_fwd_z(blk, x, ws, wn, bias, True)
    mean_b, z_b, h_b = ora.sage_layer_fwd_z(blk, x, ws, wn, bias, True, bf16_products=True)
    assert np.array_equal(mean, mean_b)
    bound = u * (np.abs(x[: blk.n_dst]) @ np.abs(ws)) + (2 * u + u * u) * (np.abs(mean) @ np.abs(wn))
    assert (np.abs(z_b - z) <= bound * (1 + 1e-6) + 1e-300).all() and np.abs(z_b - z).max() > 0
    gh = np.random.default_rng(1).standard_normal(h.shape)
    act = z > 0
    e = ora.sage_layer_bwd(blk, x, mean, h, gh, ws, wn, True, False, active=act)
    r = ora.sage_layer_bwd(blk, x, mean, h, gh, ws, wn, True, False, active=act, bf16_products=True)
    gz = gh * act
    assert (np.abs(r[0] - e[0]) <= u * (np.abs(x[: blk.n_dst]).T @ np.abs(gz)) * (1 + 1e-6)).all()
    assert (np.abs(r[1] - e[1]) <= (2 * u + u * u) * (np.abs(mean).T @ np.abs(gz)) * (1 + 1e-6)).all()
    assert np.array_equal(r[2], e[2])                          # the bias gradient is the plain column sum


def test_bf16_products_are_exact_when_every_operand_is_a_bf16_value():
    """Fanout 1 makes the mean a feature row (bf16); weights and output gradients picked from a bf16 grid: nothing is
    rounded, so the layer must equal the exact one bit for bit."""
    *_, g, feat, lab, train, weights, fanouts, B = _small_problem(F=16, dims=(16, 12, 5), fanouts=(4, 3))
    x_tab = si.bf16_bits_to_f32(si.f32_to_bf16_bits(feat)).astype(np.float64)
    blk = ora.sample_blocks(g, train[:40], [4, 1], 0, 0).blocks[1]
    x = x_tab[blk.src_global]
    rng = np.random.default_rng(3)
    ws, wn = rng.integers(-64, 64, (16, 12)) / 64.0, rng.integers(-64, 64, (16, 12)) / 128.0
    bias = rng.standard_normal(12)
    a = ora.sage_layer_fwd_z(blk, x, ws, wn, bias, True)
    b_ = ora.sage_layer_fwd_z(blk, x, ws, wn, bias, True, bf16_products=True)
    assert all(np.array_equal(p, q) for p, q in zip(a, b_))
    gh = rng.integers(-32, 32, a[2].shape) / 16.0
    e = ora.sage_layer_bwd(blk, x, a[0], a[2], gh, ws, wn, True, False)
    r = ora.sage_layer_bwd(blk, x, a[0], a[2], gh, ws, wn, True, False, bf16_products=True)
    assert all(np.array_equal(p, q) for p, q in zip(e[:3], r[:3]))


def test_step_with_a_bf16_table_uses_bf16_products_in_layer_1_only():
    *_, g, feat, lab, train, weights, fanouts, B = _small_problem()
    fb = si.f32_to_bf16_bits(feat)
    on = ora.train_step(g, fb, lab, train[:B], fanouts, weights, 0.1, 0, 0, None, feat_is_bf16=True)
    off = ora.train_step(g, fb, lab, train[:B], fanouts, weights, 0.1, 0, 0, None, feat_is_bf16=True, bf16_products=False)
    assert on.loss != off.loss and abs(on.loss - off.loss) < 2e-2 * abs(off.loss)
    # the same blocks and the same (unrounded) mean; layer 1's output differs, and with it everything above
    assert np.array_equal(on.mean[0], off.mean[0]) and not np.array_equal(on.h[0], off.h[0])
    # layers above the bottom one are computed in full precision from whatever layer 1 gave them
    blk = on.batch.blocks[-2]
    _, _, h2 = ora.sage_layer_fwd_z(blk, on.h[0], *weights[1], relu=True)
    assert np.array_equal(h2, on.h[1])
    # GCN-style layers keep exact products
    wg = [(w[0], w[2]) for w in weights]
    a = ora.train_step(g, fb, lab, train[:B], fanouts, wg, 0.1, 0, 0, None, feat_is_bf16=True, arch="gcn")
    b_ = ora.train_step(g, si.bf16_bits_to_f32(fb), lab, train[:B], fanouts, wg, 0.1, 0, 0, None, arch="gcn")
    assert a.loss == b_.loss
