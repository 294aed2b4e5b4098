"""Pins for the oracle's bulk hot refresh and super-batch schedule (Section 4.2, Stage 2 and
"Bounded Staleness"): brute force over the raw adjacency, the version-gap figures the paper
states (largest gap 2n - 1, reached in the last batch of a super-batch), and the special
cases in which reuse must be exact."""
import numpy as np

import synth_inputs as si
from oracle import oracle as ora


def _problem(V=140, E=900, F=6, dims=(6, 5, 4), B=8, seed=5):
    src, dst = si.rmat_edges(V, E, seed=seed)
    g = ora.build_csr(src, dst, V)
    feat = si.features(V, F, seed)
    lab = si.labels(V, dims[-1], seed)
    train = si.train_split(V, 0.65, seed)
    weights = [tuple(np.asarray(t, np.float64) for t in w) for w in si.init_weights(list(dims), seed)]
    return src, dst, g, feat, lab, train, weights, B


def test_refresh_with_full_neighbourhood_is_the_exact_layer1_embedding():
    """Fanout >= max degree: row i is relu(W_self^T x_v + W_neigh^T mean_{u in N_in(v)} x_u + b) for
    v = hot_ids[i], written out here over the raw edge list with Python loops."""
    src, dst, g, feat, lab, train, weights, B = _problem()
    kmax = int(np.diff(g.rowptr).max())
    cache = ora.select_hot(g, train, B, (kmax, kmax), 1, 0.25, 3, 5, 0)
    assert cache.n_hot == 35
    emb, ver = ora.refresh_hot(g, feat, cache, weights[0], kmax, 7, 11)
    assert emb.shape == (35, 5) and (ver == 7).all() and ver.dtype == np.int32
    w_self, w_neigh, bias = weights[0]
    x = feat.astype(np.float64)
    for i, v in enumerate(cache.hot_ids):
        nb = [int(s) for s, d in zip(src, dst) if d == v]          # in-neighbours with multiplicity
        mean = np.zeros(x.shape[1]) if not nb else sum(x[u] for u in nb) / len(nb)
        z = x[v] @ w_self + mean @ w_neigh + bias
        assert np.allclose(emb[i], np.maximum(z, 0.0), rtol=1e-12, atol=1e-12), (i, v)
    # the call computes, it does not install: the cache is untouched until the commit
    assert (cache.version == -1).all() and (cache.emb == 0).all()
    ora.commit_refresh(cache, emb, ver)
    assert (cache.version == 7).all() and np.array_equal(cache.emb, emb)


def test_refresh_samples_each_hot_vertex_like_a_bottom_hop_destination():
    """Structure of a sampled refresh: min(deg, fanout) distinct edge positions per hot vertex, drawn from
    its own Philox stream (domain 2), so it differs from the training stream's sample of the same vertex and
    changes with the version."""
    src, dst, g, feat, lab, train, weights, B = _problem(E=2500)
    cache = ora.select_hot(g, train, B, (3, 2), 1, 0.3, 3, 5, 0)
    k = 2
    blk = ora.sample_hop(g, cache.hot_ids, k, ora._u64(11 + 4), ora.DOMAIN_REFRESH, 0)
    deg = np.diff(g.rowptr)[cache.hot_ids]
    assert np.array_equal(np.diff(blk.indptr), np.minimum(deg, k))
    emb_a, _ = ora.refresh_hot(g, feat, cache, weights[0], k, 4, 11)
    # same rows as the layer-1 forward over that block
    x = feat[blk.src_global].astype(np.float64)
    _, h = ora.sage_layer_fwd(blk, x, *weights[0], relu=True)
    assert np.array_equal(emb_a, h)
    emb_b, _ = ora.refresh_hot(g, feat, cache, weights[0], k, 5, 11)
    emb_c, _ = ora.refresh_hot(g, feat, cache, weights[0], k, 4, 11)
    assert np.array_equal(emb_a, emb_c) and not np.array_equal(emb_a, emb_b)
    train_blk = ora.sample_hop(g, cache.hot_ids, k, ora._u64(11 + 4), ora.DOMAIN_TRAIN, 0)
    assert not np.array_equal(train_blk.nbr_global, blk.nbr_global)


def test_superbatch_schedule_version_gaps_match_the_paper():
    """n batches per super-batch, bound S = 2n - 1: from the second super-batch on every hot vertex of V^1 is
    served from the cache, the age of a served row in batch j of a super-batch is n + j, and the largest gap,
    2n - 1, is reached in the last batch of a super-batch (the case the paper singles out)."""
    src, dst, g, feat, lab, train, weights, B = _problem(E=2500)
    fan = (3, 2)
    n = 3
    cache = ora.select_hot(g, train, B, fan, 2, 0.3, 2 * n - 1, 5, 0)
    batches = [si.batch_seeds(train, B, t) for t in range(4 * n)]
    # the schedule written out, recording the versions just before each step
    pending = None
    ws = weights
    rows = []
    for t, seeds in enumerate(batches):
        if t % n == 0:
            if pending is not None:
                ora.commit_refresh(cache, *pending)
            pending = ora.refresh_hot(g, feat, cache, ws[0], fan[-1], t, 9)
        ver_before = cache.version.copy()
        r = ora.train_step(g, feat, lab, seeds, fan, ws, 0.05, 9, t, cache)
        v1 = r.batch.blocks[0].src_global
        hot_in_v1 = int((cache.slot_of_vertex[v1] >= 0).sum())
        rows.append((t, hot_in_v1, r.n_hit, t - ver_before[r.batch.hit_slot]))
        ws = r.new_weights
    max_gap = 0
    for t, hot_in_v1, n_hit, ages in rows:
        if t < n:
            # first super-batch: nothing committed yet, only rows refreshed lazily by earlier steps can hit
            assert (ages >= 1).all() and (ages <= t).all()
            continue
        assert n_hit == hot_in_v1 and hot_in_v1 > 0, (t, n_hit, hot_in_v1)
        # committed rows carry the version of the previous super-batch's first step
        assert (ages == n + t % n).all(), (t, ages)
        max_gap = max(max_gap, int(ages.max()))
        if t % n == n - 1:
            assert int(ages.max()) == 2 * n - 1
    assert max_gap == 2 * n - 1
    # the driver in the oracle walks the same schedule
    cache2 = ora.select_hot(g, train, B, fan, 2, 0.3, 2 * n - 1, 5, 0)
    res, w_end = ora.train_superbatches(g, feat, lab, batches, fan, weights, 0.05, 9, cache2, n)
    assert [x.n_hit for x in res] == [x[2] for x in rows]
    assert np.array_equal(cache2.emb, cache.emb) and np.array_equal(cache2.version, cache.version)
    for a, b in zip(w_end, ws):
        for p, q in zip(a, b):
            assert np.array_equal(p, q)


def test_frozen_weights_and_full_neighbourhood_make_the_schedule_exact():
    """lr = 0 and every neighbour sampled: a bulk-refreshed row equals the row the step would compute, so
    the losses of the super-batch schedule equal those of training without a cache."""
    src, dst, g, feat, lab, train, weights, B = _problem()
    kmax = int(np.diff(g.rowptr).max())
    fan = (kmax, kmax)
    n = 2
    cache = ora.select_hot(g, train, B, fan, 1, 0.4, 2 * n - 1, 5, 0)
    batches = [si.batch_seeds(train, B, t) for t in range(3 * n)]
    res, _ = ora.train_superbatches(g, feat, lab, batches, fan, weights, 0.0, 3, cache, n)
    hits = 0
    for t, (seeds, r) in enumerate(zip(batches, res)):
        exact = ora.train_step(g, feat, lab, seeds, fan, weights, 0.0, 3, t, None)
        assert abs(r.loss - exact.loss) < 1e-12
        hits += r.n_hit
    assert hits > 0


def test_bound_below_n_makes_committed_rows_unusable():
    """With S < n a committed row is already n > S steps old when it becomes current, and the commit replaces
    every slot: the first batch of each later super-batch reuses nothing, and every later hit is at most S
    steps old, i.e. comes from the step's own refresh-on-miss."""
    src, dst, g, feat, lab, train, weights, B = _problem(E=2500)
    fan = (3, 2)
    n, S = 3, 1
    cache = ora.select_hot(g, train, B, fan, 2, 0.3, S, 5, 0)
    batches = [si.batch_seeds(train, B, t) for t in range(3 * n)]
    pending, ws, total_hits = None, weights, 0
    for t, seeds in enumerate(batches):
        if t % n == 0:
            if pending is not None:
                ora.commit_refresh(cache, *pending)
                assert (cache.version == t - n).all()
            pending = ora.refresh_hot(g, feat, cache, ws[0], fan[-1], t, 9)
        ver_before = cache.version.copy()
        r = ora.train_step(g, feat, lab, seeds, fan, ws, 0.05, 9, t, cache)
        ws = r.new_weights
        if t >= n and t % n == 0:
            assert r.n_hit == 0
        assert (t - ver_before[r.batch.hit_slot] <= S).all()
        total_hits += r.n_hit
    assert total_hits > 0


def test_weight_drift_stays_within_the_paper_tolerance():
    """Section 4.3: with eps = (largest single-update change of a layer-1 weight) x 2n, the drift between the
    parameters a served row was made with (version kn) and the parameters of the step that uses it (at most
    2n - 1 updates later) never exceeds eps: triangle inequality over the updates in between."""
    src, dst, g, feat, lab, train, weights, B = _problem(E=2500)
    fan = (3, 2)
    n = 3
    cache = ora.select_hot(g, train, B, fan, 2, 0.3, 2 * n - 1, 5, 0)
    batches = [si.batch_seeds(train, B, t) for t in range(4 * n)]
    ws, snaps, max_upd, drifts = weights, {}, 0.0, []
    pending_snap = current_snap = None
    pending = None
    for t, seeds in enumerate(batches):
        if t % n == 0:
            if pending is not None:
                ora.commit_refresh(cache, *pending)
                current_snap = pending_snap
            pending = ora.refresh_hot(g, feat, cache, ws[0], fan[-1], t, 9)
            pending_snap = ws[0]
        if current_snap is not None:
            drifts.append(ora.weight_drift(ws[0], current_snap))
        r = ora.train_step(g, feat, lab, seeds, fan, ws, 0.05, 9, t, cache)
        upd = ora.max_weight_update(ws[0], r.new_weights[0])
        assert abs(upd - 0.05 * max(np.abs(gr).max() for gr in r.grads[0])) < 1e-15      # the SGD closed form
        max_upd = max(max_upd, upd)
        ws = r.new_weights
    eps = ora.drift_tolerance(max_upd, n)
    assert eps == max_upd * 2 * n
    assert drifts and max(drifts) > 0 and max(drifts) <= (2 * n - 1) * max_upd <= eps
