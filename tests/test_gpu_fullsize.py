"""GPU parity at the full sizes of the named workloads, in the launch configuration bench.py times:
the dense (Reddit-shaped) and sparse (Products-shaped) workloads, several training steps with hot
reuse, every integer array bit-exact and every float tensor within tolerance against the oracle.
The oracle's per-step cost at these sizes is about a second, so whole steps are compared, not
samples."""
import dataclasses

import numpy as np
import pytest

import synth_inputs as si
from tests.test_gpu_parity import nb, run_steps, make_graph
from oracle import oracle as ora

pytestmark = pytest.mark.gpu


def test_dense_workload_full_size_steps():
    print("dense full size", flush=True)
    w = si.WORKLOADS["dense"]
    hits = run_steps(w, 4, use_cache=True, lr=0.01, bits=w.rowptr_bits, presample=1)
    assert hits > 0


def test_dense_workload_full_size_steps_prepared_ahead():
    """The stepping bench.py times: no_train_step_ahead, each batch prepared (sampled, split against the cache,
    layer-1 aggregate) beside the step before it."""
    print("dense full size, batches prepared ahead", flush=True)
    w = si.WORKLOADS["dense"]
    hits = run_steps(w, 4, use_cache=True, lr=0.01, bits=w.rowptr_bits, presample=1, ahead=True)
    assert hits > 0


def test_dense_workload_csr_and_hot_set_full_size():
    print("dense csr + hot set", flush=True)
    w = si.WORKLOADS["dense"]
    src, dst, og, gg = make_graph(w.n_vertices, w.n_edges, w.seed, w.rowptr_bits)
    b = nb()
    v, e, bits, rowptr, col = b.no_graph_view(gg)
    assert (v, e, bits) == (w.n_vertices, w.n_edges, 64)
    assert np.array_equal(rowptr.cpu().numpy(), og.rowptr)
    assert np.array_equal(col.cpu().numpy(), og.col)
    train = si.train_split(w.n_vertices, 0.65, w.seed)
    import torch
    oc = ora.select_hot(og, train, w.batch, w.fanouts, 3, w.hot_fraction, w.staleness, w.hidden, w.seed)
    gc = b.no_select_hot(gg, torch.from_numpy(train).cuda(), w.batch, w.fanouts, 3, w.hot_fraction, w.staleness,
                         w.hidden, w.seed)
    view = b.no_cache_view(gc, w.n_vertices)
    assert np.array_equal(view["freq"].cpu().numpy().astype(np.int64), oc.freq)
    assert np.array_equal(view["hot_ids"].cpu().numpy(), oc.hot_ids)


def test_sparse_workload_full_size_steps():
    print("sparse full size", flush=True)
    w = si.WORKLOADS["sparse"]
    hits = run_steps(w, 3, use_cache=True, lr=0.01, bits=w.rowptr_bits, presample=1, n_train_presample=20 * w.batch)
    assert hits > 0


def test_sweep_workload_full_size_steps_prepared_ahead():
    """The shape of the hot-ratio sweep (Fig. 14) used here: batch 4096, 256 features, hot 10 %, S = 2, at full size, batches
    prepared ahead."""
    print("sweep full size, batches prepared ahead", flush=True)
    w = si.WORKLOADS["sweep"]
    hits = run_steps(w, 3, use_cache=True, lr=0.01, bits=w.rowptr_bits, presample=1, n_train_presample=5 * w.batch,
                     ahead=True)
    assert hits > 0


class _RowsFromEdgeList:
    """In-neighbour rows of the vertices the oracle asks about, cut out of the raw edge list (the oracle's own CSR
    build of 1.6 G edges takes minutes; the rows of the few ten thousand vertices a batch reaches take seconds).
    The sub-graph is a CSR over all V vertices in which only the vertices asked for so far have their (complete)
    rows; a vertex that was never asked for reads as isolated, so a sampler that wandered off would be caught."""

    def __init__(self, src, dst, n_vertices, workers=16):
        self.src, self.dst, self.V, self.workers = src, dst, n_vertices, workers
        self.have = np.zeros(n_vertices, dtype=bool)
        self.parts_s, self.parts_d = [], []
        self._graph = None

    def ensure(self, ids):
        import concurrent.futures
        ids = np.unique(np.asarray(ids, dtype=np.int64))
        new = ids[~self.have[ids]]
        if len(new) == 0:
            return 0
        want = np.zeros(self.V, dtype=bool)
        want[new] = True
        chunk = 1 << 26

        def job(lo):
            hi = min(len(self.dst), lo + chunk)
            m = want[self.dst[lo:hi]]
            return self.src[lo:hi][m], self.dst[lo:hi][m]

        with concurrent.futures.ThreadPoolExecutor(self.workers) as ex:
            parts = list(ex.map(job, range(0, len(self.dst), chunk)))
        self.parts_s += [p[0] for p in parts]
        self.parts_d += [p[1] for p in parts]
        self.have[new] = True
        self._graph = None
        return int(sum(len(p[0]) for p in parts))

    def graph(self):
        if self._graph is None:
            s = np.concatenate(self.parts_s) if self.parts_s else np.zeros(0, np.int32)
            d = np.concatenate(self.parts_d) if self.parts_d else np.zeros(0, np.int32)
            self.parts_s, self.parts_d = [s], [d]
            self._graph = ora.build_csr(s, d, self.V)
        return self._graph


def test_large_workload_full_size_spot_check(capsys):
    """The largest configuration at its full size (111 M vertices, 1.6 G edges, int64 row pointers, 28 GB of bf16
    features, 11.1 M hot vertices with an 11 GB embedding cache): array offsets beyond 2^32 bytes in the column array,
    the feature table and the cache. Row pointers are compared in full; everything a training batch touches is
    compared with the oracle exactly as at the small sizes (blocks bit for bit, floats within tolerance), the oracle
    working on the rows of the vertices it reaches, cut out of the edge list hop by hop, and on the feature rows it
    gathers, copied back from the device table. Steps run as bench.py runs them (each batch prepared ahead)."""
    import time

    import psutil
    import torch

    from tests.test_gpu_parity import RTOL_BF16, assert_close, check_step_outputs, dev, make_relu_hook

    def say(*a):
        with capsys.disabled():
            print("[large]", *a, flush=True)

    if psutil.virtual_memory().available < 96 * 2 ** 30:
        pytest.skip("needs about 96 GB of free host memory for the edge list of 1.6 G edges and the oracle's rows")
    b = nb()
    w = si.WORKLOADS["large"]
    V = w.n_vertices
    t0 = time.time()
    src, dst = si.rmat_edges(V, w.n_edges, w.seed)
    say("edge list made in %.0f s" % (time.time() - t0))
    gg = b.no_build_csr(src, dst, V, w.rowptr_bits)
    v_, e_, bits_, rowptr, col = b.no_graph_view(gg)
    assert (v_, e_, bits_) == (V, w.n_edges, 64)
    # row pointers, all of them: prefix sums of the in-degree histogram of the edge list
    import concurrent.futures
    with concurrent.futures.ThreadPoolExecutor(4) as ex:
        cnt = sum(ex.map(lambda lo: np.bincount(dst[lo:lo + (1 << 27)], minlength=V).astype(np.int32),
                         range(0, len(dst), 1 << 27)))
    rp_host = rowptr.cpu().numpy()
    assert rp_host[0] == 0 and np.array_equal(np.cumsum(cnt.astype(np.int64)), rp_host[1:])
    del cnt
    say("row pointers match the degree histogram (%.0f s)" % (time.time() - t0))

    rows = _RowsFromEdgeList(src, dst, V)
    lab = si.labels(V, w.n_classes, w.seed)
    train = si.train_split(V, 0.65, w.seed)
    weights = si.init_weights(w.dims, w.seed)
    tfeat = si.features_on_device(V, w.feat_dim, w.seed, "bf16")
    assert tfeat.numel() * 2 > 2 ** 32
    feat_host = np.zeros((V, w.feat_dim), dtype=np.uint16)      # pages are only backed where rows are copied in
    tlab = dev(lab)

    def reach(seeds, fanouts, seed, step, domain):
        """Makes sure the rows of every destination of every hop are there (the oracle walks down hop by hop)."""
        got = rows.ensure(seeds)
        for h in range(len(fanouts) - 1):       # (nobody samples from the sources of the last hop)
            sb = ora.sample_blocks(rows.graph(), seeds, fanouts[:h + 1], seed, step, None, domain)
            got += rows.ensure(sb.blocks[h].src_global)
            say("  hop %d has %d destinations; %d edges cut out so far for this batch" % (h + 1, sb.blocks[h].n_src, got))

    # hot set: hotness pre-sampled on the first two batches only (one epoch), so most of the 11.1 M slots are filled in
    # id order and batches touch slots far beyond 2^32 bytes into the cache
    n_pre, nb_pre = 2 * w.batch, 2
    pre = np.ascontiguousarray(train[:n_pre])
    for bi in range(nb_pre):
        # (pre-sampling stream of batch bi in epoch 0: seed + bi, domain 1; hops 0 .. L-2)
        reach(pre[bi * w.batch:(bi + 1) * w.batch], w.fanouts[:-1], w.seed + bi, 0, ora.DOMAIN_PRESAMPLE)
    t1 = time.time()
    oc = ora.select_hot(rows.graph(), pre, w.batch, w.fanouts, 1, w.hot_fraction, w.staleness, w.hidden, w.seed)
    say("oracle hot set: %d vertices (%.0f s)" % (oc.n_hot, time.time() - t1))
    gc = b.no_select_hot(gg, dev(pre), w.batch, w.fanouts, 1, w.hot_fraction, w.staleness, w.hidden, w.seed)
    view = b.no_cache_view(gc, V)
    assert view["n_hot"] == oc.n_hot == 11_100_000 and oc.n_hot * w.hidden * 4 > 2 ** 32
    assert np.array_equal(view["freq"].cpu().numpy().astype(np.int64), oc.freq)
    assert np.array_equal(view["hot_ids"].cpu().numpy(), oc.hot_ids)
    say("hot sets agree")

    model = b.no_model_create(gg, w.dims, w.batch, w.fanouts, b.NO_BF16)
    for l in range(w.n_layers):
        for t, a in zip(b.no_model_params(model, l + 1), weights[l]):
            t.copy_(dev(a))
    ow = [tuple(np.asarray(t, np.float64) for t in x) for x in weights]
    n_steps, lr = 3, 0.01
    seed_tensors = [dev(si.batch_seeds(train, w.batch, t)) for t in range(n_steps)]
    hits = 0
    high_col = high_feat = high_slot = False
    stamped_ahead = None
    for step in range(n_steps):
        seeds = si.batch_seeds(train, w.batch, step)
        t1 = time.time()
        reach(seeds, w.fanouts, w.seed, step, ora.DOMAIN_TRAIN)
        og = rows.graph()
        # feature rows the oracle will gather: copied back from the device table
        sb = ora.sample_blocks(og, seeds, w.fanouts, w.seed, step, oc)
        ids = sb.blocks[-1].src_global
        feat_host[ids] = tfeat[torch.from_numpy(ids.astype(np.int64)).cuda()].cpu().numpy().view(np.uint16)
        high_feat |= bool((ids.astype(np.int64) * w.feat_dim * 2 > 2 ** 32).any())
        # the CSR rows of this batch's destinations, entry by entry (offsets into a 6.4 GB column array)
        v1 = sb.blocks[-2].src_global.astype(np.int64)
        lo, hi = rp_host[v1], rp_host[v1 + 1]
        assert np.array_equal(hi - lo, og.rowptr[v1 + 1] - og.rowptr[v1])
        take = np.argsort(hi - lo)[-64:]                      # the longest rows (hubs) and ...
        take = np.concatenate([take, np.arange(0, len(v1), max(1, len(v1) // 256))])      # ... an even sample of the rest
        for i in take:
            assert np.array_equal(col[lo[i]:hi[i]].cpu().numpy(), og.col[og.rowptr[v1[i]]:og.rowptr[v1[i] + 1]]), int(v1[i])
        high_col |= bool((hi[take] * 4 > 2 ** 32).any())
        nxt = seed_tensors[step + 1] if step + 1 < n_steps else None
        st = b.no_train_step_ahead(model, gg, tfeat, tlab, seed_tensors[step], nxt, False, gc, step, w.seed, lr)
        ambiguous = []
        r = ora.train_step(og, feat_host, lab, seeds, w.fanouts, ow, lr, w.seed, step, oc, feat_is_bf16=True,
                           relu_decisions=make_relu_hook(b, model, st, w.n_layers, ambiguous, band=1e-3))
        check_step_outputs(b, model, st, r, w.n_layers, step, True, False, np.uint16, RTOL_BF16)
        ow = r.new_weights
        hits += r.n_hit
        # cache: every version (slots stamped ahead for the next batch aside), and the rows this batch wrote or read
        view = b.no_cache_view(gc, V)
        gv = view["version"].cpu().numpy()
        stamped = (gv == step + 1) if nxt is not None else np.zeros(gv.shape, dtype=bool)
        assert np.array_equal(gv[~stamped], oc.version[~stamped])
        if stamped_ahead is not None:
            assert np.array_equal(np.flatnonzero(stamped_ahead), np.flatnonzero(oc.version == step))
        stamped_ahead = stamped if nxt is not None else None
        slots = oc.slot_of_vertex[sb.blocks[-2].src_global]
        slots = np.unique(slots[slots >= 0]).astype(np.int64)
        assert_close(view["emb"][torch.from_numpy(slots).cuda()].cpu().numpy(), oc.emb[slots], "cache rows step %d" % step,
                     RTOL_BF16)
        high_slot |= bool((slots * w.hidden * 4 > 2 ** 32).any())
        say("step %d matches: |V^1| %d, hits %d, loss %.5f, relu decisions from the kernel %s (%.0f s)"
            % (step, st.n_v1, st.n_hit, st.loss, ambiguous, time.time() - t1))
    assert hits > 0
    assert high_col and high_feat and high_slot      # offsets beyond 2^32 bytes were exercised in all three arrays
