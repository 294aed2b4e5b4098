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
