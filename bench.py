#!/usr/bin/env python3
"""Benchmark of the sample -> gather -> train hot path on one MI355X.

A "step" is one pass of the whole path (sample L hops, gather, forward, loss, backward, SGD,
cache refresh) over one batch of seeds of the named synthetic workload, with graph, features,
labels, weights and the seed batches already resident in HBM. Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload dense|tiny|sparse|sweep]

`value` = train steps/s of the unprofiled timed region. A second pass over the same steps with
per-stage HIP events on the step's stream gives the stage times, the sampled-edges/s and gather
GB/s figures (`extra`) and the `roofline` object of the dominant kernel. `cpu_baseline` times the
CPU oracle on a bounded number of the same steps.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
MFMA_F32_PEAK_TFLOPS = 157.3    # MI355X dense fp32 matrix


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="dense")
    ap.add_argument("--no-cache", action="store_true", help="exact training (no hot-embedding reuse)")
    ap.add_argument("--cpu-steps", type=int, default=-1, help="oracle steps to time (-1: auto, 0: skip)")
    ap.add_argument("--presample-epochs", type=int, default=3)
    ap.add_argument("--superbatch", type=int, default=4,
                    help="also time the super-batch schedule: bulk refresh of all hot rows every n steps on a second "
                         "stream, bound 2n-1 (0 = skip)")
    ap.add_argument("--presample-batches", type=int, default=0,
                    help="pre-sample hotness on the first N batches of the train split only (0: all)")
    ap.add_argument("--device-features", action="store_true",
                    help="generate the feature table in device memory (implied for tables over 2^31 elements); "
                         "the CPU baseline is skipped then")
    ap.add_argument("--lr", type=float, default=0.01)
    ap.add_argument("--no-ahead", action="store_true",
                    help="throughput pass with no_train_step (sample, then train) instead of no_train_step_ahead "
                         "(batch t+1 sampled on a second stream while batch t trains)")
    ap.add_argument("--arch", choices=["sage", "gcn"], default="sage",
                    help="layer form: GraphSAGE-mean (the headline configuration) or the GCN-style layer")
    ap.add_argument("--batch", type=int, default=0,
                    help="seeds per batch instead of the workload's (the paper's batch-size sweep, 256 .. 10000)")
    ap.add_argument("--fanouts", default="",
                    help="comma-separated fanouts from the seeds down instead of the workload's (deeper models: the "
                         "paper repeats the last value, e.g. 25,10,5,5)")
    ap.add_argument("--hot-fraction", type=float, default=-1.0,
                    help="share of the vertices kept hot instead of the workload's (the hot-ratio sweep of Fig. 14: 0, 0.1, 0.3)")
    ap.add_argument("--staleness", type=int, default=-1, help="staleness bound S instead of the workload's")
    ap.add_argument("--copy-reference", action="store_true",
                    help="only run a plain copy of known size (1,000,000 rows x 1024 B through no_gather_features with "
                         "ids 0..n-1): the reference that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus %d is not supported."
            % args.gpus)
        sys.exit(2)

    import numpy as np
    import torch

    import synth_inputs as si
    from paper_2311_13225_amd import binding as b

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(3)
    b.lib()   # fail loudly if the HIP library is missing
    if args.copy_reference:
        rows, dim = 1_000_000, 256
        t = torch.randn(rows, dim, device="cuda")
        ids = torch.arange(rows, device="cuda", dtype=torch.int32)
        out = torch.empty(rows, dim, device="cuda")
        for _ in range(3):
            b.no_gather_features(t, ids, out)
        torch.cuda.synchronize()
        print(json.dumps({"copy_reference": True, "launches": 3, "bytes_read_per_launch": rows * dim * 4 + rows * 4,
                          "bytes_written_per_launch": rows * dim * 4}), flush=True)
        return
    w = si.WORKLOADS[args.workload]
    if args.batch > 0 or args.fanouts:
        import dataclasses
        w = dataclasses.replace(w, batch=args.batch if args.batch > 0 else w.batch,
                                fanouts=tuple(int(x) for x in args.fanouts.split(",")) if args.fanouts else w.fanouts)
    K, W = args.steps, args.warmup
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    t0 = time.time()
    src, dst = si.rmat_edges(w.n_vertices, w.n_edges, w.seed, symmetrise=w.symmetrise)
    log("[bench] R-MAT %d vertices %d edges: %.1fs" % (w.n_vertices, len(src), time.time() - t0))
    t0 = time.time()
    device_features = args.device_features or w.n_vertices * w.feat_dim > (1 << 31)
    feat = None if device_features else si.features(w.n_vertices, w.feat_dim, w.seed, w.feat_dtype)
    lab = si.labels(w.n_vertices, w.n_classes, w.seed)
    train = si.train_split(w.n_vertices, 0.65, w.seed)
    weights = si.init_weights(w.dims, w.seed)
    bf16 = w.feat_dtype == "bf16"
    log("[bench] features/labels: %.1fs" % (time.time() - t0))

    t0 = time.time()
    g = b.no_build_csr(src, dst, w.n_vertices, w.rowptr_bits)
    torch.cuda.synchronize()
    t_csr = time.time() - t0
    log("[bench] no_build_csr (incl. H2D of the edge list): %.2fs" % t_csr)
    if device_features:
        tfeat = si.features_on_device(w.n_vertices, w.feat_dim, w.seed, w.feat_dtype)
    else:
        tfeat = dev(feat.view(np.int16) if bf16 else feat)
    tlab = dev(lab)
    ttrain = dev(train)
    if args.hot_fraction >= 0.0 or args.staleness >= 0:
        import dataclasses
        w = dataclasses.replace(w, hot_fraction=args.hot_fraction if args.hot_fraction >= 0.0 else w.hot_fraction,
                                staleness=args.staleness if args.staleness >= 0 else w.staleness)
    cache = None
    t_hot = 0.0
    if not args.no_cache and w.hot_fraction > 0.0:
        t0 = time.time()
        pre = ttrain if args.presample_batches <= 0 else ttrain[: args.presample_batches * w.batch].contiguous()
        cache = b.no_select_hot(g, pre, w.batch, w.fanouts, args.presample_epochs, w.hot_fraction, w.staleness,
                                w.hidden, w.seed)
        torch.cuda.synchronize()
        t_hot = time.time() - t0
        log("[bench] no_select_hot (%d pre-sampling epochs): %.2fs" % (args.presample_epochs, t_hot))
    model = b.no_model_create(g, w.dims, w.batch, w.fanouts, b.NO_BF16 if bf16 else b.NO_F32)
    gcn = args.arch == "gcn"
    if gcn:
        b.no_model_set_arch(model, b.NO_ARCH_GCN)

    def load_weights():
        for l in range(w.n_layers):
            for t, a in zip(b.no_model_params(model, l + 1), weights[l]):
                t.copy_(dev(a))

    seed_batches = [dev(si.batch_seeds(train, w.batch, t)) for t in range(W + K)]
    stream = torch.cuda.current_stream()

    def run(first, count, want_stats=False, ahead=False):
        out = []
        for t in range(first, first + count):
            if ahead:
                nxt = seed_batches[t + 1] if t + 1 < W + K else None
                st = b.no_train_step_ahead(model, g, tfeat, tlab, seed_batches[t], nxt, False, cache, t, w.seed, args.lr,
                                           want_stats=want_stats)
            else:
                st = b.no_train_step(model, g, tfeat, tlab, seed_batches[t], cache, t, w.seed, args.lr,
                                     want_stats=want_stats)
            out.append(st)
        return out

    # ---- pass 1: throughput (no events, no host sync inside the region)
    load_weights()
    if cache is not None:
        b.no_cache_invalidate(cache)
    use_ahead = not args.no_ahead
    run(0, W, ahead=use_ahead)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(W, K, ahead=use_ahead)
    enqueue_ms_per_step = (time.perf_counter() - t0) * 1e3 / K      # host time to enqueue a step (no wait for the GPU)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / K
    steps_per_s = K / elapsed
    log("[bench] %d steps in %.3fs -> %.1f steps/s (%.3f ms/step)" % (K, elapsed, steps_per_s, ms_per_step))

    # ---- pass 1b: the super-batch schedule of Section 4.2 (reported in `extra`, never as `value`): every n steps the
    # rows refreshed during the last super-batch are committed and the refresh for the next one starts on the
    # cache's own stream; bound 2n - 1, so from the second super-batch on every hot vertex of V^1 is served
    superbatch = None
    if cache is not None and args.superbatch > 0 and w.n_layers >= 2:
        n_sb = args.superbatch
        load_weights()
        b.no_cache_invalidate(cache)
        b.no_cache_set_staleness(cache, 2 * n_sb - 1)
        w1 = b.no_model_params(model, 1)

        sb_pending = [False]

        def run_sb(first, count, want_stats=False):
            out = []
            for t in range(first, first + count):
                if t % n_sb == 0:
                    if sb_pending[0]:
                        b.no_refresh_hot_commit(cache)
                    b.no_refresh_hot_begin(cache, g, tfeat, w1[0], None if gcn else w1[1], w1[2], w.fanouts[-1], t, w.seed)
                    sb_pending[0] = True
                if use_ahead:
                    nxt = seed_batches[t + 1] if t + 1 < W + K else None
                    # the boundary commit moves inside the call that samples the first batch of the next super-batch
                    commit = nxt is not None and (t + 1) % n_sb == 0 and sb_pending[0]
                    out.append(b.no_train_step_ahead(model, g, tfeat, tlab, seed_batches[t], nxt, commit, cache, t, w.seed,
                                                     args.lr, want_stats=want_stats))
                    if commit:
                        sb_pending[0] = False
                else:
                    out.append(b.no_train_step(model, g, tfeat, tlab, seed_batches[t], cache, t, w.seed, args.lr,
                                               want_stats=want_stats))
            return out

        W_sb = max(W, 2 * n_sb) // n_sb * n_sb         # warm-up ends on a boundary, past the first super-batch
        K_sb = min(K, W + K - W_sb)
        run_sb(0, W_sb - n_sb)
        sb_stats = run_sb(W_sb - n_sb, n_sb, want_stats=True)       # last warm-up super-batch: hit statistics
        sb_hit = sum(s_.n_hit for s_ in sb_stats) / max(1.0, float(sum(s_.n_v1 for s_ in sb_stats)))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_sb(W_sb, K_sb)
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        if sb_pending[0]:
            b.no_refresh_hot_commit(cache)              # leave nothing pending
            sb_pending[0] = False
        torch.cuda.synchronize()
        # refresh alone (begin + commit back to back on an idle GPU)
        t0 = time.perf_counter()
        for _ in range(5):
            b.no_refresh_hot_begin(cache, g, tfeat, w1[0], None if gcn else w1[1], w1[2], w.fanouts[-1], 0, w.seed)
            b.no_refresh_hot_commit(cache)
        torch.cuda.synchronize()
        refresh_ms = (time.perf_counter() - t0) * 1e3 / 5
        superbatch = {"n": n_sb, "staleness": 2 * n_sb - 1, "steps_per_s": round(K_sb / el, 2),
                      "ms_per_step": round(el * 1e3 / K_sb, 4), "timed_steps": K_sb,
                      "cache_hit_rate": round(sb_hit, 4), "refresh_alone_ms": round(refresh_ms, 3), "n_hot": int(b.no_cache_view(cache, w.n_vertices)["n_hot"])}
        log("[bench] super-batch schedule n=%d: %.1f steps/s (%.3f ms/step), refresh alone %.3f ms" %
            (n_sb, K_sb / el, el * 1e3 / K_sb, refresh_ms))
        b.no_cache_set_staleness(cache, w.staleness)

    # ---- pass 2: same steps again with per-stage events and per-step statistics
    load_weights()
    if cache is not None:
        b.no_cache_invalidate(cache)
    run(0, W)
    torch.cuda.synchronize()
    b.no_model_profile(model, True)
    stats = run(W, K, want_stats=True)
    stage_ms, n_prof = b.no_model_stage_ms(model)
    b.no_model_profile(model, False)
    per_step = {k: v / max(n_prof, 1) for k, v in stage_ms.items()}
    L = w.n_layers
    es = 2 if bf16 else 4
    F = w.feat_dim
    mean = lambda xs: float(sum(xs)) / max(len(xs), 1)
    nnz_total = mean([sum(s.nnz[h] for h in range(L)) for s in stats])
    n_src_bottom = mean([s.n_src[L - 1] for s in stats])
    n_dst_bottom = mean([s.n_dst[L - 1] for s in stats])
    nnz_bottom = mean([s.nnz[L - 1] for s in stats])
    n_hit = mean([s.n_hit for s in stats])
    n_v1 = mean([s.n_v1 for s in stats])
    loss_last = stats[-1].loss
    # Gather: inside the step only the bottom destinations' rows are copied (on the side stream, next to the
    # aggregation, which reads the neighbour rows in place), so the step has no gather stage to time. The
    # gather figure is no_gather_features on the FULL source list of the last step's bottom hop (what an
    # unfused step would collect), timed alone with events on the stream it runs on.
    blocks = b.no_model_blocks(model)
    view = b.no_blocks_view(blocks, L - 1)
    n_src_last = int(stats[-1].n_src[L - 1])
    ids_last = b._view(view.d_src_global, (n_src_last,), "<i4", blocks).clone()
    gout = torch.empty((n_src_last, F), dtype=tfeat.dtype, device="cuda")
    for _ in range(3):
        b.no_gather_features(tfeat, ids_last, gout)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_rep = 20
    e0.record()
    for _ in range(n_rep):
        b.no_gather_features(tfeat, ids_last, gout)
    e1.record()
    torch.cuda.synchronize()
    per_step["gather"] = e0.elapsed_time(e1) / n_rep          # ms per launch, standalone
    gather_bytes = n_src_last * (4 + 2 * F * es)
    del gout
    # compulsory traffic (each distinct source row once) plus the reused layer-1 rows that extra blocks of the same
    # launch copy from the cache into H^1 (read + write)
    agg_bytes = n_src_bottom * F * es + n_dst_bottom * F * 4 + nnz_bottom * 4 + (n_hit * w.dims[1] * 4 * 2 if L >= 2 else 0)
    gemm_fwd_flops = 2.0 * n_dst_bottom * ((1 if gcn else 2) * F) * w.dims[1]
    # the weight-gradient launch of layer 1 also carries the (smaller) weight-gradient products of the layers above
    gemm_dw_flops = gemm_fwd_flops + sum(
        2.0 * mean([st_.n_dst[L - l] for st_ in stats]) * ((1 if gcn else 2) * w.dims[l - 1]) * w.dims[l] for l in range(2, L + 1))
    kern = {
        "gather_rows_kernel": ("hbm", gather_bytes / 1e9 / (per_step["gather"] / 1e3), HBM_PEAK_GBPS, "GB/s", per_step["gather"]),
        "segment_rows_kernel(mean,l1)": ("hbm", agg_bytes / 1e9 / (per_step["agg_l1"] / 1e3), HBM_PEAK_GBPS, "GB/s", per_step["agg_l1"]),
        "gemm_nn_kernel(l1 fwd)": ("mfma", gemm_fwd_flops / 1e12 / (per_step["gemm_fwd_l1"] / 1e3), MFMA_F32_PEAK_TFLOPS, "TFLOP/s", per_step["gemm_fwd_l1"]),
        "gemm_tn_kernel(l1 dW)": ("mfma", gemm_dw_flops / 1e12 / (per_step["gemm_dw_l1"] / 1e3), MFMA_F32_PEAK_TFLOPS, "TFLOP/s", per_step["gemm_dw_l1"]),
    }
    dominant = max(kern, key=lambda k: kern[k][4])
    bound, achieved, peak, unit, dur = kern[dominant]
    # HBM bytes per launch from the rocprofv3 --pmc runs (FETCH_SIZE + WRITE_SIZE, scaled by the copy reference),
    # recorded in profiles/dense_hbm_traffic.json for this workload; null for other workloads or kernels
    traffic_all = {}
    tpath = os.path.join(ROOT, "profiles", "dense_hbm_traffic.json")
    default_shape = (args.batch <= 0 and not args.fanouts and args.hot_fraction < 0.0 and args.staleness < 0 and
                     args.arch == "sage")
    if args.workload == "dense" and default_shape and cache is not None and os.path.exists(tpath):
        try:
            traffic_all = json.load(open(tpath)).get("bytes_per_launch", {})
        except Exception:
            traffic_all = {}
    roofline = {"kernel": dominant, "bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
                "frac": round(achieved / peak, 4), "traffic": traffic_all.get(dominant), "avg_launch_ms": round(dur, 4),
                "all": {k: {"bound": v[0], "achieved": round(v[1], 3), "peak": v[2], "unit": v[3],
                            "frac": round(v[1] / v[2], 4), "avg_launch_ms": round(v[4], 4),
                            "traffic": traffic_all.get(k)} for k, v in kern.items()}}
    extra = {
        "sampled_edges_per_s": round(nnz_total / (per_step["sample"] / 1e3), 1),
        "sampled_edges_per_step": round(nnz_total, 1),
        "gather_GBps": round(kern["gather_rows_kernel"][1], 2),
        "gather_frac_hbm_peak": round(kern["gather_rows_kernel"][1] / HBM_PEAK_GBPS, 4),
        "aggregate_GBps": round(kern["segment_rows_kernel(mean,l1)"][1], 2),
        "aggregate_frac_hbm_peak": round(kern["segment_rows_kernel(mean,l1)"][1] / HBM_PEAK_GBPS, 4),
        # the same launch priced by the bytes it moved (rocprofv3 counters; a source row shared by several destinations
        # is fetched again when it has left the L2), not by the compulsory bytes above
        "aggregate_moved_GBps": (round(traffic_all["segment_rows_kernel(mean,l1)"] / 1e9 / (per_step["agg_l1"] / 1e3), 2)
                                 if "segment_rows_kernel(mean,l1)" in traffic_all else None),
        "rows_gathered_per_step": round(n_src_bottom, 1),
        "gather_measurement": "no_gather_features alone on the %d source rows of the last step's bottom hop "
                              "(in the step the neighbour rows are read inside the aggregation)" % n_src_last,
        "cache_hit_rate": round(n_hit / max(n_v1, 1.0), 4),
        "bytes_gathered_per_step": {"features": round(n_src_bottom * F * es, 1),
                                    "embeddings": round(n_hit * w.dims[1] * 4 if L >= 2 else 0.0, 1)},
        "stage_ms_per_step": {k: round(v, 4) for k, v in per_step.items()},
        "profiled_ms_per_step": round(sum(v for k, v in per_step.items() if k != "gather"), 4),
        "host_enqueue_ms_per_step": round(enqueue_ms_per_step, 4),
        "setup_s": {"build_csr": round(t_csr, 2), "select_hot": round(t_hot, 2)},
        "loss_after_last_step": round(float(loss_last), 5),
        "superbatch_schedule": superbatch,
    }
    log("[bench] stage ms/step: " + ", ".join("%s=%.3f" % kv for kv in per_step.items()))

    # ---- CPU baseline: the oracle, as it stands, on a bounded number of the same steps
    cpu = None
    cpu_steps = 0 if device_features else args.cpu_steps
    if cpu_steps != 0:
        from oracle import oracle as ora
        try:
            from threadpoolctl import threadpool_info
            blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            blas_threads = 1
        t0 = time.time()
        og = ora.build_csr(src, dst, w.n_vertices)
        oc = None
        if cache is not None:
            pre_h = train if args.presample_batches <= 0 else train[: args.presample_batches * w.batch]
            oc = ora.select_hot(og, pre_h, w.batch, w.fanouts, args.presample_epochs, w.hot_fraction, w.staleness,
                                w.hidden, w.seed)
        log("[bench] oracle setup (CSR + hot set): %.1fs" % (time.time() - t0))
        ow = [tuple(np.asarray(t, np.float64) for t in ((x[0], x[2]) if gcn else x)) for x in weights]
        # one untimed step to estimate the cost, then time as many as fit in ~20 s (at least 2)
        t0 = time.perf_counter()
        r = ora.train_step(og, feat, lab, si.batch_seeds(train, w.batch, 0), w.fanouts, ow, args.lr, w.seed, 0, oc,
                           feat_is_bf16=bf16, arch=args.arch)
        one = time.perf_counter() - t0
        ow = r.new_weights
        if cpu_steps < 0:
            cpu_steps = int(max(2, min(K, 20.0 / max(one, 1e-3))))
        t0 = time.perf_counter()
        for t in range(1, 1 + cpu_steps):
            r = ora.train_step(og, feat, lab, si.batch_seeds(train, w.batch, t), w.fanouts, ow, args.lr, w.seed, t, oc,
                               feat_is_bf16=bf16, arch=args.arch)
            ow = r.new_weights
        cpu_elapsed = time.perf_counter() - t0
        cpu = {"value": round(cpu_steps / cpu_elapsed, 4), "unit": "steps/s", "cores": int(blas_threads), "kind": "oracle",
               "sample": "%d steps (steps 1..%d of the same workload, after 1 untimed step); C parts single-threaded, "
                         "numpy fp64 BLAS on %d threads" % (cpu_steps, cpu_steps, blas_threads)}
        log("[bench] oracle: %d steps in %.1fs" % (cpu_steps, cpu_elapsed))

    line = {
        "metric": "train_steps_per_s", "value": round(steps_per_s, 2), "unit": "steps/s", "n_gpus": 1,
        "steps": K, "warmup": W, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: R-MAT %d vertices / %d directed edges, %d x %s features, %d classes, %d-layer "
                               "%s hidden %d, fanout %s, batch %d, hot %.0f%%, S=%d"
                               % (w.name, w.n_vertices, len(src), w.feat_dim, w.feat_dtype, w.n_classes, w.n_layers,
                                  "GCN-style" if gcn else "GraphSAGE-mean", w.hidden, list(w.fanouts), w.batch, 0.0 if cache is None else 100 * w.hot_fraction,
                                  w.staleness),
                   "hot_reuse": cache is not None},
        "roofline": roofline, "cpu_baseline": cpu, "extra": extra,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
