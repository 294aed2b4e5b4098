#!/usr/bin/env python3
"""Benchmark of the sample -> gather -> train hot path on one MI355X.

A "step" is one pass of the whole path (sample L hops, gather, forward, loss, backward, SGD,
cache refresh) over one batch of seeds of the named synthetic workload, with graph, features,
labels, weights and the seed batches already resident in HBM. Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large|dense|sparse|sweep|tiny]

The default workload is `large`, the largest configuration (111 M vertices, 1.6 G edges, 28 GB of bf16
features): the one the gather / aggregation target is stated on. `value` = train steps/s of the unprofiled
timed region. A second pass over the same steps with per-stage HIP events on the step's stream gives the
stage times, the sampled-edges/s and gather GB/s figures (`extra`) and the `roofline` object of the dominant
kernel. `cpu_baseline` times the CPU oracle on a bounded sample (on the mid-size graph with this workload's
feature and model shape when the workload's own graph and table do not fit the oracle's time budget).
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
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="large")
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
    ap.add_argument("--arch", choices=["sage", "gcn", "gcn_sum", "gcn_sym"], default="sage",
                    help="layer form: GraphSAGE-mean (the headline configuration) or a GCN-style layer (average, sum, "
                         "symmetric normalisation)")
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
    gcn = args.arch != "sage"
    if gcn:
        b.no_model_set_arch(model, b.ARCH_OF_NAME[args.arch])
        if cache is not None:
            b.no_cache_set_layer_form(cache, b.ARCH_OF_NAME[args.arch])

    def load_weights():
        for l in range(w.n_layers):
            for t, a in zip(b.no_model_params(model, l + 1), weights[l]):
                t.copy_(dev(a))

    # one batch more than is trained on: the last timed step also prepares a next batch, like every other step
    seed_batches = [dev(si.batch_seeds(train, w.batch, t)) for t in range(W + K + 1)]
    stream = torch.cuda.current_stream()

    def run(first, count, want_stats=False, ahead=False):
        out = []
        for t in range(first, first + count):
            if ahead:
                nxt = seed_batches[t + 1]
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
                    nxt = seed_batches[t + 1]
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
    L = w.n_layers
    blocks = b.no_model_blocks(model)
    N_GATHER_LISTS = 16
    id_lists = []            # bottom-hop source ids of the last N_GATHER_LISTS profiled steps (device copies)
    stats = []
    for t in range(W, W + K):
        st = b.no_train_step(model, g, tfeat, tlab, seed_batches[t], cache, t, w.seed, args.lr, want_stats=True)
        stats.append(st)
        if t >= W + K - N_GATHER_LISTS:
            view = b.no_blocks_view(blocks, L - 1)
            id_lists.append(b._view(view.d_src_global, (int(st.n_src[L - 1]),), "<i4", blocks).clone())
    stage_ms, n_prof = b.no_model_stage_ms(model)
    b.no_model_profile(model, False)
    per_step = {k: v / max(n_prof, 1) for k, v in stage_ms.items()}
    es = 2 if bf16 else 4
    F = w.feat_dim
    rp = w.rowptr_bits // 8
    mean = lambda xs: float(sum(xs)) / max(len(xs), 1)
    hop = lambda name, h: mean([getattr(s_, name)[h] for s_ in stats])
    nnz_total = sum(hop("nnz", h) for h in range(L))
    n_src_bottom, n_dst_bottom, nnz_bottom = hop("n_src", L - 1), hop("n_dst", L - 1), hop("nnz", L - 1)
    n_hit = mean([s_.n_hit for s_ in stats])
    n_v1 = mean([s_.n_v1 for s_ in stats])
    loss_last = stats[-1].loss
    # Gather: inside the step only the bottom destinations' rows are copied (on the side stream; the aggregation
    # reads the neighbour rows in place), so the step has no gather stage to time. The gather figure is
    # no_gather_features on the FULL source lists of the bottom hop (what an unfused step would collect), rotating
    # over the lists of the last 16 steps and over 16 output buffers so that the rows read and written between two
    # uses of a buffer exceed the 256 MB last-level cache: a cold, HBM-bound figure, timed with events on the
    # stream it runs on.
    gouts = [torch.empty((int(ids.numel()), F), dtype=tfeat.dtype, device="cuda") for ids in id_lists]
    for ids, gout in zip(id_lists, gouts):
        b.no_gather_features(tfeat, ids, gout)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_rep = 4
    e0.record()
    for _ in range(n_rep):
        for ids, gout in zip(id_lists, gouts):
            b.no_gather_features(tfeat, ids, gout)
    e1.record()
    torch.cuda.synchronize()
    n_launch = n_rep * len(id_lists)
    per_step["gather"] = e0.elapsed_time(e1) / n_launch          # ms per launch, standalone
    gather_rows = mean([int(ids.numel()) for ids in id_lists])
    gather_bytes = gather_rows * (4 + 2 * F * es)
    gather_working_set = sum(int(ids.numel()) for ids in id_lists) * 2 * F * es
    del gouts
    # for scale: a plain contiguous device-to-device copy of as many bytes per launch, rotating over as many buffers
    # (what a perfectly coalesced kernel with no dependent id load reaches at this launch size)
    n_copy = int(gather_rows) * F * es
    c_src = [torch.empty(n_copy, dtype=torch.uint8, device="cuda") for _ in id_lists]
    c_dst = [torch.empty(n_copy, dtype=torch.uint8, device="cuda") for _ in id_lists]
    for a_, b_ in zip(c_src, c_dst):
        b_.copy_(a_)
    e0.record()
    for _ in range(n_rep):
        for a_, b_ in zip(c_src, c_dst):
            b_.copy_(a_)
    e1.record()
    torch.cuda.synchronize()
    plain_copy_gbps = 2 * n_copy / 1e9 / (e0.elapsed_time(e1) / n_launch / 1e3)
    del c_src, c_dst
    # compulsory traffic (each distinct source row once) plus the reused layer-1 rows that extra blocks of the same
    # launch copy from the cache into H^1 (read + write)
    agg_bytes = n_src_bottom * F * es + n_dst_bottom * F * 4 + nnz_bottom * 4 + (n_hit * w.dims[1] * 4 * 2 if L >= 2 else 0)
    gemm_fwd_flops = 2.0 * n_dst_bottom * ((1 if gcn else 2) * F) * w.dims[1]
    # the weight-gradient launch of layer 1 also carries the (smaller) weight-gradient products of the layers above
    gemm_dw_flops = gemm_fwd_flops + sum(
        2.0 * hop("n_dst", L - l) * ((1 if gcn else 2) * w.dims[l - 1]) * w.dims[l] for l in range(2, L + 1))
    # Sampling, algorithmic bytes. Per destination of a hop: two row pointers and its id; per sampled edge: the
    # column entry read and the neighbour id written. Relabelling: each sampled slot read and written once, one 4-byte
    # probe of the id map, the new sources' ids. Transpose (hops above the bottom one): indices and rows read, two
    # arrays written.
    sample_rows_bytes = lambda h: hop("n_dst", h) * (2 * rp + 4) + hop("nnz", h) * 8
    relabel_bytes = lambda h: hop("nnz", h) * 12 + hop("n_src", h) * 4 + hop("n_dst", h) * 4
    csc_bytes = lambda h: hop("nnz", h) * 16 if h < L - 1 else 0.0
    sampling_bytes = sum(sample_rows_bytes(h) + relabel_bytes(h) + csc_bytes(h) for h in range(L))
    ms = per_step
    AGG, FWD, DW = "padded_rows_kernel(mean,l1)", "gemm_nn_kernel(l1 fwd)", "gemm_tn_kernel(l1 dW)"
    if args.arch == "gcn_sym":
        AGG = "segment_rows_kernel(sym,l1)"        # per-source weights: through the compacted indices
    kern = {
        "gather_rows_kernel": ("hbm", gather_bytes / 1e9 / (ms["gather"] / 1e3), HBM_PEAK_GBPS, "GB/s", ms["gather"]),
        AGG: ("hbm", agg_bytes / 1e9 / (ms["agg_l1"] / 1e3), HBM_PEAK_GBPS, "GB/s", ms["agg_l1"]),
        "sample_rows_kernel(bottom hop)": ("hbm", sample_rows_bytes(L - 1) / 1e9 / (max(ms["sample_rows_bottom"], 1e-6) / 1e3),
                                           HBM_PEAK_GBPS, "GB/s", ms["sample_rows_bottom"]),
    }
    bf16_products = bf16 and not gcn
    mfma_note = None
    if bf16_products:
        # Layer 1 on a bf16 table: bf16 operands on the matrix cores. At 16x the fp32 matrix rate these two launches are
        # bound by their operands' bytes: bf16 rows + fp32 mean in, fp32 rows out (and the refreshed cache rows); for the
        # weight gradients bf16 rows + fp32 mean + fp32 output gradient in, the partial tiles out. Their matrix-core
        # share is reported beside (flops over the bf16 peak).
        FWD, DW = "gemm_bf16_nn_kernel(l1 fwd)", "gemm_bf16_tn_kernel(l1 dW)"
        n_refresh = mean([s_.n_refresh for s_ in stats]) if L >= 2 else 0.0
        H1 = w.dims[1]
        fwd_bytes = n_dst_bottom * (F * 2 + F * 4) + n_dst_bottom * H1 * 4 + n_refresh * H1 * 4
        used_splits = min(64.0, max(1.0, n_dst_bottom / 256.0))
        dw_bytes = n_dst_bottom * (F * 2 + F * 4 + H1 * 4) + used_splits * 2 * (F + 1) * H1 * 4
        l1_flops = 2.0 * n_dst_bottom * 2 * F * H1
        kern[FWD] = ("hbm", fwd_bytes / 1e9 / (ms["gemm_fwd_l1"] / 1e3), HBM_PEAK_GBPS, "GB/s", ms["gemm_fwd_l1"])
        kern[DW] = ("hbm", dw_bytes / 1e9 / (ms["gemm_dw_l1"] / 1e3), HBM_PEAK_GBPS, "GB/s", ms["gemm_dw_l1"])
        mfma_note = {FWD: round(l1_flops / 1e12 / (ms["gemm_fwd_l1"] / 1e3) / MFMA_BF16_PEAK_TFLOPS, 4),
                     DW: round(l1_flops / 1e12 / (ms["gemm_dw_l1"] / 1e3) / MFMA_BF16_PEAK_TFLOPS, 4)}
    else:
        kern[FWD] = ("mfma", gemm_fwd_flops / 1e12 / (ms["gemm_fwd_l1"] / 1e3), MFMA_F32_PEAK_TFLOPS, "TFLOP/s", ms["gemm_fwd_l1"])
        kern[DW] = ("mfma", gemm_dw_flops / 1e12 / (ms["gemm_dw_l1"] / 1e3), MFMA_F32_PEAK_TFLOPS, "TFLOP/s", ms["gemm_dw_l1"])
    dominant = max(kern, key=lambda k: kern[k][4])
    bound, achieved, peak, unit, dur = kern[dominant]
    # HBM bytes per launch from rocprofv3 --pmc runs of this workload (FETCH_SIZE + WRITE_SIZE, scaled by a copy of
    # known size), stored in profiles/<workload>_hbm_traffic.json: a constant of that profile run, not of this run;
    # null for shapes other than the workload's default
    traffic_all, traffic_source = {}, None
    tpath = os.path.join(ROOT, "profiles", "%s_hbm_traffic.json" % args.workload)
    default_shape = (args.batch <= 0 and not args.fanouts and args.hot_fraction < 0.0 and args.staleness < 0 and
                     args.arch == "sage")
    if default_shape and cache is not None and os.path.exists(tpath):
        try:
            tj = json.load(open(tpath))
            traffic_all = tj.get("bytes_per_launch", {})
            traffic_source = "stored: profiles/%s_hbm_traffic.json (%s)" % (args.workload, tj.get("measured", "rocprofv3 --pmc"))
        except Exception:
            traffic_all = {}
    entry = lambda k, v: {"bound": v[0], "achieved": round(v[1], 3), "peak": v[2], "unit": v[3],
                          "frac": round(v[1] / v[2], 4), "avg_launch_ms": round(v[4], 4), "traffic": traffic_all.get(k)}
    roofline = {"kernel": dominant, "bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
                "frac": round(achieved / peak, 4), "traffic": traffic_all.get(dominant), "avg_launch_ms": round(dur, 4),
                "traffic_source": traffic_source,
                "all": {k: entry(k, v) for k, v in kern.items()}}
    if mfma_note:
        for k, v in mfma_note.items():
            roofline["all"][k]["frac_of_bf16_mfma_peak"] = v
        if dominant in mfma_note:
            roofline["frac_of_bf16_mfma_peak"] = mfma_note[dominant]
    # the whole sampling stage (about four launches per hop plus the transposes), priced by its algorithmic bytes
    roofline["all"]["sampling stage (a1-a3, all hops, all its kernels)"] = {
        "bound": "hbm", "achieved": round(sampling_bytes / 1e9 / (ms["sample"] / 1e3), 3), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(sampling_bytes / 1e9 / (ms["sample"] / 1e3) / HBM_PEAK_GBPS, 5), "avg_launch_ms": round(ms["sample"], 4),
        "traffic": traffic_all.get("sampling stage"), "note": "a chain of dependent launches bound by latency, not by bytes"}
    target = 0.60
    gather_frac = kern["gather_rows_kernel"][1] / HBM_PEAK_GBPS
    agg_frac = kern[AGG][1] / HBM_PEAK_GBPS
    extra = {
        # every hop's sampled edges over the whole sampling stage: sampling, relabelling, hot lookup, local indices,
        # transposes and the wipe of the id map (the measurement pass joins the side stream inside the stage)
        "sampled_edges_per_s": round(nnz_total / (ms["sample"] / 1e3), 1),
        "sampled_edges_per_step": round(nnz_total, 1),
        "sampling_algorithmic_bytes_per_step": round(sampling_bytes, 1),
        "gather_GBps": round(kern["gather_rows_kernel"][1], 2),
        "gather_frac_hbm_peak": round(gather_frac, 4),
        "plain_copy_same_bytes_GBps": round(plain_copy_gbps, 2),
        "aggregate_GBps": round(kern[AGG][1], 2),
        "aggregate_frac_hbm_peak": round(agg_frac, 4),
        "target_60pct_hbm_peak": {"gather": bool(gather_frac >= target), "aggregate": bool(agg_frac >= target)},
        "rows_gathered_per_step": round(n_src_bottom, 1),
        "gather_measurement": "no_gather_features alone, rotating over the bottom-hop source lists of the last %d steps "
                              "(%.0f rows each on average) and %d output buffers: %.0f MB read + written per round, past "
                              "the 256 MB last-level cache (in the step the neighbour rows are read inside the aggregation)"
                              % (len(id_lists), gather_rows, len(id_lists), gather_working_set / 1e6),
        "cache_hit_rate": round(n_hit / max(n_v1, 1.0), 4),
        "v1_per_step": {"hit": round(n_hit, 1), "miss_hot": round(mean([s_.n_miss_hot for s_ in stats]), 1),
                        "cold": round(mean([s_.n_cold for s_ in stats]), 1)},
        # written by the step's statistics block on the device
        "bytes_gathered_per_step": {"features": round(mean([s_.bytes_gathered_features for s_ in stats]), 1),
                                    "embeddings": round(mean([s_.bytes_gathered_embeddings for s_ in stats]), 1)},
        "stage_ms_per_step": {k: round(v, 4) for k, v in per_step.items()},
        "profiled_ms_per_step": round(sum(v for k, v in per_step.items() if k not in ("gather", "sample_rows_bottom")), 4),
        "host_enqueue_ms_per_step": round(enqueue_ms_per_step, 4),
        "setup_s": {"build_csr": round(t_csr, 2), "select_hot": round(t_hot, 2)},
        "loss_after_last_step": round(float(loss_last), 5),
        "superbatch_schedule": superbatch,
    }
    log("[bench] stage ms/step: " + ", ".join("%s=%.3f" % kv for kv in per_step.items()))
    n_edges_made = len(src)

    # ---- CPU baseline: the oracle, as it stands, on a bounded sample
    cpu = None
    if args.cpu_steps != 0:
        import dataclasses
        # free what the GPU legs needed on the host (12.8 GB of edges for the large workload)
        cw, c_src, c_dst, c_feat, c_lab, c_train = w, src, dst, feat, lab, train
        where = "the same workload"
        if device_features:
            del src, dst, c_src, c_dst
            # The workload's own graph and table are beyond the oracle's time budget (its CSR build alone takes minutes
            # for 1.6 G edges): the oracle runs on the mid-size sparse graph with this workload's feature width and
            # dtype, classes, model, fanouts, batch, hot share and bound.
            sp = si.WORKLOADS["sparse"]
            cw = dataclasses.replace(sp, name="sparse graph with the %s workload's shapes" % w.name, feat_dim=w.feat_dim,
                                     feat_dtype=w.feat_dtype, n_classes=w.n_classes, hidden=w.hidden, fanouts=w.fanouts,
                                     batch=w.batch, hot_fraction=w.hot_fraction, staleness=w.staleness)
            t0 = time.time()
            c_src, c_dst = si.rmat_edges(cw.n_vertices, cw.n_edges, cw.seed, symmetrise=cw.symmetrise)
            c_feat = si.features(cw.n_vertices, cw.feat_dim, cw.seed, cw.feat_dtype)
            c_lab = si.labels(cw.n_vertices, cw.n_classes, cw.seed)
            c_train = si.train_split(cw.n_vertices, 0.65, cw.seed)
            where = ("R-MAT %d vertices / %d edges (the mid-size graph) with the %s workload's %d x %s features, %d classes, "
                     "model, fanouts and batch" % (cw.n_vertices, len(c_src), w.name, cw.feat_dim, cw.feat_dtype, cw.n_classes))
            log("[bench] oracle inputs (%s): %.1fs" % (where, time.time() - t0))
        cpu = cpu_baseline(cw, c_src, c_dst, c_feat, c_lab, c_train, weights, cache is not None, args, gcn, K, where)

    line = {
        "metric": "train_steps_per_s", "value": round(steps_per_s, 2), "unit": "steps/s", "n_gpus": 1,
        "steps": K, "warmup": W, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16+f32" if bf16_products else "f32", "data": "synthetic",
        "config": {"workload": "%s: R-MAT %d vertices / %d directed edges, %d x %s features, %d classes, %d-layer "
                               "%s hidden %d, fanout %s, batch %d, hot %.0f%%, S=%d"
                               % (w.name, w.n_vertices, n_edges_made, w.feat_dim, w.feat_dtype, w.n_classes, w.n_layers,
                                  ("GCN-style (%s)" % args.arch) if gcn else "GraphSAGE-mean", w.hidden, list(w.fanouts), w.batch, 0.0 if cache is None else 100 * w.hot_fraction,
                                  w.staleness),
                   "hot_reuse": cache is not None},
        "roofline": roofline, "cpu_baseline": cpu, "extra": extra,
    }
    print(json.dumps(line), flush=True)


def cpu_baseline(cw, src, dst, feat, lab, train, weights, with_cache, args, gcn, K, where):
    """Times the CPU oracle (never tuned for this) on a bounded number of steps: once with numpy's BLAS on all the
    threads it takes by itself, once with every library limited to one thread. The C parts (sampling, relabelling,
    gather, aggregation) are single-threaded in both."""
    import numpy as np

    import synth_inputs as si
    from oracle import oracle as ora
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threadpool_limits = None
        blas_threads = 1
    bf16 = cw.feat_dtype == "bf16"
    t0 = time.time()
    og = ora.build_csr(src, dst, cw.n_vertices)
    oc = None
    pre_batches = 64
    if with_cache and cw.hot_fraction > 0.0:
        # hotness from one pre-sampling epoch over the first batches only: bounds the oracle's set-up time
        oc = ora.select_hot(og, train[: pre_batches * cw.batch], cw.batch, cw.fanouts, 1, cw.hot_fraction, cw.staleness,
                            cw.hidden, cw.seed)
    log("[bench] oracle setup (CSR + hot set): %.1fs" % (time.time() - t0))
    ow = [tuple(np.asarray(t, np.float64) for t in ((x[0], x[2]) if gcn else x)) for x in weights]
    arch = args.arch
    state = {"w": ow, "t": 0}

    def steps(n):
        t0 = time.perf_counter()
        for _ in range(n):
            t = state["t"]
            r = ora.train_step(og, feat, lab, si.batch_seeds(train, cw.batch, t), cw.fanouts, state["w"], args.lr, cw.seed, t, oc,
                               feat_is_bf16=bf16, arch=arch)
            state["w"] = r.new_weights
            state["t"] = t + 1
        return time.perf_counter() - t0

    one = steps(1)                     # untimed for the figures: estimates the cost of a step
    n = args.cpu_steps if args.cpu_steps > 0 else int(max(2, min(K, 10.0 / max(one, 1e-3))))
    el_all = steps(n)
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            el_one = steps(n)
    else:
        el_one = None
    log("[bench] oracle: %d steps in %.1fs on %d BLAS threads, %s on one thread" %
        (n, el_all, blas_threads, "-" if el_one is None else "%.1fs" % el_one))
    return {"value": round(n / el_all, 4), "unit": "steps/s", "cores": int(blas_threads), "kind": "oracle",
            "single_thread": None if el_one is None else {"value": round(n / el_one, 4), "unit": "steps/s", "cores": 1},
            "sample": "%s; %d steps after 1 untimed step, then the next %d steps on one thread; hot set from one pre-sampling "
                      "epoch over the first %d batches; C parts (sampling, relabel, gather, aggregation) single-threaded, numpy "
                      "fp64 products on %d threads for `value`" % (where, n, n, pre_batches, blas_threads)}


if __name__ == "__main__":
    main()
