#!/usr/bin/env python3
"""Benchmark of one partition's SAT GCN training step on one MI355X.

A "step" is one pass of the whole hot path over one partition: predictor
inference for every hidden layer (reading the history ring in place), pull of
the static halo features, per layer aggregation + feature transform + push,
the cross-entropy gradient, and the backward pass. Inputs are seeded and
synthetic and are resident in HBM before the timed region starts.

Prints ONE JSON line. `value` is CSR entries aggregated per second over the
whole step (GTEPS), i.e. (entries walked by all aggregation calls of a step) /
(wall time of the step, every call included).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
# The dense products run on the bf16 MFMA pipe (2.5 PFLOP/s dense) with an exact
# three-way split of the fp32 operands: six bf16 products per fp32 product. Their
# algorithmic (fp32) flops are therefore priced against 2500 / 6 TFLOP/s.
MFMA_SPLIT_PEAK_TFLOPS = 2500.0 / 6.0

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE,
# scaled by a copy kernel of known size); filled in from the committed profile
# summaries, None where no counter run exists for that workload / kernel.
MEASURED_TRAFFIC_BYTES = {      # profiles/large_step_hbm_traffic.md, average over the class's launches
    ("large", "spmm"): 11.54e9,       # 4 launches of 12.71 GB (d = 256) and one of 6.86 GB (d = 100)
    ("large", "gather"): 1.064e9,
    ("large", "push"): 0.627e9,
    ("large", "dense_fwd"): 0.640e9,
    ("large", "dense_bwd"): 1.44e9,   # call level: weight-gradient product + its reduction + dAGG product
    ("large", "predict"): 7.68e9,     # call level: LSTM 3.52 + hop aggregation 1.24 + hop product 2.91
    ("large", "loss"): 0.136e9,
    # graph attention backbone, profiles/large_gat_step_hbm_traffic.md
    ("large", "gat_fwd"): 12.06e9,    # two launches of 16.02 GB (4 heads x 64) and one of 4.13 GB (1 x 47)
    ("large", "gat_scores"): 1.10e9,
    ("large", "gat_bwd"): 27.9e9,     # call level: mask 0.92 + destination side 16.06 + source side 12.83 + 5.88
                                      # + attention vectors 1.10 (last layer: 4.16 + 3.48 + 1.41 + 0.37)
}


KERNEL_OF_CLASS = {"spmm": "spmm_stream_kernel", "gather": "row_copy_vec_kernel (gather)",
                   "push": "row_copy_vec_kernel (scatter)", "dense_fwd": "mx::gemm_kernel",
                   "loss": "xent_grad_kernel", "gather_add": "row_gather_add_kernel",
                   "gat_fwd": "gat_fwd_kernel", "gat_scores": "gat_scores_kernel"}


class CallTimers:
    """HIP event pairs around every library call, on the stream the calls are
    enqueued on (torch's current stream), collected over the timed steps."""

    def __init__(self, torch, flush=None):
        self.torch = torch
        self.pairs = []
        self.enabled = False
        self.flush = flush      # optional: a buffer larger than every cache, rewritten
                                # before each call so that the call starts cold

    def record(self, name, fn):
        if self.flush is not None:
            self.flush.add_(1.0)
        if not self.enabled:
            fn()
            return
        a = self.torch.cuda.Event(enable_timing=True)
        b = self.torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        self.pairs.append((name, a, b))

    def summary(self):
        out = {}
        for name, a, b in self.pairs:
            out.setdefault(name, []).append(a.elapsed_time(b))
        return {k: dict(total_ms=sum(v), launches=len(v), avg_ms=sum(v) / len(v), min_ms=min(v),
                        median_ms=sorted(v)[len(v) // 2]) for k, v in out.items()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large", choices=["tiny", "medium", "dense", "large", "scale_small", "scale_rows_small", "scale"])
    ap.add_argument("--dtype", default=None, choices=["f32", "bf16"],
                    help="storage type of features, activations, history and weights "
                         "(default: the workload's own; sums are fp32 either way)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--unfused-pull", action="store_true",
                    help="assemble the predictor window with sat_history_gather first")
    ap.add_argument("--bypass", action="store_true", help="plain historical embeddings")
    ap.add_argument("--delta-t", type=int, default=1,
                    help="refresh the predicted halo embeddings every DELTA_T steps (Alg. 1's update "
                         "frequency); the default 1 predicts on every step")
    ap.add_argument("--predictor-train", action="store_true",
                    help="after the timed steps also time one training step (loss, gradients, "
                         "plain gradient update) of hidden layer 1's predictor; reported under "
                         "\"predictor_train\", outside the step time (it runs every Delta T steps)")
    ap.add_argument("--codec", type=int, default=None, metavar="DECIMALS",
                    help="after the timed steps also time the compression codec on the newest "
                         "history slot of hidden layer 1 at this many decimal places: plan + encode "
                         "of the partition's local + halo rows, decode of the halo rows through the "
                         "id list; reported under \"codec\"")
    ap.add_argument("--coded-ring", type=int, default=None, metavar="DECIMALS",
                    help="keep the history ring coded (compression codec at this many decimal "
                         "places) inside the step: the predictor's window is decoded from the "
                         "codes on every pull and every push codes the fresh rows; GCN backbone")
    ap.add_argument("--stale-grad", action="store_true",
                    help="also run the stale-gradient term of the backward: halo output of the "
                         "transpose aggregation pushed to a gradient table, table rows of the "
                         "local nodes added to their gradient")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also launch one plain row copy of known size (1 GiB read + 1 GiB "
                         "written, identity ids) so that a rocprofv3 --pmc run of this command "
                         "can scale FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--backbone", default="gcn", choices=["gcn", "gat"],
                    help="gcn: the normalised-adjacency aggregation (the headline); gat: the graph "
                         "attention backbone (edge softmax aggregation, three edge passes per layer)")
    ap.add_argument("--graph", action="store_true",
                    help="after the timed steps also replay the step from a HIP graph (one graph holds "
                         "tau consecutive steps) and report its time under \"graph\": for the workloads "
                         "whose step is bound by launch latency")
    ap.add_argument("--cold", action="store_true",
                    help="rewrite a 1 GiB buffer before every library call, so that no call finds "
                         "its inputs in the caches (for the workloads whose working set fits "
                         "them); ms_per_step is then the sum of the calls' own times")
    ap.add_argument("--quiet", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs one partition on ONE GPU; --gpus %d is not supported "
              "(no collectives, no sharding across GPUs in this library)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    if args.coded_ring is not None and (args.backbone != "gcn" or args.predictor_train
                                        or args.codec is not None or args.unfused_pull):
        print("bench.py: --coded-ring goes with the GCN backbone and without --predictor-train, "
              "--codec and --unfused-pull (they read the dense ring)", file=sys.stderr)
        sys.exit(2)

    def log(msg):
        if not args.quiet:
            print("[bench] " + msg, file=sys.stderr, flush=True)

    import numpy as np
    import torch
    import sat_synth as syn
    import paper_2308_13466_amd as sat
    from paper_2308_13466_amd.workload import build_workload
    sat.lib()   # raises if libsat.so has not been built; there is no fallback
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    flush = torch.zeros(1 << 28, dtype=torch.float32, device=dev) if args.cold else None
    timers = CallTimers(torch, flush)
    wl = build_workload(args.workload, bypass=args.bypass, fused_pull=not args.unfused_pull,
                        timers=timers, log=log, dtype=args.dtype, grad_tables=args.stale_grad,
                        predict_every=args.delta_t, backbone=args.backbone, coded_ring=args.coded_ring)
    gat = args.backbone == "gat"
    bf16 = wl.dtype == "bf16"
    cfg, g, view, step = wl.cfg, wl.graph, wl.view, wl.step
    dims, tau, d_s, L = wl.dims, wl.tau, wl.d_s, wl.L
    n_l, n_h = view["n_local"], view["n_halo"]
    n_bar = n_l + n_h

    if args.pmc_calibration:
        rows, width = 1 << 20, 256
        src = torch.ones((rows, width), dtype=torch.float32, device=dev)
        dst = torch.zeros((rows, width), dtype=torch.float32, device=dev)
        ident = torch.arange(rows, dtype=torch.int32, device=dev)
        sat.history_gather(src, rows, width, ident, rows, width, dst, width,
                           stream=torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        log("calibration copy: %d rows x %d floats (%.0f bytes read, same written)" % (
            rows, width, rows * width * 4.0))
        del src, dst, ident

    # ---- warm-up, then the timed region
    for _ in range(args.warmup):
        step.forward_backward()
    torch.cuda.synchronize()
    timers.enabled = True
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step.forward_backward()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    timers.enabled = False
    ms_per_step = 1e3 * elapsed / args.steps
    edges = step.edges_per_step()
    calls = timers.summary()
    if args.cold:       # the flushes sit between the calls: count the calls alone
        ms_per_step = sum(c["total_ms"] for c in calls.values()) / args.steps
    gteps = edges / (ms_per_step * 1e-3) / 1e9
    spmm_ms = sum(c["total_ms"] for k, c in calls.items()
                  if k.startswith(("spmm_", "gat_fwd_", "gat_bwd_"))) / args.steps
    loss = float(step.loss.item())
    log("ms/step %.3f  GTEPS %.2f  loss %.5f" % (ms_per_step, gteps, loss))
    coded_ring = None
    if wl.coded is not None:
        over = step.coded_overflow()
        assert not over, "a push did not fit its part of the coded ring: %r" % (over,)
        own = remote = dense = 0
        for l in range(1, L):
            for slot in wl.coded.slots[l]:
                o, r = slot.coded_bytes()
                own, remote = own + o, remote + r
                dense += n_bar * dims[l] * (2 if bf16 else 4)
        coded_ring = {"decimals": args.coded_ring, "coded_bytes_local_rows": own,
                      "coded_bytes_halo_rows": remote, "dense_ring_bytes": dense,
                      "ratio_vs_dense_ring": round(dense / max(1, own + remote), 3)}
        log("coded ring: %.3f GB of codes for a %.3f GB dense ring (%.2fx)" % (
            (own + remote) / 1e9, dense / 1e9, coded_ring["ratio_vs_dense_ring"]))

    # ---- per-kernel-class roofline figures (algorithmic bytes / flops per launch)
    s = 2 if bf16 else 4
    # dense MFMA peak the contractions are priced against: fp32 data is split into
    # three bf16 pieces (six products per element pair); bf16 data needs one product
    # in the feature transforms and two in the predictor (fp32 parameters to 16 bits, bf16 x)
    peak_dense = 2500.0 if bf16 else MFMA_SPLIT_PEAK_TFLOPS
    peak_predict = 2500.0 / 2.0 if bf16 else MFMA_SPLIT_PEAK_TFLOPS
    nnz, nnz_loc, nnz_halo = view["nnz"], step.nnz_local, view["nnz_halo"]

    def spmm_bytes(entries, rows, d):       # per entry: col + val + one feature row;
        return entries * (8 + d * s) + rows * (8 + d * s)   # per row: rowptr + output row

    classes = {}

    def add(cls, name, bound, work):
        if name not in calls:
            return
        c = classes.setdefault(cls, dict(bound=bound, work=0.0, ms=0.0, launches=0))
        c["work"] += work * calls[name]["launches"]
        c["ms"] += calls[name]["total_ms"]
        c["launches"] += calls[name]["launches"]

    for l in range(L):
        add("spmm", "spmm_fwd_l%d" % l, "hbm", spmm_bytes(nnz, n_l, dims[l]))
        if l >= 1:
            add("spmm", "spmm_bwd_l%d" % l, "hbm", spmm_bytes(nnz_loc, n_l, dims[l]) + (
                spmm_bytes(nnz_halo, n_h, dims[l]) if args.stale_grad else 0))
        if gat:      # the transform runs over local + halo rows; three edge passes per layer
            K = step.heads[l]
            dl = dims[l + 1]
            add("dense_fwd", "dense_fwd_l%d" % l, "mfma", 2.0 * n_bar * dims[l] * dl)
            add("dense_bwd", "dense_bwd_l%d" % l, "mfma", 2.0 * n_bar * dims[l] * dl)
            add("dense_bwd", "dense_bwd_in_l%d" % l, "mfma", 2.0 * n_l * dims[l] * dl)
            add("gat_scores", "gat_scores_l%d" % l, "hbm", n_bar * (dl * s + 4 * K) + n_l * 4 * K)
            add("gat_fwd", "gat_fwd_l%d" % l, "hbm",
                nnz * (4 + 4 * K + dl * s) + n_l * (8 + dl * s + 12 * K))
            add("gat_bwd", "gat_bwd_l%d" % l, "hbm",
                nnz * (4 + 4 * K + dl * s) + n_l * (8 + dl * s + 28 * K)          # destination side
                + nnz * (4 + 16 * K + dl * s) + n_bar * (8 + 2 * dl * s + 8 * K)  # source side
                + (3 * n_l * dl * s if l < L - 1 else 0)                          # masked gradient
                + n_bar * (dl * s + 4 * K) + n_l * 4 * K)                         # attention vectors
        else:
            add("dense_fwd", "dense_fwd_l%d" % l, "mfma", 2.0 * n_l * dims[l] * dims[l + 1])
            add("dense_bwd", "dense_bwd_l%d" % l, "mfma",
                (4.0 if l >= 1 else 2.0) * n_l * dims[l] * dims[l + 1])
        if l >= 1:
            if args.coded_ring is None:
                add("push", "push_l%d" % l, "hbm", n_l * (2 * dims[l] * s + 4))
            else:
                add("coded_push", "push_l%d" % l, "hbm", 2.0 * n_l * dims[l] * s)
            add("push", "grad_push_l%d" % l, "hbm", n_h * (2 * dims[l] * s + 4))
            add("gather_add", "grad_pull_l%d" % l, "hbm", n_l * (3 * dims[l] * s + 4))
            add("gather", "gather_l%d" % l, "hbm", n_bar * (2 * dims[l] * s + 4))
            # coded ring: a decode writes the dense rows (the codes it reads are the smaller
            # part and vary); a push reads the dense rows twice (sizes, then codes)
            add("coded_pull", "pull_l%d" % l, "hbm",
                n_h * dims[l] * s if args.bypass else n_bar * dims[l] * s / 2.0)   # two launches per slot
            if not args.bypass:
                flops = (2.0 * n_bar * 4 * d_s * (tau * dims[l] + (tau - 1) * d_s)
                         + 2.0 * nnz_halo * d_s + 2.0 * n_h * d_s * dims[l])
                add("predict", "predict_l%d" % l, "mfma", flops)
            else:
                add("gather", "predict_l%d" % l, "hbm", n_h * (2 * dims[l] * s + 4))
    add("gather", "gather_l0", "hbm", n_h * (2 * dims[0] * s + 4))
    add("loss", "loss_grad", "hbm", n_l * (2 * dims[L] * s + 4))

    roof_all = {}
    for cls, c in classes.items():
        sec = c["ms"] * 1e-3
        if c["bound"] == "hbm":
            ach, peak, unit = c["work"] / sec / 1e9, HBM_PEAK_GBS, "GB/s"
        else:
            ach, unit = c["work"] / sec / 1e12, "TFLOP/s"
            peak = round(peak_predict if cls == "predict" else peak_dense, 1)
        roof_all[cls] = dict(bound=c["bound"], achieved=round(ach, 2), peak=peak, unit=unit,
                             frac=round(ach / peak, 4),
                             avg_launch_ms=round(c["ms"] / c["launches"], 4),
                             ms_per_step=round(c["ms"] / args.steps, 4),
                             launches_per_step=c["launches"] // args.steps,
                             traffic=None if bf16 != (cfg.get("dtype") == "bf16") or (
                                 gat and not cls.startswith("gat_") and cls not in ("predict", "push", "loss")) or (
                                 args.coded_ring is not None and cls == "predict")
                             else MEASURED_TRAFFIC_BYTES.get((args.workload, cls)))
    # The dominant KERNEL: classes whose calls are one kernel each (aggregation, pull,
    # push, forward transform, loss) are kernels; "predict" and "dense_bwd" are calls
    # made of several kernels, none of which outweighs the aggregation kernel (see the
    # rocprofv3 kernel statistics under profiles/), so they are listed in
    # roofline_all at call level and not eligible here.
    single = [k for k in roof_all if k not in ("predict", "dense_bwd", "gat_bwd", "coded_pull", "coded_push")]
    dominant = max(single, key=lambda k: roof_all[k]["ms_per_step"])
    roofline = dict(kernel=KERNEL_OF_CLASS.get(dominant, dominant), **roof_all[dominant])

    # ---- optional: the same steps replayed from a HIP graph
    graph_info = None
    if args.graph:
        while step.t % step.graph_period() != 0:
            step.forward_backward()
        torch.cuda.synchronize()
        replay = step.capture()
        replay()
        torch.cuda.synchronize()
        reps = max(1, args.steps // replay.period)
        tg = time.perf_counter()
        for _ in range(reps):
            replay()
        torch.cuda.synchronize()
        g_ms = 1e3 * (time.perf_counter() - tg) / (reps * replay.period)
        graph_info = {"steps_per_replay": replay.period, "replays": reps, "ms_per_step": round(g_ms, 4),
                      "gteps": round(edges / (g_ms * 1e-3) / 1e9, 3), "loss": round(float(step.loss.item()), 6)}
        log("HIP graph replay: %.3f ms/step (eager %.3f)" % (g_ms, ms_per_step))

    # ---- optional: one training step of the predictor of hidden layer 1
    ptrain = None
    if args.predictor_train and not args.bypass and L >= 2:
        from paper_2308_13466_amd import binding as B
        l = 1
        wsb = B.predictor_train_workspace_bytes(n_l, n_h, dims[l], d_s, tau)
        ws = torch.empty((wsb + 3) // 4, dtype=torch.float32, device=dev)
        pw = step.predictors[l]
        keep_p = wl.device_keep[0][l - 1]
        grads = {k: torch.empty_like(keep_p[k]) for k in ("Wx", "Wh", "b", "Wg")}
        ploss = torch.zeros(1, dtype=torch.float32, device=dev)
        slots = [step.hist[l][sidx] for sidx in step.slot_order()]
        st_ptr = torch.cuda.current_stream().cuda_stream

        def train_once():
            B.predictor_grad(step.pv, pw, slots, slots[0].shape[0], slots[0].shape[1], step.table_ids,
                             step.Hbar[l], step.ld[l], None, grads["Wx"], grads["Wh"], grads["b"],
                             grads["Wg"], ploss, dtype=B.BF16 if bf16 else B.F32, workspace=ws,
                             workspace_bytes=wsb, stream=st_ptr)
            for k in grads:
                B.sgd_update(keep_p[k], grads[k], grads[k].numel(), 1e-3, stream=st_ptr)

        train_once()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 3
        e0.record()
        for _ in range(reps):
            train_once()
        e1.record()
        torch.cuda.synchronize()
        t_ms = e0.elapsed_time(e1) / reps
        fwd = 2.0 * n_bar * 4 * d_s * (tau * dims[l] + (tau - 1) * d_s) + 2.0 * nnz * d_s \
            + 2.0 * n_l * d_s * dims[l]
        bwd = 4.0 * n_l * d_s * dims[l] + 2.0 * nnz * d_s \
            + 2.0 * n_bar * 4 * d_s * (tau * dims[l] + 2 * (tau - 1) * d_s)
        ptrain = {"layer": l, "ms_per_training_step": round(t_ms, 4), "loss": round(float(ploss.item()), 6),
                  "flops": fwd + bwd, "achieved_tflops": round((fwd + bwd) / (t_ms * 1e-3) / 1e12, 2),
                  "workspace_gb": round(wsb / 1e9, 2),
                  "batch": "all %d local nodes" % n_l}
        log("predictor training step (layer %d): %.3f ms, loss %.6f" % (l, t_ms, ptrain["loss"]))
        del ws

    # ---- optional: compression codec on one history slot
    codec = None
    if args.codec is not None and L >= 2:
        from paper_2308_13466_amd import binding as B
        l, prec = 1, args.codec
        dt = B.BF16 if bf16 else B.F32
        st_ptr = torch.cuda.current_stream().cuda_stream
        # the rows a partition stores / pulls: its local + halo nodes, compact
        slot = step.hist[l][step.slot_order()[-1]]
        rows = torch.empty((n_bar, step.ld[l]), dtype=slot.dtype, device=dev)
        B.history_gather(slot, slot.shape[0], slot.shape[1], step.table_ids, n_bar, dims[l], rows,
                         step.ld[l], dtype=dt, stream=st_ptr)
        wsb = B.history_compress_workspace_bytes(n_bar)
        ws = torch.zeros(wsb // 8 + 1, dtype=torch.int64, device=dev)
        row_off = torch.zeros(n_bar + 1, dtype=torch.int64, device=dev)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        B.history_compress_plan(rows, step.ld[l], n_bar, dims[l], prec, row_off, dtype=dt,
                                workspace=ws, workspace_bytes=wsb, stream=st_ptr)
        torch.cuda.synchronize()
        total = int(row_off[-1].item())
        codes = torch.empty(total, dtype=torch.uint8, device=dev)
        out = torch.empty((n_h, step.ld[l]), dtype=slot.dtype, device=dev)
        halo_rows = torch.arange(n_l, n_bar, dtype=torch.int32, device=dev)
        reps = 5
        ev[0].record()
        for _ in range(reps):
            B.history_compress_plan(rows, step.ld[l], n_bar, dims[l], prec, row_off, dtype=dt,
                                    workspace=ws, workspace_bytes=wsb, stream=st_ptr)
            B.history_compress_encode(rows, step.ld[l], n_bar, dims[l], prec, row_off, codes, total,
                                      dtype=dt, stream=st_ptr)
        ev[1].record()
        for _ in range(reps):
            B.history_decompress(codes, row_off, n_bar, halo_rows, n_h, dims[l], prec, out, step.ld[l],
                                 dtype=dt, stream=st_ptr)
        ev[2].record()
        torch.cuda.synchronize()
        enc_ms, dec_ms = ev[0].elapsed_time(ev[1]) / reps, ev[1].elapsed_time(ev[2]) / reps
        dense = n_bar * dims[l] * s
        halo_coded = int((row_off[-1] - row_off[n_l]).item())
        codec = {"layer": l, "decimals": prec, "rows": n_bar, "coded_bytes": total,
                 "ratio_vs_stored": round(dense / max(total, 1), 3),
                 "encode_ms": round(enc_ms, 4),
                 "encode_gbs": round((2 * dense + total + 16 * n_bar) / (enc_ms * 1e-3) / 1e9, 1),
                 "decode_rows": n_h, "decode_ms": round(dec_ms, 4),
                 "decode_gbs": round((halo_coded + n_h * (dims[l] * s + 12)) / (dec_ms * 1e-3) / 1e9, 1)}
        log("codec (%d decimals): %.2fx, encode %.3f ms, decode of the halo rows %.3f ms" % (
            prec, codec["ratio_vs_stored"], enc_ms, dec_ms))
        del rows, codes, out, ws

    # ---- CPU oracle on a bounded sample, rank 0, host cores
    cpu = None
    if not args.no_cpu_baseline and wl.X_host is None:
        log("cpu oracle: skipped (this workload's inputs are drawn on the device)")
    elif not args.no_cpu_baseline and wl.coded is not None:
        log("cpu oracle: skipped (timed on the dense ring; run without --coded-ring)")
    elif not args.no_cpu_baseline:
        cpu = cpu_baseline(view, dims, tau, d_s, wl.X_host, wl.hist_host, wl.table_ids, wl.Ws,
                           wl.omegas, wl.y, edges, bypass=args.bypass, log=log,
                           gat_attn=wl.attn if gat else None)

    out = {
        "metric": "GTEPS aggregated (CSR entries aggregated per second over one partition's "
                  "SAT GCN step, fwd+bwd, predictor and history pull/push included)",
        "value": round(gteps, 3), "unit": "GTEPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": args.workload, "backbone": args.backbone, "graph": cfg["kind"], "N": g.N,
                   "partition": "%d of %d" % (cfg["part"], cfg["n_parts"]),
                   "n_local": n_l, "n_halo": n_h, "nnz": nnz, "nnz_local_local": nnz_loc,
                   "dims": dims, "tau": tau, "d_s": d_s,
                   "predictor": "bypass" if args.bypass else (
                       "every step" if args.delta_t <= 1 else "every %d steps" % args.delta_t),
                   "pull": "unfused" if args.unfused_pull else "fused into predict",
                   "stale_gradient_term": bool(args.stale_grad),
                   "history_ring": "dense" if args.coded_ring is None else "coded, %d decimals" % args.coded_ring,
                   "caches": "flushed before every call" if args.cold else "as the step leaves them",
                   "entries_per_step": edges},
        "ms_per_layer_step": round(ms_per_step / L, 4),
        "gteps_aggregation_calls_only": round(edges / (spmm_ms * 1e-3) / 1e9, 3) if spmm_ms else None,
        "ms_by_call": {k: round(v["total_ms"] / args.steps, 4) for k, v in sorted(calls.items())},
        "ms_by_call_min": {k: round(v["min_ms"], 4) for k, v in sorted(calls.items())},
        "ms_by_call_median": {k: round(v["median_ms"], 4) for k, v in sorted(calls.items())},
        "roofline": roofline,
        "roofline_all": roof_all,
        "cpu_baseline": cpu,
        "graph": graph_info,
        "predictor_train": ptrain,
        "codec": codec,
        "coded_ring": coded_ring,
        "loss": round(loss, 6),
    }
    print(json.dumps(out))


def cpu_baseline(view, dims, tau, d_s, X_host, hist_host, table_ids, Ws, omegas, y, edges,
                 bypass, log, sample_rows=65536, sample_nodes=524288, gat_attn=None):
    """Time the oracle (as it stands) on a row sample of every call of the step
    and extrapolate each call by rows_total / rows_sampled (rows of every call
    are independent of one another)."""
    import numpy as np
    from oracle import sat_oracle as orc
    try:
        from threadpoolctl import threadpool_limits
    except ImportError:                                   # pragma: no cover
        threadpool_limits = None
    L = len(dims) - 1
    n_l, n_h = view["n_local"], view["n_halo"]
    n_bar = n_l + n_h
    rng = np.random.default_rng(1234)
    rows = np.sort(rng.choice(n_l, size=min(sample_rows, n_l), replace=False))
    nodes = np.sort(rng.choice(n_bar, size=min(sample_nodes, n_bar), replace=False))
    halo = np.sort(rng.choice(n_h, size=min(sample_rows, n_h), replace=False)) if n_h else None
    f_rows, f_nodes = n_l / len(rows), n_bar / len(nodes)
    f_halo = (n_h / len(halo)) if n_h else 0.0

    def run():
        est = 0.0
        t_all = time.perf_counter()
        Hbars = [X_host[table_ids][:, :dims[0]]]
        for l in range(1, L):
            Hbars.append(hist_host[l][-1][table_ids][:, :dims[l]])   # stand-in activations
        prep = time.perf_counter() - t_all
        for l in range(1, L):
            if bypass:
                continue
            win = [hist_host[l][s][table_ids[nodes]][:, :dims[l]] for s in range(tau)]
            t0 = time.perf_counter()
            orc.lstm_last_hidden(win, omegas[l]["Wx"], omegas[l]["Wh"], omegas[l]["b"])
            est += (time.perf_counter() - t0) * f_nodes
            if n_h:
                sub = dict(view, n_halo=len(halo),
                           h_colptr=np.concatenate([[0], np.cumsum(
                               view["h_colptr"][halo + 1] - view["h_colptr"][halo])]),
                           h_row=np.concatenate([view["h_row"][view["h_colptr"][u]:view["h_colptr"][u + 1]]
                                                 for u in halo]),
                           h_val=np.concatenate([view["h_val"][view["h_colptr"][u]:view["h_colptr"][u + 1]]
                                                 for u in halo]),
                           h_self=view["h_self"][halo])
                S = np.zeros((n_l + len(halo), d_s), np.float32)
                t0 = time.perf_counter()
                orc.predictor_hop(sub, S, omegas[l]["Wg"])
                est += (time.perf_counter() - t0) * f_halo
        if gat_attn is not None:
            return est + run_gat(Hbars), prep
        g = None
        aggs = []
        for l in range(L):
            t0 = time.perf_counter()
            a = orc.spmm_fwd_rows(view, Hbars[l], rows)
            z, h = orc.dense_fwd(a, Ws[l], 1 if l < L - 1 else 0)
            est += (time.perf_counter() - t0) * f_rows
            aggs.append((a, z, h))
        t0 = time.perf_counter()
        _, g = orc.loss_and_grad(aggs[-1][2], y[rows])
        est += (time.perf_counter() - t0) * f_rows
        for l in range(L - 1, -1, -1):
            a, z, h = aggs[l]
            t0 = time.perf_counter()
            dW, dA, _ = orc.dense_bwd(g[:, :dims[l + 1]], z, a, Ws[l], 1 if l < L - 1 else 0)
            est += (time.perf_counter() - t0) * f_rows
            if l >= 1:
                dA_full = np.zeros((n_l, dims[l]), np.float32)      # stand-in upstream gradient
                dA_full[rows] = dA
                t0 = time.perf_counter()
                g = orc.spmm_bwd_rows(view, dA_full, rows)
                est += (time.perf_counter() - t0) * f_rows
        return est, prep

    def run_gat(Hbars):
        """The attention backbone's calls: transform and scores on the node sample,
        the edge passes on the row sample (stand-in values where a call needs the
        rows of all nodes: only the time matters here)."""
        from oracle import gat_oracle as gat
        est = 0.0
        srng = np.random.default_rng(4321)
        for l in range(L):
            a_dst, a_src = gat_attn[l]
            K = a_dst.shape[0]
            dl = dims[l + 1]
            t0 = time.perf_counter()
            Zs = Hbars[l][nodes].astype(np.float64) @ Ws[l].astype(np.float64)
            gat.gat_scores(Zs, a_dst, a_src)
            est += (time.perf_counter() - t0) * f_nodes
            Zfull = srng.standard_normal((n_bar, dl)).astype(np.float32).astype(np.float64)
            el = srng.standard_normal((n_l, K))
            er = srng.standard_normal((n_bar, K))
            dOUT = np.zeros((n_l, dl))
            dOUT[rows] = srng.standard_normal((len(rows), dl))
            t0 = time.perf_counter()
            gat.gat_aggregate_fwd(view, Zfull, el, er, 0.2, rows=rows)
            gat.gat_aggregate_bwd(view, Zfull, el, er, 0.2, dOUT, rows=rows)
            est += (time.perf_counter() - t0) * f_rows
            t0 = time.perf_counter()
            Hbars[l][nodes].astype(np.float64).T @ Zs                       # dW over local + halo rows
            est += (time.perf_counter() - t0) * f_nodes
            if l >= 1:
                t0 = time.perf_counter()
                dOUT[rows] @ Ws[l].astype(np.float64).T                     # dH_in over the local rows
                est += (time.perf_counter() - t0) * f_rows
        t0 = time.perf_counter()
        orc.loss_and_grad(srng.standard_normal((len(rows), dims[L])), y[rows])
        est += (time.perf_counter() - t0) * f_rows
        return est

    t0 = time.time()
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            est, prep = run()
        cores = 1
    else:
        est, prep = run()
        cores = os.cpu_count() or 1
    log("cpu oracle: estimated %.1f s per step on %d core(s) (sample run took %.1fs)" % (
        est, cores, time.time() - t0))
    return {"value": round(edges / est / 1e9, 6), "unit": "GTEPS", "cores": cores,
            "kind": "oracle",
            "sample": "%d of %d local rows per aggregation/transform call, %d of %d nodes for the "
                      "predictor LSTM, %d of %d halo rows for its hop; each call's time scaled by "
                      "rows_total/rows_sampled; estimated %.1f s per step" % (
                          len(rows), n_l, len(nodes), n_bar, 0 if halo is None else len(halo),
                          n_h, est)}


if __name__ == "__main__":
    main()
