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

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE, scaled by a
# copy kernel of known size): read from the data file that is written together with the
# counter summaries under profiles/. None where no counter run covers a workload / class.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_per_class.txt")


def measured_traffic():
    """{(workload, backbone, dtype, class): bytes per launch}. Lines: five whitespace-separated
    fields, '#' starts a comment."""
    table = {}
    if os.path.exists(TRAFFIC_FILE):
        for ln in open(TRAFFIC_FILE):
            f = ln.split("#")[0].split()
            if len(f) == 5:
                table[(f[0], f[1], f[2], f[3])] = float(f[4])
    return table


KERNEL_OF_CLASS = {"spmm": "spmm_stream_kernel (rows over 256 bytes) / spmm_slot_kernel (up to 256 bytes)", "gather": "row_copy_vec_kernel (gather)",
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
    ap.add_argument("--coded-chunk-rows", type=int, default=None, metavar="ROWS",
                    help="with --coded-ring: decode the predictor's window this many rows at a time "
                         "(dense scratch of tau * ROWS rows instead of tau * n_bar)")
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
    ap.add_argument("--gat-heads", type=int, default=4, choices=[1, 2, 4, 8],
                    help="heads of the hidden layers of the graph attention backbone")
    ap.add_argument("--graph", action="store_true",
                    help="after the timed steps also replay the step from a HIP graph (one graph holds "
                         "tau consecutive steps) and report its time under \"graph\": for the workloads "
                         "whose step is bound by launch latency")
    ap.add_argument("--cold", action="store_true",
                    help="rewrite a 1 GiB buffer before every library call, so that no call finds "
                         "its inputs in the caches (for the workloads whose working set fits "
                         "them); ms_per_step is then the sum of the calls' own times")
    ap.add_argument("--no-predict-ahead", action="store_true",
                    help="run the predictor's calls inside the step. By default (GCN backbone, dense "
                         "ring, fused pull) the predictions of step t + 1 are enqueued on a second "
                         "stream beside step t's backward: they only need the ring as step t's pushes "
                         "leave it; the results are bit-identical")
    ap.add_argument("--no-transform-first", action="store_true",
                    help="evaluate the last layer as (P Hbar) W like the others. By default it is "
                         "evaluated as P (Hbar W) when it narrows to half the width or less (the "
                         "appendix's Z = P H W fixes no order): the aggregation and its transpose then "
                         "gather rows of n_classes elements")
    ap.add_argument("--no-projection-cache", action="store_true",
                    help="multiply out the LSTM's input projection of every window slot on every "
                         "step. By default (when it fits 8 GiB) x Wx^T of a ring slot is kept and "
                         "read back on the steps where the slot is no longer the window's newest")
    ap.add_argument("--no-scale-leg", action="store_true",
                    help="do not append the full Scale configuration (bf16; run by a child process "
                         "after the headline workload has been timed) under the key \"scale\"")
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

    predict_ahead = not (args.no_predict_ahead or args.backbone != "gcn"
                         or args.unfused_pull or args.graph or args.cold or args.bypass)
    gat_flag = args.backbone == "gat"
    flush = torch.zeros(1 << 28, dtype=torch.float32, device=dev) if args.cold else None
    timers = CallTimers(torch, flush)
    wl = build_workload(args.workload, bypass=args.bypass, fused_pull=not args.unfused_pull,
                        timers=timers, log=log, dtype=args.dtype, grad_tables=args.stale_grad,
                        predict_every=args.delta_t, backbone=args.backbone, coded_ring=args.coded_ring,
                        coded_chunk_rows=args.coded_chunk_rows, gat_hidden_heads=args.gat_heads,
                        predict_ahead=predict_ahead,
                        transform_first=False if (args.no_transform_first or gat_flag) else "auto",
                        projection_cache=False if (args.no_projection_cache or args.predictor_train)
                        else "auto")
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

    # ---- CPU-baseline samples. Inputs that only exist on the device are read back now,
    # before any step overwrites a history slot; host copies are sampled after the timing.
    def fetch_rows(kind, l, slot, node_ids):
        tid = wl.table_ids[node_ids]
        if wl.X_host is not None:
            t = wl.X_host if kind == "X" else wl.hist_host[l][slot]
            return t[tid][:, :dims[l]]
        t = step.X_table if kind == "X" else step.hist[l][slot]
        idx = torch.from_numpy(tid.astype(np.int64)).to(dev)
        return t[idx][:, :dims[l]].float().cpu().numpy()

    want_cpu = not args.no_cpu_baseline and wl.coded is None
    cpu_prep = None
    if want_cpu and wl.X_host is None:
        cpu_prep = cpu_baseline_prepare(view, dims, tau, d_s, fetch_rows, wl.y, args.bypass, gat)
        log("cpu oracle: samples read back from the device in %.1fs" % cpu_prep["build_s"])

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

    def spmm_compulsory(entries, rows, distinct, d):
        # what the call cannot avoid moving: the index arrays once, every DISTINCT operand row
        # once (however often it is gathered), every output row once
        return 8 * entries + 8 * rows + distinct * d * s + rows * d * s

    def spmm_kernel(entries, rows, d):
        # the kernel instance the library's aggregation launcher picks for this shape
        # (labels the launches; the dispatch itself is csrc/spmm.hip's)
        row_bytes, nvec = d * s, (d * s + 15) // 16
        if nvec <= 32 and entries < 16 * rows:
            g = 1
            while g < nvec:
                g <<= 1
            return "spmm_group_kernel<%d,%d,4>" % (s, g)
        if row_bytes <= 256:
            return "spmm_slot_kernel<%d,%d,8>" % (s, 8 if row_bytes <= 128 else 16)
        if row_bytes <= 512:
            return "spmm_stream_kernel<%d,2,1,16>" % s
        if row_bytes <= 1024:
            return "spmm_stream_kernel<%d,4,1,16>" % s
        if row_bytes <= 2048 or s == 2:
            return "spmm_stream_kernel<%d,4,2,8>" % s
        return "spmm_stream_kernel<%d,4,%d,4>" % (s, 3 if row_bytes <= 3072 else 4)

    classes = {}

    def add(cls, name, bound, work, compulsory=None, kernel=None):
        if name not in calls:
            return
        for key in ((cls, kernel) if kernel else (cls,)):
            c = classes.setdefault(key, dict(bound=bound, work=0.0, ms=0.0, launches=0, compulsory=0.0))
            c["work"] += work * calls[name]["launches"]
            c["compulsory"] += (work if compulsory is None else compulsory) * calls[name]["launches"]
            c["ms"] += calls[name]["total_ms"]
            c["launches"] += calls[name]["launches"]

    tf = bool(getattr(step, "transform_first", False))
    for l in range(L):
        if tf and l == L - 1:
            # last layer as P (Hbar W): transform over all rows, both aggregations at n_classes
            # columns, the transpose one over local and halo entries (dW needs P_out^T dH too)
            C = dims[L]
            add("spmm", "spmm_fwd_l%d" % l, "hbm", spmm_bytes(nnz, n_l, C), spmm_compulsory(nnz, n_l, n_bar, C),
                kernel=spmm_kernel(nnz, n_l, C))
            # (two launches: the local block's transpose and the halo block's)
            add("spmm", "spmm_bwd_l%d" % l, "hbm", spmm_bytes(nnz_loc, n_l, C) + spmm_bytes(nnz_halo, n_h, C),
                spmm_compulsory(nnz_loc, n_l, n_l, C) + spmm_compulsory(nnz_halo, n_h, n_l, C))
            add("dense_fwd", "dense_fwd_l%d" % l, "mfma", 2.0 * n_bar * dims[l] * C)
            add("dense_bwd", "dense_bwd_l%d" % l, "mfma", 2.0 * n_bar * dims[l] * C)
            add("dense_bwd", "dense_bwd_in_l%d" % l, "mfma", 2.0 * n_l * dims[l] * C)
        else:
            add("spmm", "spmm_fwd_l%d" % l, "hbm", spmm_bytes(nnz, n_l, dims[l]),
                spmm_compulsory(nnz, n_l, n_bar, dims[l]), kernel=spmm_kernel(nnz, n_l, dims[l]))
        if l >= 1 and not (tf and l == L - 1):
            add("spmm", "spmm_bwd_l%d" % l, "hbm", spmm_bytes(nnz_loc, n_l, dims[l]) + (
                spmm_bytes(nnz_halo, n_h, dims[l]) if args.stale_grad else 0),
                spmm_compulsory(nnz_loc, n_l, n_l, dims[l]) + (
                    spmm_compulsory(nnz_halo, n_h, n_l, dims[l]) if args.stale_grad else 0),
                kernel=None if args.stale_grad else spmm_kernel(nnz_loc, n_l, dims[l]))
        if gat:      # the transform runs over local + halo rows; three edge passes per layer
            K = step.heads[l]
            dl = dims[l + 1]
            add("dense_fwd", "dense_fwd_l%d" % l, "mfma", 2.0 * n_bar * dims[l] * dl)
            add("dense_bwd", "dense_bwd_l%d" % l, "mfma", 2.0 * n_bar * dims[l] * dl)
            add("dense_bwd", "dense_bwd_in_l%d" % l, "mfma", 2.0 * n_l * dims[l] * dl)
            add("dense_bwd", "dense_bwd_halo_l%d" % l, "mfma", 2.0 * n_h * dims[l] * dl)   # (--stale-grad)
            add("gat_scores", "gat_scores_l%d" % l, "hbm", n_bar * (dl * s + 4 * K) + n_l * 4 * K)
            add("gat_fwd", "gat_fwd_l%d" % l, "hbm",
                nnz * (4 + 4 * K + dl * s) + n_l * (8 + dl * s + 12 * K))
            add("gat_bwd", "gat_bwd_l%d" % l, "hbm",
                nnz * (4 + 4 * K + dl * s) + n_l * (8 + dl * s + 28 * K)          # destination side
                + nnz * (4 + 16 * K + dl * s) + n_bar * (8 + 2 * dl * s + 8 * K)  # source side
                + (3 * n_l * dl * s if l < L - 1 else 0)                          # masked gradient
                + n_bar * (dl * s + 4 * K) + n_l * 4 * K)                         # attention vectors
        elif not (tf and l == L - 1):
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
    traffic_table = measured_traffic()
    for cls, c in classes.items():
        sec = c["ms"] * 1e-3
        if c["bound"] == "hbm":
            ach, peak, unit = c["work"] / sec / 1e9, HBM_PEAK_GBS, "GB/s"
        else:
            ach, unit = c["work"] / sec / 1e12, "TFLOP/s"
            peak = round(peak_predict if cls == "predict" else peak_dense, 1)
        # measured bytes exist for the plain configuration of a workload only
        plain_cfg = (args.coded_ring is None and not args.stale_grad and not args.bypass
                     and not args.unfused_pull and not args.no_transform_first
                     and (gat or not args.no_projection_cache))
        traffic = traffic_table.get((args.workload, args.backbone, wl.dtype, cls)) if plain_cfg else None
        roof_all[cls] = dict(bound=c["bound"], achieved=round(ach, 2), peak=peak, unit=unit,
                             frac=round(ach / peak, 4),
                             avg_launch_ms=round(c["ms"] / c["launches"], 4),
                             ms_per_step=round(c["ms"] / args.steps, 4),
                             launches_per_step=c["launches"] // args.steps,
                             traffic=traffic)
        if cls == "spmm" or cls.startswith("spmm_"):
            # Three readings of the same launches. `frac` prices what the lanes REQUEST (a row
            # per entry): re-gathered rows that a cache serves count as if they came from HBM,
            # so it is an upper bound on the HBM fraction and can pass 1. The measured one
            # divides the bytes that crossed the L2-to-fabric interface (rocprofv3 counters) by
            # the same time. The compulsory one counts every distinct row once.
            r = roof_all[cls]
            r["model"] = "gather traffic: per entry 8 B of indices + one operand row of d*s B; per row 8 B + one output row"
            r["frac_gather_model"] = r["frac"]
            r["frac_measured_traffic"] = (round(traffic * c["launches"] / sec / 1e9 / HBM_PEAK_GBS, 4)
                                          if traffic else None)
            r["compulsory_bytes"] = round(c["compulsory"] / c["launches"])
            r["frac_compulsory"] = round(c["compulsory"] / sec / 1e9 / HBM_PEAK_GBS, 4)
            r["traffic_over_compulsory"] = round(traffic * c["launches"] / c["compulsory"], 2) if traffic else None
    # The dominant KERNEL: classes whose calls are one kernel each (aggregation, pull,
    # push, forward transform, loss) are kernels; "predict" and "dense_bwd" are calls
    # made of several kernels, none of which outweighs the aggregation kernel (see the
    # rocprofv3 kernel statistics under profiles/), so they are listed in
    # roofline_all at call level and not eligible here.
    # The aggregation launches are listed twice: all together ("spmm") and by kernel instance
    # (the keys that name one); the dominant kernel is chosen among the instances.
    single = [k for k in roof_all if k not in ("spmm", "predict", "dense_bwd", "gat_bwd", "coded_pull", "coded_push")]
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

    # ---- CPU oracle on a bounded sample, rank 0, host cores (one core, then all of them)
    cpu = None
    if not args.no_cpu_baseline and wl.coded is not None:
        log("cpu oracle: skipped (timed on the dense ring; run without --coded-ring)")
    elif want_cpu:
        if cpu_prep is None:
            cpu_prep = cpu_baseline_prepare(view, dims, tau, d_s, fetch_rows, wl.y, args.bypass, gat)
        cpu = cpu_baseline_run(cpu_prep, wl.Ws, wl.omegas, wl.attn if gat else None, edges, log)
        cpu_prep = None

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
                   "predictions": "one step ahead, on a second stream" if predict_ahead else "in the step",
                   "last_layer": "P (Hbar W)" if tf else "(P Hbar) W",
                   "lstm_input_projection": "kept per ring slot" if getattr(step, "proj", None) is not None
                   else "multiplied out every step",
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
        "scale": None,
        "graph": graph_info,
        "predictor_train": ptrain,
        "codec": codec,
        "coded_ring": coded_ring,
        "loss": round(loss, 6),
    }
    # ---- the Scale configuration (bf16 by its own definition) in a child process of its own,
    # after everything of the headline workload has been measured and its memory released;
    # whatever happens to the child, the line below is printed
    plain = (not gat and args.coded_ring is None and not args.cold and not args.pmc_calibration
             and not args.stale_grad and not args.bypass and not args.predictor_train
             and args.codec is None and not args.graph and args.dtype is None and not args.no_predict_ahead)
    if args.workload == "large" and not args.no_scale_leg and plain:
        import gc
        del wl, step, timers, cpu_prep
        gc.collect()
        torch.cuda.empty_cache()
        try:
            out["scale"] = scale_leg(log)
        except Exception as e:                       # noqa: BLE001 - the headline must still print
            out["scale"] = {"error": "%s: %s" % (type(e).__name__, e)}
    print(json.dumps(out))


def scale_leg(log, steps=5, warmup=2, timeout_s=600):
    """Runs `bench.py --workload scale` (13.9 M local nodes, 412 M CSR entries, bf16 storage,
    195 GB of HBM) in a fresh child process and returns the parts of its JSON line that
    describe the measurement. The child logs to this process's stderr."""
    import subprocess
    cmd = [sys.executable, os.path.abspath(__file__), "--workload", "scale", "--steps", str(steps),
           "--warmup", str(warmup), "--no-scale-leg"]
    log("scale leg: %s" % " ".join(cmd[1:]))
    t0 = time.time()
    try:
        r = subprocess.run(cmd, stdout=subprocess.PIPE, text=True, timeout=timeout_s)
    except subprocess.TimeoutExpired:
        return {"error": "the child did not finish within %d s" % timeout_s}
    lines = [ln for ln in r.stdout.splitlines() if ln.startswith("{")]
    if r.returncode != 0 or not lines:
        return {"error": "the child exited with status %d and %d result lines" % (r.returncode, len(lines))}
    j = json.loads(lines[-1])
    keep = ("value", "unit", "ms_per_step", "steps", "warmup", "dtype", "data", "config", "ms_per_layer_step",
            "gteps_aggregation_calls_only", "ms_by_call", "roofline", "roofline_all", "cpu_baseline", "loss")
    res = {k: j.get(k) for k in keep}
    res["child_wall_s"] = round(time.time() - t0, 1)
    return res


# --------------------------------------------------------------------------
# CPU baseline: the oracle as it stands, timed on a bounded sample of the step.
# Rows of every call are independent of one another, so a call is timed on a sample of
# its rows and scaled by rows_total / rows_sampled. A "pack" holds everything the oracle
# needs for one shard of the sample, in compact numbering (the oracle's functions take
# any view; nothing in them is changed or specialised for this).
# --------------------------------------------------------------------------
def _build_pack(view, dims, tau, d_s, fetch, y, rows, nodes, halo, bypass, gat):
    """rows: sampled local rows (aggregation, transform, loss, backward); nodes: sampled
    local + halo nodes (predictor LSTM); halo: sampled halo nodes (predictor hop), or None.
    fetch(kind, l, s, node_ids) -> float32 rows of the layer-l input of those nodes in
    local-then-halo numbering: kind "X" the features, "hist" slot s of hidden layer l."""
    import numpy as np
    L = len(dims) - 1
    n_l = view["n_local"]
    rp, sp = view["rowptr"], view["split"]
    segs = [(int(rp[i]), int(rp[i + 1])) for i in rows]
    cols = np.concatenate([view["col"][a:b] for a, b in segs]) if segs else np.zeros(0, np.int32)
    uniq, inv = np.unique(np.concatenate([cols, rows.astype(cols.dtype)]), return_inverse=True)
    lens = np.array([b - a for a, b in segs], dtype=np.int64)
    m_rowptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    pack = dict(L=L, dims=list(dims), tau=tau, d_s=d_s, bypass=bypass, gat=gat,
                n_rows=len(rows), n_nodes=len(nodes), n_halo=0 if halo is None else len(halo),
                mini=dict(n_local=len(rows), n_halo=len(uniq), rowptr=m_rowptr,
                          split=m_rowptr[:-1] + np.array([int(sp[i]) - a for i, (a, b) in zip(rows, segs)],
                                                          dtype=np.int64),
                          col=inv[:len(cols)].astype(np.int32),
                          val=np.concatenate([view["val"][a:b] for a, b in segs])),
                own=inv[len(cols):].astype(np.int64),          # compact column id of each sampled row itself
                y=np.asarray(y)[rows],
                # stand-in activations of the hidden layers: the newest history slot
                Hb=[fetch("X", 0, 0, uniq)] + [fetch("hist", l, tau - 1, uniq) for l in range(1, L)])
    if not bypass:
        pack["win"] = [None] + [[fetch("hist", l, s, nodes) for s in range(tau)] for l in range(1, L)]
        if halo is not None and len(halo):
            cp = view["h_colptr"]
            nb = [view["h_row"][cp[u]:cp[u + 1]] for u in halo]
            locs, hinv = np.unique(np.concatenate(nb), return_inverse=True)
            pack["hop"] = dict(n_local=len(locs), n_halo=len(halo),
                               h_colptr=np.concatenate([[0], np.cumsum([len(x) for x in nb])]).astype(np.int64),
                               h_row=hinv.astype(np.int32),
                               h_val=np.concatenate([view["h_val"][cp[u]:cp[u + 1]] for u in halo]),
                               h_self=view["h_self"][halo])
    return pack


def _oracle_pack_seconds(args):
    """Runs the step's oracle calls on one pack; returns seconds per class of sampled unit
    ("rows", "nodes", "halo"). Top level so that a spawned worker can import it."""
    pack, Ws, omegas, gat_attn, blas_threads = args
    try:
        from threadpoolctl import threadpool_limits
    except ImportError:                                   # pragma: no cover
        return _pack_seconds(pack, Ws, omegas, gat_attn)
    with threadpool_limits(limits=blas_threads):
        return _pack_seconds(pack, Ws, omegas, gat_attn)


def _pack_seconds(pack, Ws, omegas, gat_attn):
    import numpy as np
    from oracle import sat_oracle as orc
    L, dims, tau, d_s = pack["L"], pack["dims"], pack["tau"], pack["d_s"]
    mini, Hb, yy = pack["mini"], pack["Hb"], pack["y"]
    ar = np.arange(pack["n_rows"])
    sec = dict(rows=0.0, nodes=0.0, halo=0.0)
    for l in range(1, L):
        if pack["bypass"]:
            continue
        t0 = time.perf_counter()
        orc.lstm_last_hidden(pack["win"][l], omegas[l]["Wx"], omegas[l]["Wh"], omegas[l]["b"])
        sec["nodes"] += time.perf_counter() - t0
        if "hop" in pack:
            hop = pack["hop"]
            S = np.zeros((hop["n_local"] + hop["n_halo"], d_s), np.float32)
            t0 = time.perf_counter()
            orc.predictor_hop(hop, S, omegas[l]["Wg"])
            sec["halo"] += time.perf_counter() - t0
    if pack["gat"]:
        from oracle import gat_oracle as gat
        srng = np.random.default_rng(4321)
        n_u = mini["n_halo"]
        for l in range(L):
            a_dst, a_src = gat_attn[l]
            K, dl = a_dst.shape[0], dims[l + 1]
            xs = pack["win"][l][-1] if (l >= 1 and not pack["bypass"]) else Hb[l][:pack["n_nodes"]]
            t0 = time.perf_counter()                                   # transform and scores: per node
            Zs = np.asarray(xs, np.float64) @ np.asarray(Ws[l], np.float64)
            gat.gat_scores(Zs, a_dst, a_src)
            np.asarray(xs, np.float64).T @ Zs                          # dW over local + halo rows
            sec["nodes"] += (time.perf_counter() - t0) * (pack["n_nodes"] / max(1, len(xs)))
            Z = srng.standard_normal((pack["n_rows"] + n_u, dl))       # stand-in values: only the time matters
            el = srng.standard_normal((pack["n_rows"], K))
            er = srng.standard_normal((pack["n_rows"] + n_u, K))
            dOUT = srng.standard_normal((pack["n_rows"], dl))
            t0 = time.perf_counter()                                   # the edge passes: per row
            gat.gat_aggregate_fwd(mini, Z, el, er, 0.2, rows=ar)
            gat.gat_aggregate_bwd(mini, Z, el, er, 0.2, dOUT, rows=ar)
            if l >= 1:
                dOUT @ np.asarray(Ws[l], np.float64).T                 # dH_in over the local rows
            sec["rows"] += time.perf_counter() - t0
        t0 = time.perf_counter()
        orc.loss_and_grad(srng.standard_normal((pack["n_rows"], dims[L])), yy)
        sec["rows"] += time.perf_counter() - t0
    else:
        t_rows = time.perf_counter()
        aggs = []
        for l in range(L):
            a = orc.spmm_fwd_rows(mini, Hb[l], ar)
            z, h = orc.dense_fwd(a, Ws[l], 1 if l < L - 1 else 0)
            aggs.append((a, z, h))
        _, g = orc.loss_and_grad(aggs[-1][2], yy)
        for l in range(L - 1, -1, -1):
            a, z, h = aggs[l]
            dW, dA, _ = orc.dense_bwd(g[:, :dims[l + 1]], z, a, Ws[l], 1 if l < L - 1 else 0)
            if l >= 1:
                G = np.zeros((mini["n_halo"], dims[l]), np.float32)   # stand-in upstream gradient
                G[pack["own"]] = dA
                g = orc.spmm_bwd_rows(mini, G, ar)
        sec["rows"] += time.perf_counter() - t_rows
    return sec


def host_cores():
    """Cores this process may use: its affinity mask, capped by OMP_NUM_THREADS when the
    environment sets it (a GPU machine gives one job a share of a larger machine)."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:                                 # pragma: no cover
        n = os.cpu_count() or 1
    cap = os.environ.get("OMP_NUM_THREADS", "")
    if cap.isdigit() and int(cap) > 0:
        n = min(n, int(cap))
    return max(1, n)


def cpu_baseline_prepare(view, dims, tau, d_s, fetch, y, bypass, gat, sample_rows=65536,
                         sample_nodes=524288, all_cores=True):
    """Draws the samples and builds the packs: one for the one-core run and one per core for
    the all-cores run. Done before the timed steps when the inputs only exist on the device
    (the rows are read back while the tables still hold what was drawn)."""
    import numpy as np
    n_l, n_h = view["n_local"], view["n_halo"]
    n_bar = n_l + n_h
    rng = np.random.default_rng(1234)

    def draw(k_rows, k_nodes):
        rows = np.sort(rng.choice(n_l, size=min(k_rows, n_l), replace=False))
        nodes = np.sort(rng.choice(n_bar, size=min(k_nodes, n_bar), replace=False))
        halo = np.sort(rng.choice(n_h, size=min(k_rows, n_h), replace=False)) if n_h else None
        return _build_pack(view, dims, tau, d_s, fetch, y, rows, nodes, halo, bypass, gat)

    t0 = time.time()
    prep = dict(one=draw(sample_rows, sample_nodes), many=[], totals=dict(rows=n_l, nodes=n_bar, halo=n_h))
    cores = host_cores()
    if all_cores and cores > 1:
        per_rows, per_nodes = max(256, sample_rows // (4 * cores)), max(2048, sample_nodes // (4 * cores))
        prep["many"] = [draw(per_rows, per_nodes) for _ in range(cores)]
    prep["build_s"] = time.time() - t0
    return prep


def cpu_baseline_run(prep, Ws, omegas, gat_attn, edges, log):
    """Times the oracle (as it stands) twice on row samples of every call of the step: on
    ONE core (one pack, BLAS held to one thread) and on ALL host cores (one pack per core,
    each in a worker process of its own started as a fresh interpreter, BLAS held to one
    thread per worker; the wall time of a class of calls is that of the slowest worker).
    Every call's time is scaled by rows_total / rows_sampled."""
    tot = prep["totals"]

    def estimate(sec, pack, shards):
        got = {"rows": pack["n_rows"], "nodes": pack["n_nodes"], "halo": pack["n_halo"]}
        return sum(sec[c] * tot[c] / (got[c] * shards) for c in sec if got[c])

    pack = prep["one"]
    sec1 = _oracle_pack_seconds((pack, Ws, omegas, gat_attn, 1))
    est1 = estimate(sec1, pack, 1)
    log("cpu oracle: estimated %.1f s per step on 1 core (samples built in %.1fs, run in %.1fs)" % (
        est1, prep["build_s"], sum(sec1.values())))
    out = {"value": round(edges / est1 / 1e9, 6), "unit": "GTEPS", "cores": 1, "kind": "oracle",
           "sample": "%d of %d local rows per aggregation/transform call, %d of %d nodes for the "
                     "predictor LSTM, %d of %d halo rows for its hop; each call's time scaled by "
                     "rows_total/rows_sampled; estimated %.1f s per step" % (
                         pack["n_rows"], tot["rows"], pack["n_nodes"], tot["nodes"], pack["n_halo"],
                         tot["halo"], est1)}
    packs = prep["many"]
    if packs:
        import multiprocessing as mp
        from concurrent.futures import ProcessPoolExecutor
        t0 = time.time()
        cores = len(packs)
        ctx = mp.get_context("spawn")          # fresh interpreters: the workers never see the GPU
        try:                                   # (a worker that dies breaks the pool: no endless respawn)
            with ProcessPoolExecutor(max_workers=cores, mp_context=ctx) as pool:
                futs = [pool.submit(_oracle_pack_seconds, (p, Ws, omegas, gat_attn, 1)) for p in packs]
                secs = [f.result(timeout=600) for f in futs]
        except Exception as e:                 # noqa: BLE001 - the one-core figure still stands
            log("cpu oracle on all cores failed: %s: %s" % (type(e).__name__, e))
            out["all_cores"] = {"error": "%s: %s" % (type(e).__name__, e)}
            return out
        worst = {c: max(sk[c] for sk in secs) for c in secs[0]}
        estN = estimate(worst, packs[0], cores)
        log("cpu oracle: estimated %.1f s per step on %d cores (%d worker processes, %.1fs in all)" % (
            estN, cores, cores, time.time() - t0))
        out["all_cores"] = {
            "value": round(edges / estN / 1e9, 6), "unit": "GTEPS", "cores": cores, "kind": "oracle",
            "sample": "%d worker processes, each %d local rows, %d nodes and %d halo rows of its own; a "
                      "class of calls takes the slowest worker's time, scaled by rows_total/(rows per "
                      "worker x workers); estimated %.1f s per step" % (
                          cores, packs[0]["n_rows"], packs[0]["n_nodes"], packs[0]["n_halo"], estN)}
    return out


if __name__ == "__main__":
    main()
