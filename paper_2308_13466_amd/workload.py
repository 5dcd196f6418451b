"""Seeded synthetic workloads resident in HBM, shared by bench.py and the
full-size parity tests so that both run the same launch configuration.

Nothing of the method is computed here: inputs come from sat_synth, the
partition view from the library's own host call, and the result is a
PartitionStep ready to run.
"""
import time

import numpy as np
import torch

import sat_synth as syn
from . import binding as B
from .step import CodedRing, CodedSlot, PartitionStep, encode_rows


def ld_of(d, mult=32):
    return (d + mult - 1) // mult * mult


class Workload:
    pass


def _upload(a, bf16, dev):
    """Host fp32 matrix -> device tensor; in bf16 mode the values are rounded to
    bfloat16 on the host (a storage conversion) and the 16-bit patterns uploaded.
    Returns (device tensor, host fp32 array holding exactly the uploaded values)."""
    if not bf16:
        return torch.from_numpy(a).to(dev), a
    bits = syn.bf16_bits_from_f32(a)
    t = torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
    return t, syn.f32_from_bf16_bits(bits)


def build_workload(name, bypass=False, fused_pull=True, timers=None, log=lambda m: None,
                   keep_host=True, device="cuda:0", dtype=None, grad_tables=False, predict_every=1,
                   backbone="gcn", coded_ring=None, own_headroom=1.5, predict_ahead=False,
                   transform_first="auto", projection_cache="auto", coded_chunk_rows=None,
                   gat_hidden_heads=4):
    """Generate workload `name` (see sat_synth.configs) and put it on the GPU.

    grad_tables: also allocate a pair of zeroed gradient tables per hidden layer (shape
    of the history tables) and run the stale-gradient term of the backward.
    backbone: "gcn" (normalised-adjacency aggregation) or "gat" (graph attention; heads per
    layer from sat_synth.gat_heads, attention vectors from sat_synth.attention_vectors_f32).
    coded_ring: None, or the number of decimals: the history ring is kept coded. Every dense
    slot generated below is coded once - the local nodes' rows into the
    `own` part (allocated own_headroom times the size they need now, since later pushes have
    other sizes), the halo nodes' rows into the `remote` part (exact size) - and then freed.
    transform_first: see PartitionStep ("auto": the last layer is evaluated as P (Hbar W)
    when it narrows to half the width or less).
    coded_chunk_rows: see PartitionStep (with coded_ring: rows of the window decoded at a time).
    projection_cache: see PartitionStep ("auto": when the matrices of all slots and hidden
    layers together stay under 8 GiB - the full Scale configuration would need 137 GB - and
    the tables are not bf16 rows the library's registers-only LSTM kernel serves).
    dtype: "f32" or "bf16" (default: the configuration's own). In bf16 mode the
    host copies kept for the tests hold the rounded values the device holds.

    History tables hold the seeded stand-in described in sat_synth.tensors
    (true unpartitioned embeddings are only affordable for the small
    workloads, where the tests build them with the oracle instead).
    """
    dev = torch.device(device)
    cfg = syn.get_config(name)
    dims, tau, d_s = cfg["dims"], cfg["tau"], cfg["d_s"]
    dtype = dtype or cfg.get("dtype", "f32")
    bf16 = dtype == "bf16"
    L = len(dims) - 1
    ss = syn.substreams(cfg["seed"])
    t0 = time.time()
    device_inputs = bool(cfg.get("device_inputs"))
    if device_inputs:     # too large to be worth a disk cache
        g = syn.make_graph(cfg, np.random.Generator(np.random.PCG64(ss["graph"])))
    else:
        g = syn.cached_graph(cfg, ss["graph"])
    log("graph: N=%d nnz=%d (%.1fs)" % (g.N, g.nnz, time.time() - t0))
    wss = ss["weights"].spawn(L)
    Ws = [syn.glorot_uniform_f32(wss[l], dims[l], dims[l + 1]) for l in range(L)]
    pss = ss["predictor"].spawn(L)
    omegas = [None] + [syn.predictor_params_f32(pss[l], dims[l], d_s) for l in range(1, L)]

    t0 = time.time()
    view = B.partition_view_build(g.N, g.rowptr, g.col, g.part, cfg["part"], g_deg=g.deg)
    n_l, n_h = view["n_local"], view["n_halo"]
    log("partition view: n_local=%d n_halo=%d nnz=%d nnz_halo=%d max_deg=%d (%.1fs)" % (
        n_l, n_h, view["nnz"], view["nnz_halo"],
        int(np.diff(view["rowptr"]).max()) if n_l else 0, time.time() - t0))

    t0 = time.time()
    ld = [ld_of(d) for d in dims]
    n_bar = n_l + n_h
    relabelled = cfg.get("tables") == "relabelled"
    # table row of every local-then-halo node: its global id, or (tables = "relabelled":
    # tables that hold the partition's local + halo rows only) its relabelled id
    if relabelled:
        table_ids = np.arange(n_bar, dtype=np.int32)
        n_table = n_bar
    else:
        table_ids = np.concatenate([view["local_ids"], view["halo_ids"]]).astype(np.int32)
        n_table = g.N
    hss = ss["history"].spawn(L)
    hist_d, hist_host = [None], [None]
    if device_inputs:
        # drawn on the device; tests read back the rows they need before the first step
        seeds = np.random.Generator(np.random.PCG64(ss["features"])).integers(0, 2**31 - 1, size=L)
        X_d, X_host = syn.device_normal(n_table, dims[0], ld[0], seeds[0], dev, bf16), None
        for l in range(1, L):
            hist_d.append(syn.device_history_standin(n_table, dims[l], ld[l], tau, cfg["noise_std"],
                                                     seeds[l], dev, bf16))
            hist_host.append(None)
    else:
        X_host = syn.normal_f32(ss["features"], n_table, dims[0], ld=ld[0])
        X_d, X_host = _upload(X_host, bf16, dev)
        for l in range(1, L):
            slots = syn.history_standin_f32(hss[l], n_table, dims[l], tau, cfg["noise_std"], ld=ld[l])
            up = [_upload(s, bf16, dev) for s in slots]
            del slots
            hist_d.append([u[0] for u in up])
            hist_host.append([u[1] for u in up] if keep_host else None)
            del up
    ids_d = torch.from_numpy(table_ids).to(dev)
    Ws_d = []
    for l in range(L):
        w = np.zeros((dims[l], ld_of(dims[l + 1], 8 if bf16 else 4)), np.float32)
        w[:, :dims[l + 1]] = Ws[l]
        w_d, w_host = _upload(w, bf16, dev)
        Ws_d.append(w_d)
        Ws[l] = w_host[:, :dims[l + 1]]
    preds, keep = [None], []
    for l in range(1, L):
        pd = {k: torch.from_numpy(omegas[l][k]).to(dev) for k in omegas[l]}
        keep.append(pd)
        preds.append(B.Predictor(pd["Wx"], pd["Wh"], pd["b"], pd["Wg"], dims[l], d_s, tau,
                                 bypass=bypass))
    y = syn.labels_i32(ss["labels"], n_l, dims[-1])
    y_d = torch.from_numpy(y).to(dev)
    gt = None
    if grad_tables:
        gt = [None] + [[torch.zeros_like(hist_d[l][0]) for _ in range(2)] for l in range(1, L)]
    coded = None
    if coded_ring is not None:
        dt = B.BF16 if bf16 else B.F32
        st = torch.cuda.current_stream().cuda_stream
        cslots = [None]
        for l in range(1, L):
            dense = torch.zeros((n_bar, ld[l]), dtype=hist_d[l][0].dtype, device=dev)
            layer = []
            for s in range(tau):
                tab = hist_d[l][s]
                B.history_gather(tab, tab.shape[0], tab.shape[1], ids_d, n_bar, dims[l], dense, ld[l],
                                 dtype=dt, stream=st)
                oc, oo = encode_rows(dense, ld[l], n_l, dims[l], coded_ring, dt, headroom=own_headroom,
                                     stream=st)
                rc, ro = encode_rows(dense[n_l:], ld[l], n_h, dims[l], coded_ring, dt, stream=st)
                layer.append(CodedSlot(oc, oo, rc, ro))
                hist_d[l][s] = None
                del tab
            cslots.append(layer)
            del dense
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        coded = CodedRing(coded_ring, cslots)
    attn = None
    if projection_cache == "auto":
        # (bf16 rows of 256 elements with d_s = 64 and enough nodes: the library's LSTM kernel
        # for that case, all weights in registers, is faster without kept projections than
        # the one that reads them)
        regs_only = bf16 and d_s == 64 and n_bar >= 32768 and all(dims[l] == 256 for l in range(1, L))
        projection_cache = (not bypass and coded is None and fused_pull and d_s <= 64 and not regs_only
                            and (L - 1) * tau * n_bar * 16 * d_s <= (8 << 30))
    if backbone == "gat":
        from .step_gat import GatPartitionStep
        heads = syn.gat_heads(dims, gat_hidden_heads)
        ass = ss["misc"].spawn(L)
        attn = [syn.attention_vectors_f32(ass[l], heads[l], dims[l + 1] // heads[l]) for l in range(L)]
        attn_d = [(torch.from_numpy(a.reshape(-1)).to(dev), torch.from_numpy(b.reshape(-1)).to(dev),
                   heads[l]) for l, (a, b) in enumerate(attn)]
        step = GatPartitionStep(view, dims, X_d, hist_d, ids_d, Ws_d, attn_d, preds, y_d, tau,
                                timers=timers, dtype=B.BF16 if bf16 else B.F32,
                                predict_every=predict_every, grad_tables=gt, coded=coded,
                                coded_chunk_rows=coded_chunk_rows,
                                projection_cache=bool(projection_cache) and coded is None)
    else:
        step = PartitionStep(view, dims, X_d, hist_d, ids_d, Ws_d, preds, y_d, tau,
                             fused_pull=fused_pull, timers=timers, dtype=B.BF16 if bf16 else B.F32,
                             grad_tables=gt, predict_every=predict_every, coded=coded,
                             predict_ahead=predict_ahead, transform_first=transform_first,
                             projection_cache=bool(projection_cache) and coded is None and fused_pull,
                             coded_chunk_rows=coded_chunk_rows)
    torch.cuda.synchronize()
    log("inputs resident in HBM: %.2f GB allocated (%.1fs)" % (
        torch.cuda.memory_allocated() / 1e9, time.time() - t0))

    w = Workload()
    w.name, w.cfg, w.graph, w.view, w.step = name, cfg, g, view, step
    w.dims, w.tau, w.d_s, w.L, w.ld, w.dtype = dims, tau, d_s, L, ld, dtype
    w.X_host, w.hist_host, w.table_ids, w.Ws, w.omegas, w.y = X_host, hist_host, table_ids, Ws, omegas, y
    w.device_keep = (keep, X_d, hist_d, ids_d, Ws_d, y_d)
    w.backbone, w.attn, w.coded = backbone, attn, coded
    return w
