"""GPU parity of the partition step with the history ring kept CODED (the paper's
section on compressing the stored historical embeddings): the predictor's window is
decoded from the codes, the push codes the fresh rows.

Oracle side: the same chain as in test_gpu_step.py, with every table the step reads
replaced by what a reader of the coded table gets back (orc.polyline_stored_value,
pinned against the byte-by-byte functions) and every push followed by that rounding.
The first step starts from bit-identical windows on both sides. A pushed row is the
quantisation of an fp32 row on the GPU and of an fp64 row in the oracle: where an
element lies within rounding of a quantisation boundary both codes are valid, so
the pushed part is compared as values (half a unit of the kept decimal plus the
fp32 tolerance), the differing elements must be exactly one unit apart, and in the
second step the rows such an element reaches (through the predictor's hop, then one hop
per layer: most rows of a power-law graph after three layers) are held to LOOSE only -
one unit of the kept decimal in one of a row's inputs - and all other rows to the fp32
tolerance.
"""
import numpy as np
import pytest

import sat_synth as syn
from oracle import sat_oracle as orc
from tests.test_gpu_step import RTOL, build_problem, check_backward, fresh_history, neighbours, oracle_step

pytestmark = pytest.mark.gpu
LOOSE = 5e-3


def _coded_ring(sat, gu, hist, ids_own, ids_remote, dims, ld, tau, prec, own_cap_per_value=4.0):
    """Device CodedRing from host fp32 tables: rows ids_own -> `own`, ids_remote -> `remote`."""
    from paper_2308_13466_amd.step import CodedRing, CodedSlot, encode_rows
    slots = [None]
    for l in range(1, len(hist)):
        layer = []
        for s in range(tau):
            own = gu.to_dev(hist[l][s][ids_own], ld[l])
            rem = gu.to_dev(hist[l][s][ids_remote], ld[l])
            oc, oo = encode_rows(own, ld[l], len(ids_own), dims[l], prec, sat.F32,
                                 capacity=int(len(ids_own) * dims[l] * own_cap_per_value),
                                 stream=gu.stream_ptr())
            rc, ro = encode_rows(rem, ld[l], len(ids_remote), dims[l], prec, sat.F32, stream=gu.stream_ptr())
            layer.append(CodedSlot(oc, oo, rc, ro))
        slots.append(layer)
    gu.sync()
    return CodedRing(prec, slots)


def _decode_part(sat, gu, codes, row_off, n, d, ld, prec):
    out = gu.dev_empty(n, ld, fill=0.0)
    sat.history_decompress(codes, row_off, n, None, n, d, prec, out, ld, stream=gu.stream_ptr())
    gu.sync()
    return gu.to_host(out, d)


@pytest.mark.parametrize("name,prec,bypass", [("tiny", 3, False), ("tiny", 2, True), ("medium", 2, False)])
def test_partition_step_with_a_coded_ring(name, prec, bypass):
    import paper_2308_13466_amd as sat
    from paper_2308_13466_amd.step import PartitionStep
    from tests import gpu_util as gu
    print("[case] coded-ring step %s, %d decimals, bypass=%s" % (name, prec, bypass), flush=True)
    cfg, ss, g, X, Ws, omegas = build_problem(name)
    dims, L, tau = cfg["dims"], len(Ws), cfg["tau"]
    Hfull, hist = fresh_history(cfg, ss, g, X, Ws)
    view = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, cfg["part"])
    oview = orc.partition_view(g.N, g.rowptr, g.col, g.part, cfg["part"])
    n_l, n_h = view["n_local"], view["n_halo"]
    y = syn.labels_i32(ss["labels"], n_l, dims[-1])
    print("[case] n_local=%d n_halo=%d nnz=%d" % (n_l, n_h, view["nnz"]), flush=True)

    ld = [gu.ld_for(d) for d in dims]
    X_d = gu.to_dev(X, ld[0])
    ids_d = gu.to_dev(np.concatenate([view["local_ids"], view["halo_ids"]]).astype(np.int32))
    Ws_d = [gu.to_dev(Ws[l], gu.ld_for(dims[l + 1], 4)) for l in range(L)]
    preds, keep = [None], []
    for l in range(1, L):
        pd = {k: gu.to_dev(omegas[l][k]) for k in omegas[l]}
        keep.append(pd)
        preds.append(sat.Predictor(pd["Wx"], pd["Wh"], pd["b"], pd["Wg"], dims[l], cfg["d_s"], tau,
                                   bypass=bypass))
    ring = _coded_ring(sat, gu, hist, view["local_ids"], view["halo_ids"], dims, ld, tau, prec)
    step = PartitionStep(view, dims, X_d, [None] * L, ids_d, Ws_d, preds, gu.to_dev(y), tau, coded=ring)

    # the oracle's tables: what a reader of the coded tables gets back
    ohist = [None] + [[orc.polyline_stored_value(t, prec) for t in hist[l]] for l in range(1, L)]
    for l in range(1, L):       # both sides start from the same bits
        slot = ring.slots[l][tau - 1]
        got = _decode_part(sat, gu, slot.remote_codes, slot.remote_off, n_h, dims[l], ld[l], prec)
        assert np.array_equal(got.view(np.uint32), ohist[l][tau - 1][view["halo_ids"]].view(np.uint32))
        got = _decode_part(sat, gu, slot.own_codes, slot.own_off, n_l, dims[l], ld[l], prec)
        assert np.array_equal(got.view(np.uint32), ohist[l][tau - 1][view["local_ids"]].view(np.uint32))

    unit = 10.0 ** -prec
    doubtful = set()            # local rows whose stored value differs between the two sides
    for t in range(2):
        order = [(t + s) % tau for s in range(tau)]
        step.forward_backward()
        gu.sync()
        assert step.coded_overflow() == []
        st = oracle_step(oview, X, ohist, order, t % tau, Ws, omegas, y, bypass=bypass)
        st["y"] = y
        for l in range(1, L):   # the oracle's push, as a coded table stores it
            tab = ohist[l][t % tau]
            tab[view["local_ids"]] = orc.polyline_stored_value(tab[view["local_ids"]], prec)

        # rows a differing stored element reaches: predicted halo rows next to it, then
        # one hop per aggregation
        halo_bad = set()
        if doubtful and not bypass:
            for u in range(n_h):
                lo, hi = view["h_colptr"][u], view["h_colptr"][u + 1]
                if doubtful.intersection(int(r) for r in view["h_row"][lo:hi]):
                    halo_bad.add(u)
        rows_bad = set()
        if halo_bad:
            for i in range(n_l):
                cols = view["col"][view["split"][i]:view["rowptr"][i + 1]]
                if halo_bad.intersection(int(c) - n_l for c in cols):
                    rows_bad.add(i)
        halo_ok = np.ones(n_h, dtype=bool)
        halo_ok[sorted(halo_bad)] = False
        for l in range(1, L):
            for rows, tol in ((halo_ok, RTOL), (~halo_ok, LOOSE)):
                if rows.any():
                    gu.assert_close(gu.to_host(step.Hbar[l], dims[l])[n_l:][rows], st["halo_hat"][l][rows],
                                    tol, "halo rows fed to layer %d, step %d" % (l, t))
        reach = set()           # grows by one hop per layer from layer 1 on
        for l in range(L):
            if l >= 1:
                reach = reach | neighbours(oview, reach) | rows_bad
            ok = np.ones(n_l, dtype=bool)
            ok[sorted(reach)] = False
            out = step.logits if l == L - 1 else step.Hbar[l + 1]
            for rows, tol in ((ok, RTOL), (~ok, LOOSE)):
                if rows.any():
                    gu.assert_close(gu.to_host(step.AGG[l], dims[l])[rows], st["AGG"][l][rows], tol,
                                    "AGG %d" % l)
                    gu.assert_close(gu.to_host(out, dims[l + 1])[:n_l][rows], st["H"][l + 1][rows], tol,
                                    "H %d" % (l + 1))
        if not reach:
            assert abs(float(step.loss.item()) - st["loss"]) <= 2 * RTOL * abs(st["loss"])
            dW_gpu = [gu.to_host(step.dW[l], dims[l + 1]) for l in range(L)]
            dAGG_gpu = [None] + [gu.to_host(step.dAGG[l], dims[l]) for l in range(1, L)]
            dH_gpu = [None] + [gu.to_host(step.dH[l], dims[l]) for l in range(1, L)]
            check_backward(gu, oview, st, dW_gpu, dAGG_gpu, dH_gpu, dims)
        else:
            assert abs(float(step.loss.item()) - st["loss"]) <= 1e-3 * abs(st["loss"])
        assert len(reach) < 0.75 * n_l, "too few rows held to the fp32 tolerance: %d left out" % len(reach)

        # the push: the `own` part of the write slot decodes to the fresh rows within half a
        # unit; against the oracle's stored values only elements next to a boundary differ,
        # by exactly one unit; the `remote` part is untouched
        n_diff = 0
        for l in range(1, L):
            slot = ring.slots[l][t % tau]
            got = _decode_part(sat, gu, slot.own_codes, slot.own_off, n_l, dims[l], ld[l], prec)
            fresh = gu.to_host(step.Hbar[l], dims[l])[:n_l]
            assert np.array_equal(got.view(np.uint32), orc.polyline_stored_value(fresh, prec).view(np.uint32))
            ref = st["H"][l]
            rms = np.sqrt(np.mean(ref * ref))
            assert np.all(np.abs(got - ref) <= 0.5 * unit * (1 + 1e-5) + RTOL * (np.abs(ref) + rms) + 1e-6)
            want = ohist[l][t % tau][view["local_ids"]]
            diff = got != want
            if diff.any():
                assert np.all(np.abs(np.abs(got[diff].astype(np.float64) - want[diff]) - unit) <= 1e-3 * unit)
                frac = ref[diff] / unit + 0.5
                assert np.all(np.abs(frac - np.round(frac)) <= 1e-3), "differing codes away from a boundary"
                doubtful |= set(int(i) for i in np.flatnonzero(diff.any(axis=1)))
                n_diff += int(diff.sum())
            got_r = _decode_part(sat, gu, slot.remote_codes, slot.remote_off, n_h, dims[l], ld[l], prec)
            assert np.array_equal(got_r.view(np.uint32), ohist[l][t % tau][view["halo_ids"]].view(np.uint32))
        print("[case] step %d ok: loss %.6f, %d rows left out, %d stored elements on a boundary"
              % (t, st["loss"], len(reach), n_diff), flush=True)


class _StoredTable:
    """Rows of a host table as a reader of its coded form gets them back."""

    def __init__(self, table, prec):
        self.table, self.prec = table, prec

    def __getitem__(self, ids):
        return orc.polyline_stored_value(self.table[ids], self.prec)


def test_coded_ring_step_at_full_size():
    """The benchmark's workload with its ring coded at two decimals, in the configuration
    `bench.py --coded-ring 2` times: decoded windows and predicted halo rows on samples
    the oracle computes one by one, the pushed part against the forward's rows in full."""
    import types
    import torch
    import paper_2308_13466_amd as sat
    from paper_2308_13466_amd.workload import build_workload
    from tests import gpu_util as gu
    from tests.test_gpu_large import _oracle_predict_rows
    prec = 2
    print("[case] coded-ring step, workload large, %d decimals" % prec, flush=True)
    wl = build_workload("large", coded_ring=prec, log=lambda m: print("[case] " + m, flush=True))
    v, step, dims, tau = wl.view, wl.step, wl.dims, wl.tau
    n_l, n_h = v["n_local"], v["n_halo"]
    rng = np.random.default_rng(23)
    order = step.slot_order()
    step.forward_backward()
    gu.sync()
    assert step.coded_overflow() == []
    stored = types.SimpleNamespace(
        view=v, dims=dims, table_ids=wl.table_ids, omegas=wl.omegas,
        hist_host=[None] + [[_StoredTable(t, prec) for t in wl.hist_host[l]] for l in range(1, wl.L)])
    # the decoded window of the step: sampled local and halo rows, bit for bit
    rows = np.sort(rng.choice(n_l + n_h, size=4096, replace=False))
    ridx = torch.from_numpy(rows).to(gu.DEV)
    for l in (wl.L - 1,):       # the layers share the window's memory: the last one's is left
        for k, s in enumerate(order):
            got = step.window[l][k][ridx].cpu().numpy()[:, :dims[l]]
            want = stored.hist_host[l][s][wl.table_ids[rows]][:, :dims[l]]
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), "window %d slot %d" % (l, s)
    # predicted halo rows from the stored values
    cp = v["h_colptr"]
    halo_sample = np.sort(rng.choice(n_h, size=1024, replace=False))
    halo_sample = np.unique(np.concatenate([halo_sample, np.argsort(np.diff(cp))[-4:]]))
    for l in range(1, wl.L):
        ref = _oracle_predict_rows(stored, l, halo_sample, order)
        got = step.Hbar[l][torch.from_numpy(n_l + halo_sample).to(gu.DEV)].cpu().numpy()[:, :dims[l]]
        gu.assert_close(got, ref, RTOL, "predicted halo rows, layer %d" % l)
    # push: the `own` part of slot 0 holds the stored values of the forward's local rows
    total = dense = 0
    for l in range(1, wl.L):
        slot = wl.coded.slots[l][0]
        got = _decode_part(sat, gu, slot.own_codes, slot.own_off, n_l, dims[l], step.ld[l], prec)
        fresh = step.Hbar[l][:n_l].cpu().numpy()[:, :dims[l]]
        assert np.array_equal(got.view(np.uint32), orc.polyline_stored_value(fresh, prec).view(np.uint32))
        for s in range(tau):
            total += sum(wl.coded.slots[l][s].coded_bytes())
            dense += (n_l + n_h) * dims[l] * 4
    print("[case] ring: %.3f GB coded, %.3f GB dense" % (total / 1e9, dense / 1e9), flush=True)
    assert dense / total > 2.5
    assert np.isfinite(float(step.loss.item()))
    step.forward_backward()
    gu.sync()
    assert step.coded_overflow() == [] and np.isfinite(float(step.loss.item()))


@pytest.mark.parametrize("name", ["tiny", "medium"])
def test_coded_ring_step_bf16_storage(name):
    """bf16 tables behind the codec: a coded value is the quantised bfloat16 element, a decoded
    one is rounded to bfloat16 again. One step from bit-identical windows; the pushed part
    must hold exactly the stored form of the forward's own rows."""
    import torch
    import paper_2308_13466_amd as sat
    from paper_2308_13466_amd import binding as B
    from paper_2308_13466_amd.step import CodedRing, CodedSlot, PartitionStep, encode_rows
    from tests import gpu_util as gu
    prec, rtol = 2, 2e-2
    print("[case] coded-ring step %s, bf16 storage, %d decimals" % (name, prec), flush=True)

    def r(a):
        return syn.f32_from_bf16_bits(syn.bf16_bits_from_f32(a))

    def up(a, ld):
        return gu.to_dev_bits(syn.bf16_bits_from_f32(a), ld).view(torch.bfloat16)

    def down(t, d):
        return syn.f32_from_bf16_bits(gu.bits_to_host(t.view(torch.int16), d))

    def stored(a):      # oracle: what a reader of a coded bf16 table gets back
        return orc.round_bf16(orc.polyline_stored_value(a, prec)).astype(np.float32)

    cfg, ss, g, X, Ws, omegas = build_problem(name)
    dims, L, tau = cfg["dims"], len(Ws), cfg["tau"]
    _, hist = fresh_history(cfg, ss, g, X, Ws)
    X = r(X)
    Ws = [r(w) for w in Ws]
    hist = [None] + [[r(t) for t in hist[l]] for l in range(1, L)]
    view = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, cfg["part"])
    oview = orc.partition_view(g.N, g.rowptr, g.col, g.part, cfg["part"])
    n_l, n_h = view["n_local"], view["n_halo"]
    y = syn.labels_i32(ss["labels"], n_l, dims[-1])
    ld = [gu.ld_for(d) for d in dims]
    X_d = up(X, ld[0])
    ids_d = gu.to_dev(np.concatenate([view["local_ids"], view["halo_ids"]]).astype(np.int32))
    Ws_d = [up(Ws[l], gu.ld_for(dims[l + 1], 8)) for l in range(L)]
    preds, keep = [None], []
    for l in range(1, L):
        pd = {k: gu.to_dev(omegas[l][k]) for k in omegas[l]}
        keep.append(pd)
        preds.append(sat.Predictor(pd["Wx"], pd["Wh"], pd["b"], pd["Wg"], dims[l], cfg["d_s"], tau))
    slots = [None]
    for l in range(1, L):
        layer = []
        for s in range(tau):
            own, rem = up(hist[l][s][view["local_ids"]], ld[l]), up(hist[l][s][view["halo_ids"]], ld[l])
            oc, oo = encode_rows(own, ld[l], n_l, dims[l], prec, B.BF16, capacity=n_l * dims[l] * 4,
                                 stream=gu.stream_ptr())
            rc, ro = encode_rows(rem, ld[l], n_h, dims[l], prec, B.BF16, stream=gu.stream_ptr())
            layer.append(CodedSlot(oc, oo, rc, ro))
        slots.append(layer)
    gu.sync()
    ring = CodedRing(prec, slots)
    step = PartitionStep(view, dims, X_d, [None] * L, ids_d, Ws_d, preds, gu.to_dev(y), tau,
                         dtype=B.BF16, coded=ring)
    ohist = [None] + [[stored(t) for t in hist[l]] for l in range(1, L)]
    order = step.slot_order()
    step.forward_backward()
    gu.sync()
    assert step.coded_overflow() == []
    ids = np.concatenate([view["local_ids"], view["halo_ids"]])
    for k, s in enumerate(order):       # the decoded window (last hidden layer's is left in place)
        assert np.array_equal(down(step.window[L - 1][k], dims[L - 1]), ohist[L - 1][s][ids])
    st = oracle_step(oview, X, ohist, order, 0, Ws, omegas, y, store=orc.round_bf16)
    for l in range(1, L):
        gu.assert_close(down(step.Hbar[l], dims[l])[n_l:], st["halo_hat"][l], rtol,
                        "predicted halo rows, layer %d" % l)
    for l in range(L):
        gu.assert_close(down(step.AGG[l], dims[l]), st["AGG"][l], rtol, "AGG %d" % l)
        out = step.logits if l == L - 1 else step.Hbar[l + 1]
        gu.assert_close(down(out, dims[l + 1])[:n_l], st["H"][l + 1], rtol, "H %d" % (l + 1))
    assert abs(float(step.loss.item()) - st["loss"]) <= 5e-3 * abs(st["loss"])
    unit = 10.0 ** -prec
    for l in range(1, L):
        slot = ring.slots[l][0]
        out = torch.zeros((n_l, ld[l]), dtype=torch.bfloat16, device=gu.DEV)
        sat.history_decompress(slot.own_codes, slot.own_off, n_l, None, n_l, dims[l], prec, out, ld[l],
                               dtype=B.BF16, stream=gu.stream_ptr())
        gu.sync()
        got = down(out, dims[l])
        fresh = down(step.Hbar[l], dims[l])[:n_l]
        assert np.array_equal(got, stored(fresh)), "pushed part, layer %d" % l
        ref = st["H"][l]
        rms = np.sqrt(np.mean(ref * ref))
        assert np.all(np.abs(got - ref) <= 0.5 * unit + rtol * (np.abs(ref) + rms))
    print("[case] ok: loss %.6f" % st["loss"], flush=True)


@pytest.mark.parametrize("name", ["tiny", "medium"])
def test_coded_ring_predictions_one_step_ahead_change_nothing(name):
    """With the coded ring, predict_ahead moves the decode of the window and the predictor's
    calls to a second stream, beside the previous step's backward: every buffer after three
    steps, the codes in the ring included, equals bit for bit what the in-step order leaves.
    The halo rows then already hold the predictions FOR step 3, which the in-step order makes
    at the start of its fourth call."""
    import torch
    from paper_2308_13466_amd.workload import build_workload
    print("[case] coded ring, predictions one step ahead, %s" % name, flush=True)

    def snapshot(st):
        n_l = st.n_local
        keep = [st.logits.clone(), st.loss.clone()] + [w.clone() for w in st.dW]
        keep += [h[:n_l].clone() for h in st.Hbar[1:]] + [g.clone() for g in st.dH[1:]]
        for l in range(1, st.L):
            for slot in st.coded.slots[l]:
                used = int(slot.own_off[-1].item())
                keep += [slot.own_off.clone(), slot.own_codes[:used].clone()]
        return keep

    runs, halo = [], []
    for ahead in (False, True):
        wl = build_workload(name, coded_ring=2, predict_ahead=ahead)
        st = wl.step
        for _ in range(3):
            st.forward_backward()
        torch.cuda.synchronize()
        assert st.coded_overflow() == []
        runs.append(snapshot(st))
        if not ahead:
            st.forward_backward()
            torch.cuda.synchronize()
        halo.append([h[st.n_local:].clone() for h in st.Hbar[1:]])
        del wl, st

    def same(a, b):
        if a.dtype == torch.float32:
            a, b = a.view(torch.int32), b.view(torch.int32)
        return a.shape == b.shape and torch.equal(a, b)
    for k, (a, b) in enumerate(zip(*runs)):
        assert same(a, b), "buffer %d differs" % k
    for k, (a, b) in enumerate(zip(*halo)):
        assert same(a, b), "predicted halo rows of hidden layer %d differ" % (k + 1)


@pytest.mark.parametrize("name,chunk,ahead", [("tiny", 777, False), ("medium", 10_000, False), ("medium", 30_011, True)])
def test_coded_ring_window_decoded_a_range_of_rows_at_a_time(name, chunk, ahead):
    """coded_chunk_rows: the window is decoded `chunk` rows at a time, each range goes through
    the LSTM alone (sat_predict_states) and the hop adds its term in place on the newest
    slot's halo rows (sat_predict_hop). Nothing but the size of the dense scratch may change:
    every buffer after three steps, and the predictions of the fourth, equal bit for bit those
    of the step that decodes the whole window (which the tests above hold to the oracle)."""
    import torch
    from paper_2308_13466_amd.workload import build_workload
    print("[case] coded ring decoded %d rows at a time, %s, ahead=%s" % (chunk, name, ahead), flush=True)

    def snapshot(st):
        n_l = st.n_local
        keep = [st.logits.clone(), st.loss.clone()] + [w.clone() for w in st.dW]
        keep += [h[:n_l].clone() for h in st.Hbar[1:]] + [g.clone() for g in st.dH[1:]]
        for l in range(1, st.L):
            for slot in st.coded.slots[l]:
                used = int(slot.own_off[-1].item())
                keep += [slot.own_off.clone(), slot.own_codes[:used].clone()]
        return keep

    runs, halo = [], []
    for c in (None, chunk):
        wl = build_workload(name, coded_ring=2, predict_ahead=ahead, coded_chunk_rows=c)
        st = wl.step
        if c is not None:
            assert st.window[1][0].shape[0] == min(chunk, st.n_bar)
        for _ in range(3):
            st.forward_backward()
        torch.cuda.synchronize()
        assert st.coded_overflow() == []
        runs.append(snapshot(st))
        if not ahead:
            st.forward_backward()
            torch.cuda.synchronize()
        halo.append([h[st.n_local:].clone() for h in st.Hbar[1:]])
        del wl, st

    def same(a, b):
        if a.dtype == torch.float32:
            a, b = a.view(torch.int32), b.view(torch.int32)
        return a.shape == b.shape and torch.equal(a, b)
    for k, (a, b) in enumerate(zip(*runs)):
        assert same(a, b), "buffer %d differs" % k
    for k, (a, b) in enumerate(zip(*halo)):
        assert same(a, b), "predicted halo rows of hidden layer %d differ" % (k + 1)
