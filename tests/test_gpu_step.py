"""GPU parity of the whole partition step (pull, predict, forward, push, loss,
backward) against the oracle's chain started from the same seeded inputs, on
the Tiny and Medium configurations, for two consecutive steps so that the
history ring rotates once."""
import numpy as np
import pytest

import sat_synth as syn
from oracle import sat_oracle as orc

pytestmark = pytest.mark.gpu
RTOL = 1e-5


def build_problem(name, scale_nodes=None):
    """Seeded inputs of one configuration (host arrays only)."""
    cfg = syn.get_config(name)
    if scale_nodes:
        cfg["N"] = scale_nodes
    ss = syn.substreams(cfg["seed"])
    g = syn.make_graph(cfg, np.random.default_rng(ss["graph"]))
    dims, L, tau = cfg["dims"], len(cfg["dims"]) - 1, cfg["tau"]
    X = syn.normal_f32(ss["features"], g.N, dims[0])
    wss = ss["weights"].spawn(L)
    Ws = [syn.glorot_uniform_f32(wss[l], dims[l], dims[l + 1]) for l in range(L)]
    pss = ss["predictor"].spawn(L)
    omegas = [None] + [syn.predictor_params_f32(pss[l], dims[l], cfg["d_s"]) for l in range(1, L)]
    return cfg, ss, g, X, Ws, omegas


def fresh_history(cfg, ss, g, X, Ws):
    """History tables per the configuration: the unpartitioned GCN's embeddings
    of every node (computed by the oracle) plus N(0, noise_std^2) per slot."""
    L, tau = len(Ws), cfg["tau"]
    Hfull = orc.full_graph_gcn(g.N, g.rowptr, g.col, X, Ws)
    nss = ss["noise"].spawn(L * tau)
    hist = [None]
    for l in range(1, L):
        base = Hfull[l].astype(np.float32)
        hist.append([base + syn.normal_f32(nss[l * tau + s], g.N, base.shape[1], std=cfg["noise_std"])
                     for s in range(tau)])
    return Hfull, hist


def oracle_step(view, X, hist, order, w_slot, Ws, omegas, y, bypass=False, store=None):
    """store: rounding applied to everything the step keeps in memory (None: exact)."""
    ids = np.concatenate([view["local_ids"], view["halo_ids"]])
    L = len(Ws)
    halo_hat = [None]
    for l in range(1, L):
        win = [hist[l][s][ids] for s in order]
        hh = orc.predict(view, omegas[l], win, bypass=bypass)
        halo_hat.append(hh if store is None else store(hh))
    st = orc.partition_step(view, X[view["local_ids"]], X[view["halo_ids"]], halo_hat, Ws, y,
                            store=store)
    for l in range(1, L):
        orc.history_push(hist[l][w_slot], view["local_ids"], st["H"][l].astype(np.float32))
    st["halo_hat"] = halo_hat
    return st


def neighbours(view, rows):
    """Local rows sharing a P_in entry with any of `rows` (P_in is symmetric)."""
    out = set()
    for i in rows:
        out.update(int(c) for c in view["col"][view["rowptr"][i]:view["split"][i]])
    return out


def check_backward(gu, view, st, dW_gpu, dAGG_gpu, dH_gpu, dims, rtol=RTOL, amb_rel=2e-6,
                   max_bad_rows=0):
    """Compare the backward pass. relu'(Z) is a 0/1 decision taken on an fp32 Z
    by the GPU and on an fp64 Z by the oracle; where |Z| is within rounding of 0
    either decision is valid, so rows reached by such an element are left out
    of the row-wise comparisons and their possible contribution is added to
    the tolerance of dW."""
    L = len(dims) - 1
    bad = set()                 # rows of dH^(l+1) whose value may legitimately differ
    n_amb_total = 0
    for l in range(L - 1, -1, -1):
        Z, AGG = st["Z"][l], st["AGG"][l]
        if l < L - 1:
            thr = amb_rel * np.sqrt(np.mean(Z * Z))   # default: ~20x the fp32 rounding of Z
            amb = np.abs(Z) < thr
            n_amb_total += int(amb.sum())
            bad |= set(int(i) for i in np.flatnonzero(amb.any(axis=1)))
        rows_bad = np.array(sorted(bad), dtype=np.int64)
        ok = np.ones(view["n_local"], dtype=bool)
        ok[rows_bad] = False
        # dW: contribution of the doubtful rows bounds the admissible difference
        ref = st["dW"][l]
        slack = np.zeros_like(ref)
        if rows_bad.size:
            up = np.abs(dH_or(st, l + 1, L)[rows_bad])
            slack = 2.0 * np.abs(AGG[rows_bad]).T @ up
        rms = np.sqrt(np.mean(ref * ref))
        err = np.abs(dW_gpu[l] - ref)
        assert np.all(err <= rtol * (np.abs(ref) + rms) + slack), "dW layer %d" % l
        if l >= 1:
            gu.assert_close(dAGG_gpu[l][ok], st["dAGG"][l][ok], rtol, "dAGG layer %d" % l,
                            max_bad_rows=max_bad_rows)
            bad = neighbours(view, bad) | bad
            ok = np.ones(view["n_local"], dtype=bool)
            ok[np.array(sorted(bad), dtype=np.int64)] = False
            gu.assert_close(dH_gpu[l][ok], st["dH_in"][l][ok], rtol, "dH_in layer %d" % l,
                            max_bad_rows=max_bad_rows * 32)
    return n_amb_total, len(bad)


def dH_or(st, l, L):
    """Gradient arriving at H^(l): loss gradient for l = L, else dH_in[l]."""
    if l == L:
        return orc.loss_and_grad(st["H"][L], st["y"])[1]
    return st["dH_in"][l]


@pytest.mark.parametrize("name,fused", [("tiny", True), ("tiny", False), ("medium", True)])
def test_partition_step_two_steps(name, fused):
    import torch
    import paper_2308_13466_amd as sat
    from paper_2308_13466_amd.step import PartitionStep
    from tests import gpu_util as gu
    print("[case] step %s fused_pull=%s" % (name, fused), flush=True)
    cfg, ss, g, X, Ws, omegas = build_problem(name)
    dims, L, tau = cfg["dims"], len(Ws), cfg["tau"]
    m = cfg["part"]
    Hfull, hist = fresh_history(cfg, ss, g, X, Ws)
    view = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, m)
    oview = orc.partition_view(g.N, g.rowptr, g.col, g.part, m)
    for k in ("rowptr", "split", "col", "halo_ids", "local_ids", "h_colptr", "h_row"):
        assert np.array_equal(view[k], oview[k])
    y = syn.labels_i32(ss["labels"], view["n_local"], dims[-1])
    print("[case] n_local=%d n_halo=%d nnz=%d" % (view["n_local"], view["n_halo"], view["nnz"]),
          flush=True)

    ld = [gu.ld_for(d) for d in dims]
    X_d = gu.to_dev(X, ld[0])
    hist_d = [None] + [[gu.to_dev(t, ld[l]) for t in hist[l]] for l in range(1, L)]
    ids_d = gu.to_dev(np.concatenate([view["local_ids"], view["halo_ids"]]).astype(np.int32))
    Ws_d = [gu.to_dev(Ws[l], gu.ld_for(dims[l + 1], 4)) for l in range(L)]
    preds = [None]
    keep = []
    for l in range(1, L):
        pd = {k: gu.to_dev(omegas[l][k]) for k in omegas[l]}
        keep.append(pd)
        preds.append(sat.Predictor(pd["Wx"], pd["Wh"], pd["b"], pd["Wg"], dims[l], cfg["d_s"], tau))
    step = PartitionStep(view, dims, X_d, hist_d, ids_d, Ws_d, preds, gu.to_dev(y), tau,
                         fused_pull=fused)
    ohist = [None] + [[t.copy() for t in hist[l]] for l in range(1, L)]
    n_l = view["n_local"]
    for t in range(2):
        order = [(t + s) % tau for s in range(tau)]
        assert step.slot_order() == order
        step.forward_backward()
        gu.sync()
        st = oracle_step(oview, X, ohist, order, t % tau, Ws, omegas, y)
        st["y"] = y
        for l in range(1, L):
            gu.assert_close(gu.to_host(step.Hbar[l], dims[l])[n_l:], st["halo_hat"][l], RTOL,
                            "predicted halo rows, layer %d step %d" % (l, t))
        for l in range(L):
            gu.assert_close(gu.to_host(step.AGG[l], dims[l]), st["AGG"][l], RTOL, "AGG %d" % l)
            out = step.logits if l == L - 1 else step.Hbar[l + 1]
            gu.assert_close(gu.to_host(out, dims[l + 1])[:n_l], st["H"][l + 1], RTOL, "H %d" % (l + 1))
        assert abs(float(step.loss.item()) - st["loss"]) <= 2 * RTOL * abs(st["loss"])
        # push: the table rows hold exactly what the forward produced
        for l in range(1, L):
            tab = step.hist[l][t % tau].cpu().numpy()
            assert np.array_equal(tab[view["local_ids"], :dims[l]],
                                  gu.to_host(step.Hbar[l], dims[l])[:n_l])
            others = np.setdiff1d(np.arange(g.N), view["local_ids"])
            assert np.array_equal(tab[others, :dims[l]], ohist[l][t % tau][others])
        dW_gpu = [gu.to_host(step.dW[l], dims[l + 1]) for l in range(L)]
        dAGG_gpu = [None] + [gu.to_host(step.dAGG[l], dims[l]) for l in range(1, L)]
        dH_gpu = [None] + [gu.to_host(step.dH[l], dims[l]) for l in range(1, L)]
        n_amb, n_bad = check_backward(gu, oview, st, dW_gpu, dAGG_gpu, dH_gpu, dims)
        print("[case] step %d ok: loss %.6f, %d relu decisions within rounding of 0, %d rows excluded"
              % (t, st["loss"], n_amb, n_bad), flush=True)
        assert n_bad < 0.02 * n_l


def test_zero_staleness_invariant_on_gpu():
    """History equal to the fresh embeddings and the predictor bypassed: the
    partition's forward must reproduce rows V_m of the unpartitioned GCN."""
    import paper_2308_13466_amd as sat
    from paper_2308_13466_amd.step import PartitionStep
    from tests import gpu_util as gu
    print("[case] zero-staleness invariant, tiny", flush=True)
    cfg, ss, g, X, Ws, omegas = build_problem("tiny")
    dims, L, tau = cfg["dims"], len(Ws), cfg["tau"]
    Hfull = orc.full_graph_gcn(g.N, g.rowptr, g.col, X, Ws)
    for m in (0, 1):
        view = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, m)
        y = syn.labels_i32(ss["labels"], view["n_local"], dims[-1])
        ld = [gu.ld_for(d) for d in dims]
        hist_d = [None] + [[gu.to_dev(Hfull[l].astype(np.float32), ld[l]) for _ in range(tau)]
                           for l in range(1, L)]
        ids_d = gu.to_dev(np.concatenate([view["local_ids"], view["halo_ids"]]).astype(np.int32))
        Ws_d = [gu.to_dev(Ws[l], gu.ld_for(dims[l + 1], 4)) for l in range(L)]
        # the two spellings of "no predictor": an explicit bypass predictor, or None
        preds = [None] + [sat.Predictor(None, None, None, None, dims[l], 32, tau, bypass=True)
                          if m == 0 else None for l in range(1, L)]
        step = PartitionStep(view, dims, gu.to_dev(X, ld[0]), hist_d, ids_d, Ws_d, preds,
                             gu.to_dev(y), tau)
        step.forward_backward()
        gu.sync()
        n_l = view["n_local"]
        for l in range(1, L + 1):
            out = step.logits if l == L else step.Hbar[l]
            gu.assert_close(gu.to_host(out, dims[l])[:n_l], Hfull[l][view["local_ids"]], 2e-5,
                            "H^(%d) vs unpartitioned GCN, partition %d" % (l, m))


def test_predictor_update_frequency():
    """Delta T of Alg. 1: with predict_every = 2 the predicted halo rows of step 1 are the
    ones step 0 left in place, and step 2 refreshes them from the ring as it stands then."""
    import paper_2308_13466_amd as sat
    from paper_2308_13466_amd.step import PartitionStep
    from tests import gpu_util as gu
    print("[case] predictor every 2 steps, tiny", flush=True)
    cfg, ss, g, X, Ws, omegas = build_problem("tiny")
    dims, L, tau = cfg["dims"], len(Ws), cfg["tau"]
    _, hist = fresh_history(cfg, ss, g, X, Ws)
    view = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, 0)
    oview = orc.partition_view(g.N, g.rowptr, g.col, g.part, 0)
    y = syn.labels_i32(ss["labels"], view["n_local"], dims[-1])
    ld = [gu.ld_for(d) for d in dims]
    hist_d = [None] + [[gu.to_dev(t, ld[l]) for t in hist[l]] for l in range(1, L)]
    ids_d = gu.to_dev(np.concatenate([view["local_ids"], view["halo_ids"]]).astype(np.int32))
    pd = {k: gu.to_dev(omegas[1][k]) for k in omegas[1]}
    preds = [None, sat.Predictor(pd["Wx"], pd["Wh"], pd["b"], pd["Wg"], dims[1], 32, tau)]
    step = PartitionStep(view, dims, gu.to_dev(X, ld[0]), hist_d, ids_d,
                         [gu.to_dev(Ws[l], gu.ld_for(dims[l + 1], 4)) for l in range(L)], preds,
                         gu.to_dev(y), tau, predict_every=2)
    n_l = view["n_local"]
    halo = []
    for t in range(3):
        step.forward_backward()
        gu.sync()
        halo.append(gu.to_host(step.Hbar[1], dims[1])[n_l:].copy())
    assert np.array_equal(halo[0], halo[1])
    assert not np.array_equal(halo[1], halo[2])
    # step 2's prediction is the oracle's from the ring after two pushes (slot order [0, 1] again)
    ids = np.concatenate([oview["local_ids"], oview["halo_ids"]])
    ring = [gu.to_host(hist_d[1][s], dims[1])[ids] for s in (0, 1)]
    gu.assert_close(halo[2], orc.predict(oview, omegas[1], ring), RTOL, "refreshed prediction")


@pytest.mark.parametrize("coded_ring", [None, 3])
def test_step_replayed_from_a_hip_graph_matches_eager_steps(coded_ring):
    """tau consecutive steps captured into one HIP graph and replayed several times, with the
    program's own eager work and synchronisations between the replays: after every replay the
    loss, the weight gradients and the history ring (dense tables, or the codes and offsets
    of a coded ring) equal, bit for bit, what the same number of eager steps leaves on an
    identical second instance."""
    import torch
    import paper_2308_13466_amd as sat
    from paper_2308_13466_amd.workload import build_workload
    print("[case] HIP graph replay vs eager steps, tiny, coded ring: %s" % coded_ring, flush=True)
    sat.lib()
    eager = build_workload("tiny", coded_ring=coded_ring, own_headroom=2.0).step
    graphed = build_workload("tiny", coded_ring=coded_ring, own_headroom=2.0).step
    period = graphed.graph_period()
    assert period == graphed.tau
    for _ in range(period):           # one eager period on both before the capture
        eager.forward_backward()
        graphed.forward_backward()
    torch.cuda.synchronize()
    replay = graphed.capture()
    scratch = torch.zeros(1 << 20, device="cuda:0")
    for rep in range(4):
        replay()
        for _ in range(period):
            eager.forward_backward()
        scratch.add_(1.0)             # unrelated eager work between the replays
        torch.cuda.synchronize()
        assert graphed.t == eager.t
        assert torch.equal(graphed.loss, eager.loss), rep
        for l in range(eager.L):
            assert torch.equal(graphed.dW[l], eager.dW[l]), (rep, l)
        for l in range(1, eager.L):
            for s in range(eager.tau):
                if coded_ring is None:
                    assert torch.equal(graphed.hist[l][s], eager.hist[l][s]), (rep, l, s)
                    continue
                a, b = graphed.coded.slots[l][s], eager.coded.slots[l][s]
                assert torch.equal(a.own_off, b.own_off), (rep, l, s)
                used = int(a.own_off[-1].item())
                assert torch.equal(a.own_codes[:used], b.own_codes[:used]), (rep, l, s)
            assert torch.equal(graphed.Hbar[l], eager.Hbar[l]), (rep, l)
    assert graphed.coded_overflow() == []
    assert float(scratch[0].item()) == 4.0


@pytest.mark.parametrize("name", ["tiny", "medium"])
def test_predictions_one_step_ahead_change_nothing(name):
    """predict_ahead only moves the predictor's calls to a second stream, beside the previous
    step's backward: every buffer of three steps must equal, bit for bit, what the in-step
    order leaves (same kernels, same inputs, fixed-order reductions). After step 2 the halo
    rows of Hbar_l already hold the predictions FOR step 3: those are compared with what the
    in-step order computes at the start of its step 3."""
    import torch
    from paper_2308_13466_amd.workload import build_workload
    print("[case] predictions one step ahead, %s" % name, flush=True)

    def snapshot(st):
        n_l = st.n_local
        keep = [st.logits.clone(), st.loss.clone()] + [w.clone() for w in st.dW]
        keep += [h[:n_l].clone() for h in st.Hbar[1:]] + [g.clone() for g in st.dH[1:]]
        keep += [t.clone() for l in range(1, st.L) for t in st.hist[l]]
        return keep

    runs, halo = [], []
    for ahead in (False, True):
        wl = build_workload(name, predict_ahead=ahead)
        st = wl.step
        for _ in range(3):
            st.forward_backward()
        torch.cuda.synchronize()
        runs.append(snapshot(st))
        if not ahead:
            st.forward_backward()          # its predictions are the ones the other order has made already
            torch.cuda.synchronize()
        halo.append([h[st.n_local:].clone() for h in st.Hbar[1:]])
        del wl, st

    def same(a, b):
        return a.dtype == b.dtype and torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a,
                                                  b.view(torch.int32) if b.dtype == torch.float32 else b)
    for k, (a, b) in enumerate(zip(*runs)):
        assert same(a, b), "buffer %d differs" % k
    for k, (a, b) in enumerate(zip(*halo)):
        assert same(a, b), "predicted halo rows of hidden layer %d differ" % (k + 1)
