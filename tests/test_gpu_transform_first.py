"""The last layer evaluated as P (Hbar W) instead of (P Hbar) W (PartitionStep(transform_first=
True); the appendix's Z = P H W fixes no order of the two products): every output of two
steps against the oracle, which aggregates first as everywhere else - logits, loss, every
weight gradient, every gradient to a hidden layer - plus the two intermediate matrices the
order introduces: Zbar = Hbar_{L-1} W_{L-1} over local and halo rows, and G = [P_in | P_out]^T
dH^(L) over local and halo rows."""
import numpy as np
import pytest

import sat_synth as syn
from oracle import sat_oracle as orc
from tests.test_gpu_step import build_problem, check_backward, fresh_history, oracle_step

pytestmark = pytest.mark.gpu
RTOL = 1e-5


@pytest.mark.parametrize("name", ["tiny", "medium"])
def test_transform_first_last_layer_two_steps(name):
    import paper_2308_13466_amd as sat
    from paper_2308_13466_amd.step import PartitionStep
    from tests import gpu_util as gu
    print("[case] last layer as P (Hbar W), %s" % name, flush=True)
    cfg, ss, g, X, Ws, omegas = build_problem(name)
    dims, L, tau = cfg["dims"], len(Ws), cfg["tau"]
    m = cfg["part"]
    _, hist = fresh_history(cfg, ss, g, X, Ws)
    view = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, m)
    oview = orc.partition_view(g.N, g.rowptr, g.col, g.part, m)
    y = syn.labels_i32(ss["labels"], view["n_local"], dims[-1])
    ld = [gu.ld_for(d) for d in dims]
    hist_d = [None] + [[gu.to_dev(t, ld[l]) for t in hist[l]] for l in range(1, L)]
    ids_d = gu.to_dev(np.concatenate([view["local_ids"], view["halo_ids"]]).astype(np.int32))
    Ws_d = [gu.to_dev(Ws[l], gu.ld_for(dims[l + 1], 4)) for l in range(L)]
    preds, keep = [None], []
    for l in range(1, L):
        pd = {k: gu.to_dev(omegas[l][k]) for k in omegas[l]}
        keep.append(pd)
        preds.append(sat.Predictor(pd["Wx"], pd["Wh"], pd["b"], pd["Wg"], dims[l], cfg["d_s"], tau))
    step = PartitionStep(view, dims, gu.to_dev(X, ld[0]), hist_d, ids_d, Ws_d, preds, gu.to_dev(y), tau,
                         transform_first=True)
    assert step.transform_first and step.AGG[L - 1] is None and step.dAGG[L - 1] is None
    ohist = [None] + [[t.copy() for t in hist[l]] for l in range(1, L)]
    n_l, n_h = view["n_local"], view["n_halo"]
    for t in range(2):
        order = [(t + s) % tau for s in range(tau)]
        step.forward_backward()
        gu.sync()
        st = oracle_step(oview, X, ohist, order, t % tau, Ws, omegas, y)
        st["y"] = y
        for l in range(L - 1):
            gu.assert_close(gu.to_host(step.AGG[l], dims[l]), st["AGG"][l], RTOL, "AGG %d" % l)
            gu.assert_close(gu.to_host(step.Hbar[l + 1], dims[l + 1])[:n_l], st["H"][l + 1], RTOL, "H %d" % (l + 1))
        # the transformed rows of ALL nodes, from the oracle's own layer input
        hbar = np.concatenate([st["H"][L - 1], st["halo_hat"][L - 1]]) if L >= 2 else \
            np.concatenate([X[view["local_ids"]], X[view["halo_ids"]]])
        zbar = orc.dense_fwd(hbar, Ws[L - 1], 0)[0]
        gu.assert_close(gu.to_host(step.Zbar, dims[L]), zbar, RTOL, "Zbar")
        gu.assert_close(gu.to_host(step.logits, dims[L]), st["H"][L], RTOL, "logits")
        assert abs(float(step.loss.item()) - st["loss"]) <= 2 * RTOL * abs(st["loss"])
        # G = [P_in | P_out]^T dH^(L): the oracle's transpose scatter with the halo rows asked for
        gL = orc.loss_and_grad(st["H"][L], y)[1]
        g_loc, g_halo = orc.spmm_bwd(oview, gL, want_halo=True)
        G = gu.to_host(step.G, dims[L])
        gu.assert_close(G[:n_l], g_loc, RTOL, "G local rows")
        if n_h:
            gu.assert_close(G[n_l:], g_halo, RTOL, "G halo rows")
        # the backward as a whole; the last layer has no dAGG in this order: the oracle's is used
        # in its place (check_backward only compares layers that have one)
        dW_gpu = [gu.to_host(step.dW[l], dims[l + 1]) for l in range(L)]
        dAGG_gpu = [None] + [gu.to_host(step.dAGG[l], dims[l]) if step.dAGG[l] is not None
                             else st["dAGG"][l] for l in range(1, L)]
        dH_gpu = [None] + [gu.to_host(step.dH[l], dims[l]) for l in range(1, L)]
        n_amb, n_bad = check_backward(gu, oview, st, dW_gpu, dAGG_gpu, dH_gpu, dims)
        print("[case] step %d ok: loss %.6f, %d rows excluded" % (t, st["loss"], n_bad), flush=True)
        assert n_bad < 0.02 * n_l


def test_transform_first_auto_rule():
    """"auto" turns the order on when the last layer narrows to half or less, never with
    gradient tables (the stale-gradient term is formed from dAGG)."""
    import paper_2308_13466_amd as sat
    from paper_2308_13466_amd.workload import build_workload
    assert build_workload("tiny").step.transform_first                      # 32 -> 8
    assert not build_workload("tiny", transform_first=False).step.transform_first
    assert not build_workload("tiny", grad_tables=True).step.transform_first
    assert not build_workload("scale_rows_small").step.transform_first      # 256 -> 172
