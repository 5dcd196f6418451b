"""GPU parity of the stale-gradient term of the appendix's SAT backward
(G_H = P_in^T D W^T + P_out^T D~^(t-1) W^T): the accumulate-pull
sat_history_gather_add, the halo output of sat_spmm_bwd routed through a
gradient table, and the two-partition exchange that must reproduce the
unpartitioned GCN's gradients when nothing is stale."""
import numpy as np
import pytest

import sat_synth as syn
from oracle import sat_oracle as orc
from tests.test_gpu_step import build_problem

pytestmark = pytest.mark.gpu
RTOL = 1e-5


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available()
    import paper_2308_13466_amd as sat
    sat.lib()
    from tests import gpu_util as gu
    return sat, gu, torch


@pytest.mark.parametrize("d,ld_t,ld_o", [(256, 256, 256), (100, 128, 104), (7, 8, 12), (1, 4, 4),
                                         (602, 608, 640)])
def test_gather_add_fp32(env, d, ld_t, ld_o):
    sat, gu, torch = env
    print("[case] gather_add fp32 d=%d" % d, flush=True)
    rng = np.random.default_rng(d)
    n_rows, n = 3000, 2500
    table = rng.standard_normal((n_rows, d)).astype(np.float32)
    out0 = rng.standard_normal((n, d)).astype(np.float32)
    ids = rng.integers(0, n_rows, size=n).astype(np.int32)        # with repeats
    ids[5], ids[17] = -3, n_rows + 2                              # bad ids add nothing
    out = gu.to_dev(out0, ld_o, pad_value=-7.0)
    sat.history_gather_add(gu.to_dev(table, ld_t), n_rows, ld_t, gu.to_dev(ids), n, d, out, ld_o,
                           stream=gu.stream_ptr())
    gu.sync()
    ok = (ids >= 0) & (ids < n_rows)
    ref = out0.astype(np.float64)
    ref[ok] += orc.history_gather(table, ids[ok]).astype(np.float64)
    got = out.cpu().numpy()
    # one fp32 addition per element: the correctly rounded sum
    assert np.array_equal(got[:, :d], ref.astype(np.float32))
    assert np.all(got[:, d:] == -7.0)


def test_gather_add_bf16_and_errors(env):
    sat, gu, torch = env
    print("[case] gather_add bf16", flush=True)
    from paper_2308_13466_amd import binding as B
    rng = np.random.default_rng(2)
    n_rows, n, d, ld = 1000, 900, 100, 104
    tb = syn.bf16_bits_from_f32(rng.standard_normal((n_rows, d)).astype(np.float32))
    ob = syn.bf16_bits_from_f32(rng.standard_normal((n, d)).astype(np.float32))
    ids = rng.integers(0, n_rows, size=n).astype(np.int32)
    out = gu.to_dev_bits(ob, ld, pad_bits=0x1234)
    sat.history_gather_add(gu.to_dev_bits(tb, ld), n_rows, ld, gu.to_dev(ids), n, d, out, ld,
                           dtype=B.BF16, stream=gu.stream_ptr())
    gu.sync()
    ref = orc.round_bf16(syn.f32_from_bf16_bits(ob).astype(np.float64)
                         + orc.history_gather(syn.f32_from_bf16_bits(tb), ids))
    got = gu.bits_to_host(out)
    assert np.array_equal(syn.f32_from_bf16_bits(got[:, :d]), ref.astype(np.float32))
    assert np.all(got[:, d:] == 0x1234)
    with pytest.raises(sat.SatError):           # rows must be 16-byte aligned for this call
        sat.history_gather_add(gu.to_dev_bits(tb, ld), n_rows, ld + 1, gu.to_dev(ids), n, d, out, ld,
                               dtype=B.BF16)


def test_two_partitions_exchange_reproduces_the_full_graph_backward(env):
    """Both partitions of the Tiny graph on the GPU, true embeddings in the history
    tables and the predictor bypassed, gradient tables exchanged between them: after
    the second step (same weights: nothing here updates them) every local row of
    dH^(1) equals the unpartitioned GCN's G_H^(1) and the partitions' dW add up to
    the full gradient (oracle: full_graph_backward)."""
    sat, gu, torch = env
    from paper_2308_13466_amd.step import PartitionStep
    print("[case] stale-gradient exchange, tiny, 2 partitions", flush=True)
    cfg, ss, g, X, Ws, omegas = build_problem("tiny")
    dims, L, tau = cfg["dims"], len(Ws), cfg["tau"]
    y_all = syn.labels_i32(ss["labels"], g.N, dims[-1])
    Hfull = orc.full_graph_gcn(g.N, g.rowptr, g.col, X, Ws)
    G_H, dW_full = orc.full_graph_backward(g.N, g.rowptr, g.col, X, Ws, y_all, g.part)
    ld = [gu.ld_for(d) for d in dims]
    # one pair of gradient tables shared by the two partitions (rows = global ids)
    gt = [None] + [[torch.zeros((g.N, ld[l]), dtype=torch.float32, device=gu.DEV) for _ in range(2)]
                   for l in range(1, L)]
    steps, views = [], []
    for m in (0, 1):
        view = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, m)
        views.append(view)
        hist_d = [None] + [[gu.to_dev(Hfull[l].astype(np.float32), ld[l]) for _ in range(tau)]
                           for l in range(1, L)]
        ids_d = gu.to_dev(np.concatenate([view["local_ids"], view["halo_ids"]]).astype(np.int32))
        Ws_d = [gu.to_dev(Ws[l], gu.ld_for(dims[l + 1], 4)) for l in range(L)]
        preds = [None] + [sat.Predictor(None, None, None, None, dims[l], 32, tau, bypass=True)
                          for l in range(1, L)]
        steps.append(PartitionStep(view, dims, gu.to_dev(X, ld[0]), hist_d, ids_d, Ws_d, preds,
                                   gu.to_dev(y_all[view["local_ids"]]), tau, grad_tables=gt))
    for t in range(2):
        for st in steps:
            st.forward_backward()
        gu.sync()
    dW_sum = [np.zeros_like(dW_full[l]) for l in range(L)]
    for m, st in enumerate(steps):
        v = views[m]
        got = gu.to_host(st.dH[1], dims[1])
        gu.assert_close(got, G_H[1][v["local_ids"]], 3e-5, "G_H^(1), partition %d" % m)
        for l in range(L):
            dW_sum[l] += gu.to_host(st.dW[l], dims[l + 1])
    for l in range(L):
        gu.assert_close(dW_sum[l], dW_full[l], 3e-5, "sum of the partitions' dW_%d" % l)


def test_step_with_gradient_tables_matches_oracle_chain(env):
    """One partition, two steps, seeded gradient tables standing in for what other
    partitions wrote: dH_in = P_in^T dAGG + table rows, the halo term lands in the
    write table's halo rows bit for bit as the step computed it, every other row
    of the tables is untouched."""
    sat, gu, torch = env
    from paper_2308_13466_amd.step import PartitionStep
    print("[case] step with gradient tables, tiny", flush=True)
    cfg, ss, g, X, Ws, omegas = build_problem("tiny")
    dims, L, tau = cfg["dims"], len(Ws), cfg["tau"]
    view = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, 0)
    oview = orc.partition_view(g.N, g.rowptr, g.col, g.part, 0)
    n_l = view["n_local"]
    y = syn.labels_i32(ss["labels"], n_l, dims[-1])
    Hfull = orc.full_graph_gcn(g.N, g.rowptr, g.col, X, Ws)
    ld = [gu.ld_for(d) for d in dims]
    rng = np.random.default_rng(9)
    gt_host = [None] + [[(1e-3 * rng.standard_normal((g.N, dims[l]))).astype(np.float32)
                         for _ in range(2)] for l in range(1, L)]
    gt = [None] + [[gu.to_dev(t, ld[l], pad_value=0.0) for t in gt_host[l]] for l in range(1, L)]
    hist = [None] + [[Hfull[l].astype(np.float32) for _ in range(tau)] for l in range(1, L)]
    hist_d = [None] + [[gu.to_dev(t, ld[l]) for t in hist[l]] for l in range(1, L)]
    ids_d = gu.to_dev(np.concatenate([view["local_ids"], view["halo_ids"]]).astype(np.int32))
    Ws_d = [gu.to_dev(Ws[l], gu.ld_for(dims[l + 1], 4)) for l in range(L)]
    preds = [None] + [sat.Predictor(None, None, None, None, dims[l], 32, tau, bypass=True)
                      for l in range(1, L)]
    step = PartitionStep(view, dims, gu.to_dev(X, ld[0]), hist_d, ids_d, Ws_d, preds, gu.to_dev(y), tau,
                         grad_tables=gt)
    for t in range(2):
        step.forward_backward()
        gu.sync()
        rd, wr = t % 2, (t + 1) % 2
        halo_hat = [None] + [hist[l][-1][oview["halo_ids"]] for l in range(1, L)]
        stale = [None] + [gt_host[l][rd][oview["local_ids"]] for l in range(1, L)]
        st = orc.partition_step(oview, X[oview["local_ids"]], X[oview["halo_ids"]], halo_hat, Ws, y,
                                stale_grad=stale)
        for l in range(1, L):
            gu.assert_close(gu.to_host(step.dH[l], dims[l]), st["dH_in"][l], RTOL, "dH_in %d" % l)
            gu.assert_close(gu.to_host(step.dH_halo[l], dims[l]), st["dH_halo"][l], RTOL,
                            "dH_halo %d" % l)
            tab = gt[l][wr].cpu().numpy()[:, :dims[l]]
            assert np.array_equal(tab[oview["halo_ids"]], gu.to_host(step.dH_halo[l], dims[l]))
            others = np.setdiff1d(np.arange(g.N), oview["halo_ids"])
            assert np.array_equal(tab[others], gt_host[l][wr][others])
            gt_host[l][wr][oview["halo_ids"]] = st["dH_halo"][l].astype(np.float32)
        for l in range(L):
            gu.assert_close(gu.to_host(step.dW[l], dims[l + 1]), st["dW"][l], RTOL, "dW %d" % l)
        # push of the forward into the history ring is unchanged by the extra calls
        for l in range(1, L):
            hist[l][t % tau][oview["local_ids"]] = st["H"][l].astype(np.float32)
