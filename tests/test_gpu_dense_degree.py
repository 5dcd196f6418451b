"""Full-size parity on the Dense-degree configuration (233k-node SBM, mean degree
about 490, 602 input features, 2-layer GCN 602 -> 256 -> 41): partition view
bit-exact, wide-row aggregation (three 16-byte accumulators per lane) on
sampled rows, and one whole step with sampled outputs against the oracle."""
import time

import numpy as np
import pytest

import sat_synth as syn
from oracle import sat_oracle as orc
from tests.test_gpu_large import _oracle_predict_rows, _sample_rows, _say

pytestmark = pytest.mark.gpu
RTOL = 1e-5


@pytest.fixture(scope="module")
def dense():
    import torch
    assert torch.cuda.is_available()
    import paper_2308_13466_amd as sat
    sat.lib()
    from paper_2308_13466_amd.workload import build_workload
    from tests import gpu_util as gu
    t0 = time.time()
    wl = build_workload("dense", log=_say)
    _say("workload built in %.0fs" % (time.time() - t0))
    return sat, gu, torch, wl


def test_dense_view_bit_exact(dense):
    sat, gu, torch, wl = dense
    _say("dense-degree: partition view vs oracle, full size")
    g, v = wl.graph, wl.view
    ref = orc.partition_view(g.N, g.rowptr, g.col, g.part, wl.cfg["part"])
    for k in ("local_ids", "halo_ids", "rowptr", "split", "col", "h_colptr", "h_row"):
        assert np.array_equal(v[k], ref[k]), k
    for k in ("val", "h_val", "h_self"):
        assert np.array_equal(v[k].view(np.uint32), ref[k].view(np.uint32)), k
    assert v["n_halo"] > 6 * v["n_local"]          # large halo, as the configuration says


def test_dense_whole_step_sampled(dense):
    sat, gu, torch, wl = dense
    _say("dense-degree: one whole step; sampled outputs vs the oracle")
    v, step, dims = wl.view, wl.step, wl.dims
    n_l, n_h = v["n_local"], v["n_halo"]
    rng = np.random.default_rng(23)
    order = step.slot_order()
    step.forward_backward()
    gu.sync()
    halo_sample = np.sort(rng.choice(n_h, size=512, replace=False))
    ref = _oracle_predict_rows(wl, 1, halo_sample, order)
    got = step.Hbar[1][torch.from_numpy(n_l + halo_sample).to(gu.DEV)].cpu().numpy()[:, :dims[1]]
    gu.assert_close(got, ref, RTOL, "predicted halo rows")
    rows = _sample_rows(v, 300, rng)
    Hbar0 = wl.X_host[wl.table_ids][:, :dims[0]]
    a0 = orc.spmm_fwd_rows(v, Hbar0, rows)
    ridx = torch.from_numpy(rows).to(gu.DEV)
    gu.assert_close(step.AGG[0][ridx].cpu().numpy()[:, :dims[0]], a0, RTOL, "AGG_0 rows (d = 602)")
    _, h1 = orc.dense_fwd(a0, wl.Ws[0], 1)
    gu.assert_close(step.Hbar[1][ridx].cpu().numpy()[:, :dims[1]], h1, RTOL, "H_1 rows")
    tab = step.hist[1][0]
    assert torch.equal(tab[step.local_table_ids.long(), :dims[1]], step.Hbar[1][:n_l, :dims[1]])
    assert np.isfinite(float(step.loss.item()))
    # the last layer (256 -> 41) runs as P (Hbar W) in this configuration: its transform over
    # all rows, both aggregations at 41 columns on the dense rows, dW over all rows
    from tests.last_layer_util import check_last_layer_transform_first
    check_last_layer_transform_first(gu, torch, wl, rows[:64], halo_sample[:64], RTOL, say=_say)
