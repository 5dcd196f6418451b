"""Full-size parity in bf16 storage mode on the reduced Scale configuration
(papers100M-shaped: 128 features, 172 classes, mean degree 29, exponent 2.2, at
1/32 of the node count; one partition of 8 = 434 k local nodes): partition view
bit-exact, pull bit-exact, one whole step with sampled outputs against the
oracle chain that rounds every stored tensor to bfloat16. Tolerance 2e-2."""
import time

import numpy as np
import pytest

import sat_synth as syn
from oracle import sat_oracle as orc
from tests.test_gpu_large import _oracle_predict_rows, _sample_rows, _say

pytestmark = pytest.mark.gpu
RTOL = 2e-2


@pytest.fixture(scope="module")
def scale():
    import torch
    assert torch.cuda.is_available()
    import paper_2308_13466_amd as sat
    sat.lib()
    from paper_2308_13466_amd.workload import build_workload
    from tests import gpu_util as gu
    t0 = time.time()
    wl = build_workload("scale_small", log=_say)
    assert wl.dtype == "bf16"
    _say("workload built in %.0fs" % (time.time() - t0))
    return sat, gu, torch, wl


def test_scale_view_bit_exact(scale):
    sat, gu, torch, wl = scale
    _say("scale_small: partition view vs oracle, full size")
    g, v = wl.graph, wl.view
    ref = orc.partition_view(g.N, g.rowptr, g.col, g.part, wl.cfg["part"])
    for k in ("local_ids", "halo_ids", "rowptr", "split", "col", "h_colptr", "h_row"):
        assert np.array_equal(v[k], ref[k]), k
    for k in ("val", "h_val", "h_self"):
        assert np.array_equal(v[k].view(np.uint32), ref[k].view(np.uint32)), k


def test_scale_whole_step_sampled_bf16(scale):
    sat, gu, torch, wl = scale
    _say("scale_small bf16: one whole step; sampled outputs vs the oracle")
    v, step, dims = wl.view, wl.step, wl.dims
    n_l, n_h = v["n_local"], v["n_halo"]
    rng = np.random.default_rng(29)
    order = step.slot_order()
    step.forward_backward()
    gu.sync()

    def rows_of(t, idx, d):
        return t[torch.from_numpy(idx).to(gu.DEV)].float().cpu().numpy()[:, :d]

    # pull of the static halo features: bit-exact copy of the table rows
    halo_sample = np.sort(rng.choice(n_h, size=1024, replace=False))
    got = rows_of(step.Hbar[0], n_l + halo_sample, dims[0])
    assert np.array_equal(got, wl.X_host[wl.table_ids[n_l + halo_sample]][:, :dims[0]])
    halo_sample = np.unique(np.concatenate([halo_sample, np.argsort(np.diff(v["h_colptr"]))[-4:]]))
    for l in (1, 2):
        ref = orc.round_bf16(_oracle_predict_rows(wl, l, halo_sample, order))
        gu.assert_close(rows_of(step.Hbar[l], n_l + halo_sample, dims[l]), ref, RTOL,
                        "predicted halo rows, layer %d" % l)
    rows = _sample_rows(v, 1000, rng)
    Hbar0 = wl.X_host[wl.table_ids][:, :dims[0]]
    a0 = orc.round_bf16(orc.spmm_fwd_rows(v, Hbar0, rows))
    gu.assert_close(rows_of(step.AGG[0], rows, dims[0]), a0, RTOL, "AGG_0 rows")
    _, h1 = orc.dense_fwd(a0, wl.Ws[0], 1)
    h1 = orc.round_bf16(h1)
    gu.assert_close(rows_of(step.Hbar[1], rows, dims[1]), h1, RTOL, "H_1 rows")
    # push: slot 0 of each ring holds the bits the forward stored
    for l in (1, 2):
        tab = step.hist[l][0]
        assert torch.equal(tab[step.local_table_ids.long(), :dims[l]].view(torch.int16),
                           step.Hbar[l][:n_l, :dims[l]].contiguous().view(torch.int16))
    loss = float(step.loss.item())
    assert np.isfinite(loss) and 0.5 * np.log(dims[-1]) < loss < 4 * np.log(dims[-1])
    for l in range(3):
        assert torch.isfinite(step.dW[l][:, :dims[l + 1]]).all()
    # dW_2 = AGG_2^T dH_3 from the device's own stored operands is NOT checked here
    # (no oracle input may come from the device); the reduced tests cover it.
    step.forward_backward()
    gu.sync()
    assert np.isfinite(float(step.loss.item()))
