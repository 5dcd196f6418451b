"""Full-size parity of the graph attention backbone: the benchmark's workload
(Large) in the launch configuration `bench.py --backbone gat` times. The oracle
computes sampled outputs one by one: a row of the forward needs the row's own
entries only; a row of dZ needs every local row that has it as a neighbour, so
the oracle's backward is restricted to the union of those rows."""
import time

import numpy as np
import pytest

import sat_synth as syn
from oracle import gat_oracle as gat

pytestmark = pytest.mark.gpu
RTOL = 1e-5
SLOPE = 0.2


def _say(msg):
    print("[case] " + msg, flush=True)


@pytest.fixture(scope="module")
def large_gat():
    import torch
    assert torch.cuda.is_available()
    import paper_2308_13466_amd as sat
    sat.lib()
    from paper_2308_13466_amd.workload import build_workload
    from tests import gpu_util as gu
    t0 = time.time()
    wl = build_workload("large", log=_say, backbone="gat")
    _say("workload built in %.0fs" % (time.time() - t0))
    return sat, gu, torch, wl


def _sample_rows(view, n, rng):
    n_l = view["n_local"]
    deg = np.diff(view["rowptr"])
    rows = set(int(r) for r in rng.choice(n_l, size=n, replace=False))
    rows.update(int(r) for r in np.argsort(deg)[-4:])      # the cooperative long-row path
    rows.update([0, n_l - 1])
    return np.array(sorted(rows), dtype=np.int64)


def test_gat_calls_sampled_at_full_size(large_gat):
    sat, gu, torch, wl = large_gat
    v, step = wl.view, wl.step
    n_l, n_h = v["n_local"], v["n_halo"]
    n_bar, K, F = n_l + n_h, 4, 64
    d = K * F
    _say("gat calls at full size: n_bar=%d, %d heads x %d" % (n_bar, K, F))
    rng = np.random.default_rng(5)
    Z = syn.normal_f32(np.random.SeedSequence(55), n_bar, d)
    a_dst, a_src = syn.attention_vectors_f32(np.random.SeedSequence(56), K, F)
    Z_d = gu.to_dev(Z)
    a_dst_d, a_src_d = gu.to_dev(a_dst.reshape(-1)), gu.to_dev(a_src.reshape(-1))
    st = gu.stream_ptr()
    # scores: every row
    el_d = torch.empty((n_l, K), dtype=torch.float32, device=gu.DEV)
    er_d = torch.empty((n_bar, K), dtype=torch.float32, device=gu.DEV)
    sat.gat_scores(Z_d, d, n_bar, n_l, K, F, a_dst_d, a_src_d, el_d, er_d, stream=st)
    gu.sync()
    el_ref, er_ref = gat.gat_scores(Z, a_dst, a_src)
    gu.assert_close(el_d.cpu().numpy(), el_ref[:n_l], RTOL, "el")
    gu.assert_close(er_d.cpu().numpy(), er_ref, RTOL, "er")
    el32, er32 = el_ref[:n_l].astype(np.float32), er_ref.astype(np.float32)
    el64, er64 = el32.astype(np.float64), er32.astype(np.float64)
    el_d, er_d = gu.to_dev(el32), gu.to_dev(er32)
    # forward: sampled rows
    H_d = torch.empty((n_l, d), dtype=torch.float32, device=gu.DEV)
    stats_d = torch.empty((n_l, K, 2), dtype=torch.float32, device=gu.DEV)
    sat.gat_aggregate_fwd(step.pv, Z_d, d, K, F, el_d, er_d, SLOPE, sat.ACT_IDENTITY, H_d, d, stats_d,
                          stream=st)
    gu.sync()
    rows = _sample_rows(v, 3000, rng)
    ref = gat.gat_aggregate_fwd(v, Z, el64, er64, SLOPE, rows=rows)
    got = H_d[torch.from_numpy(rows).to(gu.DEV)].cpu().numpy()
    gu.assert_close(got, ref, RTOL, "aggregated rows")
    # backward: dZ of sampled local and halo rows; the oracle's backward over every local
    # row that has one of them as a neighbour (and the sampled local rows themselves)
    dH = syn.normal_f32(np.random.SeedSequence(57), n_l, d, std=1.0 / np.sqrt(n_l))
    dH_d = gu.to_dev(dH)
    wsb = sat.gat_aggregate_bwd_workspace_bytes(n_l, n_h, K, F, sat.F32)
    ws = gu.workspace(wsb)
    dZ_d = torch.empty((n_bar, d), dtype=torch.float32, device=gu.DEV)
    da1 = torch.empty(d, dtype=torch.float32, device=gu.DEV)
    da2 = torch.empty(d, dtype=torch.float32, device=gu.DEV)
    sat.gat_aggregate_bwd(step.pv, Z_d, d, K, F, el_d, er_d, stats_d, SLOPE, sat.ACT_IDENTITY, dH_d, d,
                          None, 0, a_dst_d, a_src_d, dZ_d, d, da1, da2, workspace=ws,
                          workspace_bytes=wsb, stream=st)
    gu.sync()
    deg = np.diff(v["rowptr"])
    loc_j = np.unique(np.concatenate([rng.choice(n_l, size=150, replace=False), np.argsort(deg)[-2:]]))
    hdeg = np.diff(v["h_colptr"])
    halo_j = np.unique(np.concatenate([rng.choice(n_h, size=150, replace=False), np.argsort(hdeg)[-2:]]))
    need = [loc_j]
    for j in loc_j:
        need.append(v["col"][v["rowptr"][j]:v["split"][j]].astype(np.int64))
    for u in halo_j:
        need.append(v["h_row"][v["h_colptr"][u]:v["h_colptr"][u + 1]].astype(np.int64))
    src_rows = np.unique(np.concatenate(need))
    _say("oracle backward over %d source rows for %d sampled rows of dZ" % (
        len(src_rows), len(loc_j) + len(halo_j)))
    dZa, d_el, d_er = gat.gat_aggregate_bwd(v, Z, el64, er64, SLOPE, dH.astype(np.float64), rows=src_rows)
    js = np.concatenate([loc_j, n_l + halo_j])
    A = np.zeros((len(js), K, F))
    A[:len(loc_j)] = d_el[loc_j][:, :, None] * a_dst[None].astype(np.float64)
    B = d_er[js][:, :, None] * a_src[None].astype(np.float64)
    A, B = A.reshape(len(js), d), B.reshape(len(js), d)
    ref = dZa[js] + A + B
    got = dZ_d[torch.from_numpy(js).to(gu.DEV)].cpu().numpy().astype(np.float64)
    mag = np.abs(dZa[js]) + np.abs(A) + np.abs(B)
    rms = np.sqrt(np.mean(ref * ref))
    assert np.all(np.abs(got - ref) <= RTOL * (mag + rms)), "dZ rows: worst %g" % float(
        (np.abs(got - ref) / (mag + rms)).max())
    assert torch.isfinite(da1).all() and torch.isfinite(da2).all()


def test_gat_whole_step_sampled(large_gat):
    sat, gu, torch, wl = large_gat
    _say("one whole GAT step in the benchmark's configuration; sampled outputs vs the oracle")
    v, step, dims = wl.view, wl.step, wl.dims
    n_l = v["n_local"]
    rng = np.random.default_rng(23)
    assert step.t == 0
    step.forward_backward()
    gu.sync()
    rows = _sample_rows(v, 800, rng)
    K = step.heads[0]
    a_dst, a_src = wl.attn[0]
    # layer 0 from the original features: Z of the sampled rows and of all their neighbours
    nb = np.unique(np.concatenate([v["col"][v["rowptr"][i]:v["rowptr"][i + 1]].astype(np.int64)
                                   for i in rows] + [rows]))
    Znb = wl.X_host[wl.table_ids[nb]][:, :dims[0]].astype(np.float64) @ wl.Ws[0].astype(np.float64)
    Z_d = step.Z[0][torch.from_numpy(nb).to(gu.DEV)].cpu().numpy()[:, :dims[1]]
    gu.assert_close(Z_d, Znb, RTOL, "Z_0 rows")
    pos = {int(j): k for k, j in enumerate(nb)}
    el, er = gat.gat_scores(Znb, a_dst, a_src)
    ref = np.zeros((len(rows), dims[1]))
    F = dims[1] // K
    for r, i in enumerate(rows):
        cols = v["col"][v["rowptr"][i]:v["rowptr"][i + 1]]
        idx = np.array([pos[int(c)] for c in cols])
        s = el[pos[int(i)]][None, :] + er[idx]
        e = gat.leaky_relu(s, SLOPE)
        p = np.exp(e - e.max(axis=0, keepdims=True))
        alpha = p / p.sum(axis=0, keepdims=True)
        ref[r] = np.einsum("jk,jkf->kf", alpha, Znb[idx].reshape(-1, K, F)).reshape(-1)
    ref = np.maximum(ref, 0.0)
    got = step.Hbar[1][torch.from_numpy(rows).to(gu.DEV)].cpu().numpy()[:, :dims[1]]
    gu.assert_close(got, ref, 3 * RTOL, "H_1 rows")
    # push: slot 0 of each ring now holds exactly the forward's local rows
    for l in (1, 2):
        tab = step.hist[l][0]
        assert torch.equal(tab[step.local_table_ids.long(), :dims[l]], step.Hbar[l][:n_l, :dims[l]])
    assert np.isfinite(float(step.loss.item()))
    for l in range(3):
        assert torch.isfinite(step.dW[l][:, :dims[l + 1]]).all()
        assert torch.isfinite(step.da_dst[l]).all() and torch.isfinite(step.da_src[l]).all()
    step.forward_backward()
    gu.sync()
    assert np.isfinite(float(step.loss.item()))
