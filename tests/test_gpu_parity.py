"""GPU parity: every exported compute call against the CPU oracle, element by
element, on identical seeded inputs. Index and copy work is bit-exact; fp32
results are held to 1e-5 (see gpu_util.assert_close for the rule)."""
import numpy as np
import pytest

import sat_synth as syn
from oracle import sat_oracle as orc

pytestmark = pytest.mark.gpu

RTOL = 1e-5


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2308_13466_amd as sat
    sat.lib()                       # raises if libsat.so is missing: no fallback
    from tests import gpu_util as gu
    return sat, gu, torch


def _say(msg):
    print("[case] " + msg, flush=True)


def _graph(kind, seed=0):
    if kind == "tiny":
        cfg = syn.get_config("tiny")
        g = syn.make_graph(cfg, np.random.default_rng(syn.substreams(seed)["graph"]))
    elif kind == "powerlaw":
        g = syn.chung_lu_planted_graph(30_000, 4, 13.0, 2.1, 0.15, np.random.default_rng(seed))
    elif kind == "powerlaw_big":    # 78k local + halo rows in partition 0
        g = syn.chung_lu_planted_graph(170_000, 4, 13.0, 2.1, 0.15, np.random.default_rng(seed))
    elif kind == "onepart":
        g = syn.chung_lu_planted_graph(3_000, 1, 9.0, 2.3, 0.0, np.random.default_rng(seed))
    elif kind == "hub":
        # star-heavy graph: node 0 of partition 0 touches 12,000 nodes, half of them outside
        N = 16_000
        rng = np.random.default_rng(seed)
        u = np.concatenate([np.zeros(12_000, np.int64), rng.integers(0, N, 20_000)])
        v = np.concatenate([rng.choice(np.arange(1, N), 12_000, replace=False),
                            rng.integers(0, N, 20_000)])
        from sat_synth.graphs import _csr_from_pairs, _contiguous_parts, Graph
        rowptr, col = _csr_from_pairs(N, u, v)
        part, _ = _contiguous_parts(N, 2)
        g = Graph(N, rowptr, col, part, 2)
    else:
        raise ValueError(kind)
    return g


# ---------------------------------------------------------------- gather / push
@pytest.mark.parametrize("d,ld_t,ld_o", [(1, 1, 1), (3, 3, 5), (4, 4, 8), (64, 64, 64),
                                         (100, 128, 100), (256, 256, 288), (602, 608, 640),
                                         (7, 9, 11)])
def test_history_gather_bit_exact(env, d, ld_t, ld_o):
    sat, gu, torch = env
    _say("gather d=%d ld_t=%d ld_o=%d" % (d, ld_t, ld_o))
    rng = np.random.default_rng(d)
    n_rows, n = 5000, 3333
    table = rng.standard_normal((n_rows, ld_t)).astype(np.float32)
    ids = rng.integers(0, n_rows, size=n).astype(np.int32)
    ids[:5] = [0, n_rows - 1, 7, 7, 0]
    ref = orc.history_gather(table, ids)[:, :d]
    t_d, i_d = gu.to_dev(table), gu.to_dev(ids)
    out = torch.full((n, ld_o), -7.0, dtype=torch.float32, device=gu.DEV)
    sat.history_gather(t_d, n_rows, ld_t, i_d, n, d, out, ld_o, stream=gu.stream_ptr())
    gu.sync()
    got = out.cpu().numpy()
    assert np.array_equal(got[:, :d].view(np.uint32), ref.view(np.uint32))
    assert np.all(got[:, d:] == -7.0)          # padding columns untouched


@pytest.mark.parametrize("d,ld_t,ld_h", [(1, 2, 1), (32, 32, 32), (100, 128, 128),
                                         (256, 256, 256), (41, 44, 48), (5, 7, 6)])
def test_history_push_bit_exact_and_roundtrip(env, d, ld_t, ld_h):
    sat, gu, torch = env
    _say("push d=%d ld_t=%d ld_h=%d" % (d, ld_t, ld_h))
    rng = np.random.default_rng(100 + d)
    n_rows, n = 4000, 1777
    table = rng.standard_normal((n_rows, ld_t)).astype(np.float32)
    ids = rng.permutation(n_rows)[:n].astype(np.int32)
    H = rng.standard_normal((n, ld_h)).astype(np.float32)
    ref = orc.history_push(table.copy(), ids, H[:, :d])
    t_d, i_d, h_d = gu.to_dev(table), gu.to_dev(ids), gu.to_dev(H)
    sat.history_push(t_d, n_rows, ld_t, i_d, n, d, h_d, ld_h, stream=gu.stream_ptr())
    gu.sync()
    got = t_d.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
    back = torch.zeros((n, ld_h), dtype=torch.float32, device=gu.DEV)
    sat.history_gather(t_d, n_rows, ld_t, i_d, n, d, back, ld_h, stream=gu.stream_ptr())
    gu.sync()
    assert np.array_equal(back.cpu().numpy()[:, :d].view(np.uint32), H[:, :d].view(np.uint32))


def test_gather_push_edge_cases(env):
    sat, gu, torch = env
    _say("gather/push empty and out-of-range ids")
    table = torch.arange(40, dtype=torch.float32, device=gu.DEV).reshape(10, 4)
    out = torch.full((3, 4), -1.0, device=gu.DEV)
    ids = gu.to_dev(np.array([2, 99, -5], dtype=np.int32))
    sat.history_gather(table, 10, 4, ids, 0, 4, out, 4)           # n = 0
    sat.history_gather(table, 10, 4, ids, 3, 4, out, 4)           # bad ids are skipped
    gu.sync()
    got = out.cpu().numpy()
    assert np.array_equal(got[0], [8, 9, 10, 11]) and np.all(got[1:] == -1.0)
    with pytest.raises(sat.SatError):
        sat.history_gather(table, 10, 4, ids, 3, 8, out, 4)       # ld < d


# ------------------------------------------------------------------------ SpMM
@pytest.mark.parametrize("kind,d", [("tiny", 64), ("tiny", 32), ("tiny", 8), ("tiny", 1),
                                    ("powerlaw", 128), ("powerlaw", 256), ("powerlaw", 100),
                                    ("powerlaw", 40), ("hub", 256), ("hub", 64),
                                    ("onepart", 602), ("tiny", 1030), ("powerlaw", 3)])
def test_spmm_fwd_bwd_parity(env, kind, d):
    sat, gu, torch = env
    _say("spmm %s d=%d" % (kind, d))
    g = _graph(kind)
    v = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, 0)
    n_l, n_h = v["n_local"], v["n_halo"]
    rng = np.random.default_rng(d)
    Hbar = rng.standard_normal((n_l + n_h, d)).astype(np.float32)
    G = rng.standard_normal((n_l, d)).astype(np.float32)
    ld_in, ld_out = gu.ld_for(d, 4), gu.ld_for(d, 32)
    pv = gu.upload_view(v)
    Hb_d, G_d = gu.to_dev(Hbar, ld_in), gu.to_dev(G, ld_in)
    agg = gu.dev_empty(n_l, ld_out, fill=-3.0)
    sat.spmm_fwd(pv, Hb_d, ld_in, d, agg, ld_out, stream=gu.stream_ptr())
    dl = gu.dev_empty(n_l, ld_out, fill=-3.0)
    dh = gu.dev_empty(max(n_h, 1), ld_out, fill=-3.0)
    sat.spmm_bwd(pv, G_d, ld_in, d, dl, ld_out, dh if n_h else None, ld_out, stream=gu.stream_ptr())
    gu.sync()
    gu.assert_close(gu.to_host(agg, d), orc.spmm_fwd(v, Hbar), RTOL, "spmm_fwd")
    assert np.all(agg.cpu().numpy()[:, d:] == -3.0)
    rl, rh = orc.spmm_bwd(v, G, want_halo=True)
    gu.assert_close(gu.to_host(dl, d), rl, RTOL, "spmm_bwd local")
    if n_h:
        gu.assert_close(gu.to_host(dh, d)[:n_h], rh, RTOL, "spmm_bwd halo")
    # local-only variant must give the same local rows
    dl2 = gu.dev_empty(n_l, ld_out)
    sat.spmm_bwd(pv, G_d, ld_in, d, dl2, ld_out, stream=gu.stream_ptr())
    gu.sync()
    assert np.array_equal(gu.to_host(dl2, d), gu.to_host(dl, d))


def test_spmm_sqrt_degree_fixed_vector_on_gpu(env):
    sat, gu, torch = env
    _say("spmm closed form A_hat sqrt(d) = sqrt(d)")
    g = _graph("powerlaw", seed=3)
    v = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, 1)
    sd = np.sqrt(1.0 + np.diff(g.rowptr)).astype(np.float32)
    ids = np.concatenate([v["local_ids"], v["halo_ids"]])
    x = np.repeat(sd[ids][:, None], 4, axis=1)
    agg = gu.dev_empty(v["n_local"], 4)
    sat.spmm_fwd(gu.upload_view(v), gu.to_dev(x), 4, 4, agg, 4)
    gu.sync()
    np.testing.assert_allclose(agg.cpu().numpy()[:, 0], sd[v["local_ids"]], rtol=2e-6)


def test_spmm_rejects_misaligned(env):
    sat, gu, torch = env
    g = _graph("tiny")
    v = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, 0)
    pv = gu.upload_view(v)
    x = gu.dev_empty(v["n_local"] + v["n_halo"], 6)
    y = gu.dev_empty(v["n_local"], 8)
    with pytest.raises(sat.SatError) as e:
        sat.spmm_fwd(pv, x, 6, 6, y, 8)
    assert e.value.status == -3


# ----------------------------------------------------------------------- dense
@pytest.mark.parametrize("n,d_in,d_out,act", [(2048, 64, 32, 1), (2051, 32, 8, 0),
                                              (1000, 128, 256, 1), (777, 256, 256, 1),
                                              (513, 256, 40, 0), (300, 602, 256, 1),
                                              (129, 100, 47, 0), (5, 4, 4, 1), (1, 1, 1, 0),
                                              # many rows onto few columns: the weights-in-LDS forward
                                              # kernel and the 64-column tile of the weight gradient
                                              (20011, 256, 47, 0), (9000, 64, 8, 1), (8192, 128, 64, 1),
                                              (8200, 256, 33, 0), (9001, 40, 17, 1),
                                              # many rows onto many columns: the weights-in-registers
                                              # kernel (whole 32-row tiles) plus the tile GEMM for the
                                              # last rows; full and ragged K and N, with and without mask
                                              (65606, 256, 256, 1), (66001, 100, 256, 1),
                                              (65600, 256, 200, 0), (70000, 128, 256, 1),
                                              (65540, 200, 136, 1), (65537, 64, 160, 0)])
def test_dense_fwd_bwd_parity(env, n, d_in, d_out, act):
    sat, gu, torch = env
    _say("dense n=%d %d->%d act=%d" % (n, d_in, d_out, act))
    rng = np.random.default_rng(n + d_in)
    A = rng.standard_normal((n, d_in)).astype(np.float32)
    W = syn.glorot_uniform_f32(np.random.SeedSequence(n), d_in, d_out)
    dH = rng.standard_normal((n, d_out)).astype(np.float32)
    ld_a, ld_w, ld_h = gu.ld_for(d_in, 4), gu.ld_for(d_out, 4), gu.ld_for(d_out, 32)
    A_d, W_d, dH_d = gu.to_dev(A, ld_a), gu.to_dev(W, ld_w), gu.to_dev(dH, ld_h)
    H_d = gu.dev_empty(n, ld_h, fill=-3.0)
    sat.dense_fwd(A_d, ld_a, n, d_in, d_out, W_d, ld_w, act, H_d, ld_h, stream=gu.stream_ptr())
    gu.sync()
    Z, H = orc.dense_fwd(A, W, act)
    gu.assert_close(gu.to_host(H_d, d_out), H, RTOL, "dense_fwd")
    assert np.all(H_d.cpu().numpy()[:, d_out:] == -3.0)
    # backward: the mask comes from the forward output; feed the oracle's H
    # rounded to fp32 so both sides decide relu' on the same numbers
    H32 = H.astype(np.float32)
    Hm_d = gu.to_dev(H32, ld_h)
    dW_d = gu.dev_empty(d_in, ld_w, fill=-3.0)
    dA_d = gu.dev_empty(n, ld_a, fill=-3.0)
    wsb = sat.dense_bwd_workspace_bytes(n, d_in, d_out)
    ws = gu.workspace(wsb)
    sat.dense_bwd(dH_d, ld_h, Hm_d, ld_h, A_d, ld_a, W_d, ld_w, n, d_in, d_out, act, dW_d, ld_w,
                  dA_d, ld_a, workspace=ws, workspace_bytes=wsb, stream=gu.stream_ptr())
    gu.sync()
    dW, dA, _ = orc.dense_bwd(dH, H32, A, W, act)
    gu.assert_close(gu.to_host(dW_d, d_out), dW, RTOL, "dW")
    gu.assert_close(gu.to_host(dA_d, d_in), dA, RTOL, "dAGG")
    assert np.all(dW_d.cpu().numpy()[:, d_out:] == -3.0)
    # run-to-run identical (fixed-order reduction), and dAGG may be skipped
    dW2 = gu.dev_empty(d_in, ld_w)
    sat.dense_bwd(dH_d, ld_h, Hm_d, ld_h, A_d, ld_a, W_d, ld_w, n, d_in, d_out, act, dW2, ld_w,
                  None, 0, workspace=ws, workspace_bytes=wsb, stream=gu.stream_ptr())
    gu.sync()
    assert np.array_equal(gu.to_host(dW2, d_out), gu.to_host(dW_d, d_out))


def test_dense_bwd_workspace_is_checked(env):
    sat, gu, torch = env
    x = gu.dev_empty(64, 32, fill=0.0)
    w = gu.dev_empty(32, 32, fill=0.0)
    with pytest.raises(sat.SatError) as e:
        sat.dense_bwd(x, 32, x, 32, x, 32, w, 32, 64, 32, 32, 1, w, 32, x, 32,
                      workspace=None, workspace_bytes=0)
    assert e.value.status == -4


# ------------------------------------------------------------------------ loss
@pytest.mark.parametrize("n,C", [(2048, 8), (1001, 40), (333, 47), (70, 172), (1, 2), (500, 128),
                                 (301, 256), (203, 300), (37, 65)])
def test_loss_grad_parity(env, n, C):
    sat, gu, torch = env
    _say("loss n=%d C=%d" % (n, C))
    rng = np.random.default_rng(C)
    HL = (3.0 * rng.standard_normal((n, C))).astype(np.float32)
    y = rng.integers(0, C, size=n).astype(np.int32)
    ld = gu.ld_for(C, 4)
    g_d = gu.dev_empty(n, ld, fill=-3.0)
    loss_d = torch.zeros(1, dtype=torch.float32, device=gu.DEV)
    wsb = sat.loss_workspace_bytes(n)
    ws = gu.workspace(wsb)
    sat.loss_grad(gu.to_dev(HL, ld), ld, n, C, gu.to_dev(y), g_d, ld, loss=loss_d, workspace=ws,
                  workspace_bytes=wsb, stream=gu.stream_ptr())
    gu.sync()
    loss, g = orc.loss_and_grad(HL, y)
    gu.assert_close(gu.to_host(g_d, C), g, RTOL, "dH^(L)")
    assert torch.all(g_d[:, C:] == -3.0)          # padding columns untouched
    assert abs(float(loss_d.item()) - loss) <= RTOL * abs(loss) * 2


@pytest.mark.parametrize("n,C,ld", [(400, 47, 47), (129, 300, 301), (64, 130, 131), (1000, 1100, 1100)])
def test_loss_grad_rows_not_on_16_byte_boundaries(env, n, C, ld):
    """Leading dimensions that do not put rows on 16-byte boundaries (and more classes than the
    register-resident kernels hold) take the element-wise kernels."""
    sat, gu, torch = env
    _say("loss n=%d C=%d ld=%d" % (n, C, ld))
    rng = np.random.default_rng(C + ld)
    HL = (3.0 * rng.standard_normal((n, C))).astype(np.float32)
    y = rng.integers(0, C, size=n).astype(np.int32)
    g_d = gu.dev_empty(n, ld, fill=-3.0)
    loss_d = torch.zeros(1, dtype=torch.float32, device=gu.DEV)
    wsb = sat.loss_workspace_bytes(n)
    ws = gu.workspace(wsb)
    sat.loss_grad(gu.to_dev(HL, ld), ld, n, C, gu.to_dev(y), g_d, ld, loss=loss_d, workspace=ws,
                  workspace_bytes=wsb, stream=gu.stream_ptr())
    gu.sync()
    loss, g = orc.loss_and_grad(HL, y)
    gu.assert_close(gu.to_host(g_d, C), g, RTOL, "dH^(L)")
    assert torch.all(g_d[:, C:] == -3.0)
    assert abs(float(loss_d.item()) - loss) <= RTOL * abs(loss) * 2


# ------------------------------------------------------------------- predictor
@pytest.mark.parametrize("kind,d,d_s,tau,use_ids", [("tiny", 32, 32, 2, False),
                                                    ("tiny", 32, 32, 1, True),
                                                    ("powerlaw", 256, 64, 2, True),
                                                    ("powerlaw", 100, 64, 3, False),
                                                    ("tiny", 64, 128, 2, True),
                                                    ("hub", 40, 32, 2, True)])
def test_predict_parity(env, kind, d, d_s, tau, use_ids):
    sat, gu, torch = env
    _say("predict %s d=%d d_s=%d tau=%d ids=%s" % (kind, d, d_s, tau, use_ids))
    g = _graph(kind)
    v = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, 0)
    n_l, n_h = v["n_local"], v["n_halo"]
    n_bar = n_l + n_h
    rng = np.random.default_rng(d + d_s)
    p = syn.predictor_params_f32(np.random.SeedSequence(d_s), d, d_s)
    ld = gu.ld_for(d, 32)
    if use_ids:      # slots are whole tables indexed by global node id
        ids = np.concatenate([v["local_ids"], v["halo_ids"]]).astype(np.int32)
        n_rows = g.N
    else:            # slots are already in local-then-halo order
        ids = None
        n_rows = n_bar
    base = np.maximum(rng.standard_normal((n_rows, d)), 0).astype(np.float32)
    tables = [(base + 0.05 * rng.standard_normal((n_rows, d))).astype(np.float32)
              for _ in range(tau)]
    win = [t[ids] if use_ids else t for t in tables]          # oracle sees the window
    ref = orc.predict(v, p, win)
    pv = gu.upload_view(v)
    pd = {k: gu.to_dev(p[k]) for k in p}
    w = sat.Predictor(pd["Wx"], pd["Wh"], pd["b"], pd["Wg"], d, d_s, tau)
    slots_d = [gu.to_dev(t, ld) for t in tables]
    Hbar = gu.dev_empty(n_bar, ld, fill=-3.0)
    wsb = sat.predict_workspace_bytes(n_l, n_h, d, d_s, tau)
    ws = gu.workspace(wsb)
    ids_d = gu.to_dev(ids) if use_ids else None
    sat.predict(pv, w, slots_d, n_rows, ld, ids_d, Hbar, ld, workspace=ws, workspace_bytes=wsb,
                stream=gu.stream_ptr())
    gu.sync()
    got = Hbar.cpu().numpy()
    assert np.all(got[:n_l] == -3.0) and np.all(got[:, d:] == -3.0)     # only halo rows written
    gu.assert_close(got[n_l:, :d], ref, RTOL, "predict")
    # identity cases: bypass, and Wg = 0, both return the newest cached rows bit for bit
    newest = win[-1][n_l:]
    wb = sat.Predictor(pd["Wx"], pd["Wh"], pd["b"], pd["Wg"], d, d_s, tau, bypass=True)
    Hb2 = gu.dev_empty(n_bar, ld, fill=-3.0)
    sat.predict(pv, wb, slots_d, n_rows, ld, ids_d, Hb2, ld, stream=gu.stream_ptr())
    w0 = sat.Predictor(pd["Wx"], pd["Wh"], pd["b"], torch.zeros_like(pd["Wg"]), d, d_s, tau)
    Hb3 = gu.dev_empty(n_bar, ld, fill=-3.0)
    sat.predict(pv, w0, slots_d, n_rows, ld, ids_d, Hb3, ld, workspace=ws, workspace_bytes=wsb,
                stream=gu.stream_ptr())
    gu.sync()
    assert np.array_equal(Hb2.cpu().numpy()[n_l:, :d], newest)
    assert np.array_equal(Hb3.cpu().numpy()[n_l:, :d], newest)
    # the two halves as calls of their own: states in two ranges of rows, then the hop with the
    # residual rows (a) read through the halo ids from the table, (b) already in the halo rows
    # of the output, summed in place - the same bits as the one call either way
    if d_s <= 64:
        S = torch.full((n_bar, d_s), -7.0, dtype=torch.float32, device=gu.DEV)
        ws_s = gu.workspace(sat.predict_states_workspace_bytes(d, d_s))
        cut = (n_bar // 3) | 1
        for b, e in ((0, cut), (cut, n_bar)):
            if use_ids:
                sat.predict_states(w, slots_d, n_rows, ld, ids_d[b:], e - b, S[b:], workspace=ws_s,
                                   workspace_bytes=ws_s.numel() * ws_s.element_size(), stream=gu.stream_ptr())
            else:
                sat.predict_states(w, [t[b:] for t in slots_d], e - b, ld, None, e - b, S[b:], workspace=ws_s,
                                   workspace_bytes=ws_s.numel() * ws_s.element_size(), stream=gu.stream_ptr())
        wsb_h = sat.predict_hop_workspace_bytes(n_h, d_s)
        ws_h = gu.workspace(wsb_h)
        Ha = gu.dev_empty(n_bar, ld, fill=-3.0)
        if use_ids:
            sat.predict_hop(pv, w, S, slots_d[-1], n_rows, ld, ids_d[n_l:], Ha, ld, workspace=ws_h,
                            workspace_bytes=wsb_h, stream=gu.stream_ptr())
        else:
            sat.predict_hop(pv, w, S, slots_d[-1][n_l:], n_h, ld, None, Ha, ld, workspace=ws_h,
                            workspace_bytes=wsb_h, stream=gu.stream_ptr())
        Hi = gu.dev_empty(n_bar, ld, fill=-3.0)
        Hi[n_l:, :d] = torch.from_numpy(np.ascontiguousarray(newest)).to(gu.DEV)
        sat.predict_hop(pv, w, S, Hi[n_l:], n_h, ld, None, Hi, ld, workspace=ws_h, workspace_bytes=wsb_h,
                        stream=gu.stream_ptr())
        gu.sync()
        assert np.array_equal(Ha.cpu().numpy().view(np.uint32), got.view(np.uint32))
        assert np.array_equal(Hi.cpu().numpy().view(np.uint32), got.view(np.uint32))
        # residual rows that overlap the output rows in any other way are refused
        if n_h > 1:
            with pytest.raises(sat.SatError) as e:
                sat.predict_hop(pv, w, S, Hi[n_l + 1:], n_h - 1, ld, None, Hi, ld, workspace=ws_h,
                                workspace_bytes=wsb_h, stream=gu.stream_ptr())
            assert e.value.status == -1
        with pytest.raises(sat.SatError) as e:
            sat.predict_hop(pv, w, S, slots_d[-1], n_rows, ld, None, Ha, ld, workspace=None, workspace_bytes=0)
        assert e.value.status == -4


def test_predict_unsupported_hidden_size(env):
    sat, gu, torch = env
    g = _graph("tiny")
    v = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, 0)
    pv = gu.upload_view(v)
    z = gu.dev_empty(64, 64, fill=0.0)
    w = sat.Predictor(z, z, z, z, 32, 16, 2)
    slots = [gu.dev_empty(v["n_local"] + v["n_halo"], 32, fill=0.0)] * 2
    with pytest.raises(sat.SatError) as e:
        sat.predict(pv, w, slots, v["n_local"] + v["n_halo"], 32, None, slots[0], 32)
    assert e.value.status == -2
