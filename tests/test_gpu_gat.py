"""GPU parity of the graph attention backbone against the CPU oracle: the three
calls on their own (scores, edge softmax aggregation, backward) over graphs with
short rows, hub rows longer than the workgroup-cooperative threshold on both the
row side and the transposed side, several head layouts and both storage types;
then the whole partition step for two consecutive steps."""
import numpy as np
import pytest

import sat_synth as syn
from oracle import gat_oracle as gat
from oracle import sat_oracle as orc

pytestmark = pytest.mark.gpu
SLOPE = 0.2


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2308_13466_amd as sat
    sat.lib()
    from tests import gpu_util as gu
    return sat, gu, torch


def _say(msg):
    print("[case] " + msg, flush=True)


_GRAPHS = {}


def _view(kind, m):
    """(graph, oracle's partition view) of a small seeded graph."""
    if (kind, m) not in _GRAPHS:
        from tests.test_gpu_parity import _graph
        g = _graph(kind)
        _GRAPHS[(kind, m)] = (g, orc.partition_view(g.N, g.rowptr, g.col, g.part, m))
    return _GRAPHS[(kind, m)]


def _upload(gu, torch, a, ld, bf16):
    """Host fp32 [rows, d] -> device [rows, ld] in the storage type; returns the tensor
    and the values it holds as fp32."""
    if not bf16:
        return gu.to_dev(a, ld), a
    bits = syn.bf16_bits_from_f32(a)
    return gu.to_dev_bits(bits, ld).view(torch.bfloat16), syn.f32_from_bf16_bits(bits)


def _download(gu, torch, t, d, bf16):
    if not bf16:
        return gu.to_host(t, d)
    return syn.f32_from_bf16_bits(gu.bits_to_host(t.view(torch.int16), d))


CASES = [
    # kind, partition, heads, d_head, relu, bf16
    ("tiny", 0, 4, 8, True, False),
    ("tiny", 0, 1, 8, False, False),
    ("powerlaw", 0, 4, 64, True, False),
    ("powerlaw", 1, 8, 32, True, False),
    ("powerlaw", 0, 2, 16, False, False),
    ("powerlaw", 2, 1, 47, False, False),
    ("powerlaw", 0, 1, 256, True, False),
    ("hub", 0, 4, 64, True, False),      # a 12,000-entry row; its transposed local row is long too
    ("hub", 1, 2, 32, True, False),      # the hub is a halo node: a long row of the transposed halo block
    ("hub", 0, 1, 41, False, False),
    ("powerlaw", 0, 4, 64, True, True),
    ("hub", 1, 1, 40, False, True),
    # bf16 rows of 256 bytes and more: 16-byte lane shares (8 elements per lane)
    ("hub", 0, 4, 64, True, True),       # long rows combined through LDS
    ("hub", 1, 2, 64, True, True),       # 256-byte rows; the hub is a halo node
    ("powerlaw", 1, 8, 32, True, True),
    ("powerlaw", 0, 1, 128, False, True),
    ("powerlaw", 2, 1, 256, True, True),
    ("powerlaw", 0, 2, 16, False, True),  # 64-byte rows: 4 elements per lane
    ("onepart", 0, 4, 16, True, False),  # no halo at all
]


@pytest.mark.parametrize("kind,m,heads,d_head,relu,bf16", CASES)
def test_gat_calls_match_oracle(env, kind, m, heads, d_head, relu, bf16):
    sat, gu, torch = env
    _say("gat ops %s part %d heads=%d d_head=%d relu=%s bf16=%s" % (kind, m, heads, d_head, relu, bf16))
    g, view = _view(kind, m)
    n_l, n_h = view["n_local"], view["n_halo"]
    n_bar, d = n_l + n_h, heads * d_head
    rtol = 2e-2 if bf16 else 1e-5
    dt = sat.BF16 if bf16 else sat.F32
    rng = np.random.default_rng(1000 + heads * 7 + d_head)
    ld = gu.ld_for(d, 8)
    Z_d, Z = _upload(gu, torch, rng.standard_normal((n_bar, d)).astype(np.float32), ld, bf16)
    a_dst = (rng.standard_normal((heads, d_head)) / np.sqrt(d_head)).astype(np.float32)
    a_src = (rng.standard_normal((heads, d_head)) / np.sqrt(d_head)).astype(np.float32)
    a_dst_d, a_src_d = gu.to_dev(a_dst.reshape(-1)), gu.to_dev(a_src.reshape(-1))
    pv = gu.upload_view(view)
    st = gu.stream_ptr()

    # ---- scores
    el_d = torch.full((n_l, heads), float("nan"), dtype=torch.float32, device=gu.DEV)
    er_d = torch.full((n_bar, heads), float("nan"), dtype=torch.float32, device=gu.DEV)
    sat.gat_scores(Z_d, ld, n_bar, n_l, heads, d_head, a_dst_d, a_src_d, el_d, er_d, dtype=dt, stream=st)
    gu.sync()
    el_ref, er_ref = gat.gat_scores(Z, a_dst, a_src)
    gu.assert_close(el_d.cpu().numpy(), el_ref[:n_l], 1e-5, "el")
    gu.assert_close(er_d.cpu().numpy(), er_ref, 1e-5, "er")

    # ---- forward: both sides start from the same fp32 scores (the oracle's, rounded)
    el32, er32 = el_ref[:n_l].astype(np.float32), er_ref.astype(np.float32)
    el_d, er_d = gu.to_dev(el32), gu.to_dev(er32)
    act = sat.ACT_RELU if relu else sat.ACT_IDENTITY
    H_d = torch.full((n_l, ld), float("nan"), dtype=Z_d.dtype, device=gu.DEV)
    stats_d = torch.full((n_l, heads, 2), float("nan"), dtype=torch.float32, device=gu.DEV)
    sat.gat_aggregate_fwd(pv, Z_d, ld, heads, d_head, el_d, er_d, SLOPE, act, H_d, ld, stats_d,
                          dtype=dt, stream=st)
    gu.sync()
    OUT = gat.gat_aggregate_fwd(view, Z, el32.astype(np.float64), er32.astype(np.float64), SLOPE)
    H_ref = np.maximum(OUT, 0.0) if relu else OUT
    H_gpu = _download(gu, torch, H_d, d, bf16)
    gu.assert_close(H_gpu, H_ref, rtol, "H")
    if not bf16:       # padding columns untouched
        assert torch.isnan(H_d[:, d:]).all()
    stats = stats_d.cpu().numpy()
    m_ref = np.zeros((n_l, heads))
    il_ref = np.zeros((n_l, heads))
    for i in range(n_l):
        _, s, _ = gat.gat_row_attention(view, i, el32.astype(np.float64), er32.astype(np.float64), SLOPE)
        e = gat.leaky_relu(s, SLOPE)
        m_ref[i] = e.max(axis=0)
        il_ref[i] = 1.0 / np.exp(e - e.max(axis=0, keepdims=True)).sum(axis=0)
    gu.assert_close(stats[:, :, 0], m_ref, 1e-5, "row maxima")
    gu.assert_close(stats[:, :, 1], il_ref, 1e-5, "reciprocal sums")

    # ---- backward: the mask comes from the oracle's forward output on both sides
    dH = (rng.standard_normal((n_l, d)) / np.sqrt(n_l)).astype(np.float32)
    dH_d, dH = _upload(gu, torch, dH, ld, bf16)
    H_store = orc.round_bf16(H_ref) if bf16 else H_ref
    Hm_d, _ = _upload(gu, torch, H_store.astype(np.float32), ld, bf16)
    store = orc.round_bf16 if bf16 else None
    cache = dict(Z=Z.astype(np.float64), el=el32.astype(np.float64), er=er32.astype(np.float64),
                 H=H_store, Hbar=np.zeros((n_bar, 1)))
    ref = gat.gat_layer_bwd(view, cache, np.zeros((1, d)), a_dst, a_src, SLOPE, 1 if relu else 0,
                            dH.astype(np.float64), store)
    wsb = sat.gat_aggregate_bwd_workspace_bytes(n_l, n_h, heads, d_head, dt)
    ws = gu.workspace(wsb)
    dZ_d = torch.full((n_bar, ld), float("nan"), dtype=Z_d.dtype, device=gu.DEV)
    da_dst_d = torch.full((d,), float("nan"), dtype=torch.float32, device=gu.DEV)
    da_src_d = torch.full((d,), float("nan"), dtype=torch.float32, device=gu.DEV)
    sat.gat_aggregate_bwd(pv, Z_d, ld, heads, d_head, el_d, er_d, stats_d, SLOPE, act, dH_d, ld,
                          Hm_d if relu else None, ld if relu else 0, a_dst_d, a_src_d, dZ_d, ld,
                          da_dst_d, da_src_d, dtype=dt, workspace=ws, workspace_bytes=wsb, stream=st)
    gu.sync()
    dZ_gpu = _download(gu, torch, dZ_d, d, bf16)
    # dZ_j is the sum of three terms that may cancel (the aggregated gradient against the two
    # score terms): the bound is relative to the terms' magnitudes, not to their sum
    A = np.zeros((n_bar, heads, d_head))
    A[:n_l] = ref["d_el"][:, :, None] * a_dst[None].astype(np.float64)
    Bt = ref["d_er"][:, :, None] * a_src[None].astype(np.float64)
    A, Bt = A.reshape(n_bar, d), Bt.reshape(n_bar, d)
    mag = np.abs(ref["dZ"] - A - Bt) + np.abs(A) + np.abs(Bt)
    rms = np.sqrt(np.mean(ref["dZ"] ** 2))
    err = np.abs(dZ_gpu.astype(np.float64) - ref["dZ"])
    assert np.all(np.isfinite(dZ_gpu))
    bad = err > rtol * (mag + rms)
    assert not bad.any(), "dZ: %d elements outside, worst %g" % (int(bad.sum()), float((err / (mag + rms)).max()))
    gu.assert_close(da_dst_d.cpu().numpy().reshape(heads, d_head), ref["da_dst"], rtol, "da_dst")
    gu.assert_close(da_src_d.cpu().numpy().reshape(heads, d_head), ref["da_src"], rtol, "da_src")
    # a second run gives the same bits (fixed summation order, no atomics)
    dZ2 = torch.empty_like(dZ_d)
    da2 = torch.empty_like(da_dst_d)
    da3 = torch.empty_like(da_src_d)
    sat.gat_aggregate_bwd(pv, Z_d, ld, heads, d_head, el_d, er_d, stats_d, SLOPE, act, dH_d, ld,
                          Hm_d if relu else None, ld if relu else 0, a_dst_d, a_src_d, dZ2, ld,
                          da2, da3, dtype=dt, workspace=ws, workspace_bytes=wsb, stream=st)
    gu.sync()
    assert torch.equal(dZ2[:, :d].view(torch.int16 if bf16 else torch.int32),
                       dZ_d[:, :d].view(torch.int16 if bf16 else torch.int32))
    assert torch.equal(da2, da_dst_d) and torch.equal(da3, da_src_d)


def test_gat_rejects_unsupported_shapes(env):
    sat, gu, torch = env
    g, view = _view("tiny", 0)
    pv = gu.upload_view(view)
    n_l, n_bar = view["n_local"], view["n_local"] + view["n_halo"]
    Z = torch.zeros((n_bar, 512), dtype=torch.float32, device=gu.DEV)
    el = torch.zeros((n_l, 8), dtype=torch.float32, device=gu.DEV)
    er = torch.zeros((n_bar, 8), dtype=torch.float32, device=gu.DEV)
    a = torch.zeros(512, dtype=torch.float32, device=gu.DEV)
    for heads, d_head in ((3, 8), (4, 12), (2, 6), (1, 257), (8, 64)):
        with pytest.raises(sat.SatError) as e:
            sat.gat_scores(Z, 512, n_bar, n_l, heads, d_head, a, a, el, er, stream=gu.stream_ptr())
        assert e.value.status == -2, (heads, d_head)
    with pytest.raises(sat.SatError) as e:   # more destination rows than rows
        sat.gat_scores(Z, 512, 4, 5, 1, 8, a, a, el, er, stream=gu.stream_ptr())
    assert e.value.status == -1
    gu.sync()


def _compare_grad(gu, got, ref, rtol, what, exact_masks, scale=None):
    """Element-wise when no ReLU decision of the step was within rounding of zero;
    otherwise (either decision is valid there, and it reaches the rows around it)
    a norm-wise bound, relative to `scale` (the norm of the sum of the magnitudes of
    the terms the result is formed from; default: the norm of the reference). One flipped
    decision changes one element of a gradient by its whole magnitude, which for the 2 * 10^7
    elements of the medium case is already 2 * 10^-4 of the norm: the bound leaves room for a
    handful of them."""
    if exact_masks:
        gu.assert_close(got, ref, rtol, what)
    else:
        ref = np.asarray(ref, np.float64)
        scale = np.linalg.norm(ref) if scale is None else scale
        err = np.linalg.norm(np.asarray(got, np.float64) - ref)
        assert err < 60 * rtol * scale, "%s: |diff| %g, scale %g" % (what, err, scale)


@pytest.mark.parametrize("name,bf16,stale", [("tiny", False, False), ("medium", False, False),
                                             ("tiny", True, False), ("tiny", False, True),
                                             ("tiny", True, True)])
def test_gat_partition_step_two_steps(env, name, bf16, stale):
    """stale: with seeded gradient tables standing in for what other partitions wrote (the
    stale-gradient term of the appendix's SAT backward): dH_l = local term + the read table's
    rows, the gradient for the halo inputs lands in the write table's halo rows as the step
    computed it, every other row of the tables stays as it was."""
    sat, gu, torch = env
    from paper_2308_13466_amd import binding as B
    from paper_2308_13466_amd.step_gat import GatPartitionStep
    from tests.test_gpu_step import build_problem, fresh_history
    _say("gat step %s bf16=%s stale=%s" % (name, bf16, stale))
    cfg, ss, g, X, Ws, omegas = build_problem(name)
    dims, L, tau = cfg["dims"], len(Ws), cfg["tau"]
    heads = syn.gat_heads(dims)
    ass = ss["misc"].spawn(L)
    attn = [syn.attention_vectors_f32(ass[l], heads[l], dims[l + 1] // heads[l]) for l in range(L)]
    _, hist = fresh_history(cfg, ss, g, X, Ws)
    view = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, cfg["part"])
    n_l, n_h = view["n_local"], view["n_halo"]
    y = syn.labels_i32(ss["labels"], n_l, dims[-1])
    rtol = 2e-2 if bf16 else 1e-5
    store = orc.round_bf16 if bf16 else None
    dt = B.BF16 if bf16 else B.F32
    ld = [gu.ld_for(d) for d in dims]

    def up(a, ldv):
        t, host = _upload(gu, torch, np.ascontiguousarray(a, dtype=np.float32), ldv, bf16)
        return t, host

    X_d, X = up(X, ld[0])
    hist_d = [None]
    for l in range(1, L):
        pairs = [up(h, ld[l]) for h in hist[l]]
        hist_d.append([p[0] for p in pairs])
        hist[l] = [p[1].copy() for p in pairs]
    Ws_d = []
    for l in range(L):
        w = np.zeros((dims[l], gu.ld_for(dims[l + 1], 8)), np.float32)
        w[:, :dims[l + 1]] = Ws[l]
        w_d, w_host = up(w, None)
        Ws_d.append(w_d)
        Ws[l] = w_host[:, :dims[l + 1]]
    attn_d = [(gu.to_dev(a.reshape(-1)), gu.to_dev(b.reshape(-1)), heads[l])
              for l, (a, b) in enumerate(attn)]
    ids = np.concatenate([view["local_ids"], view["halo_ids"]]).astype(np.int32)
    preds = [None]
    keep = []
    for l in range(1, L):
        pd = {k: gu.to_dev(omegas[l][k]) for k in omegas[l]}
        keep.append(pd)
        preds.append(B.Predictor(pd["Wx"], pd["Wh"], pd["b"], pd["Wg"], dims[l], cfg["d_s"], tau))
    gt = gt_host = None
    if stale:
        rng = np.random.default_rng(9)
        gt_host, gt = [None], [None]
        for l in range(1, L):
            pairs = [up((1e-3 * rng.standard_normal((g.N, dims[l]))).astype(np.float32), ld[l]) for _ in range(2)]
            gt.append([p[0] for p in pairs])
            gt_host.append([p[1].copy() for p in pairs])
    step = GatPartitionStep(view, dims, X_d, hist_d, gu.to_dev(ids), Ws_d, attn_d, preds,
                            gu.to_dev(y), tau, slope=SLOPE, dtype=dt, grad_tables=gt)
    params = [dict(W=Ws[l], a_dst=attn[l][0], a_src=attn[l][1]) for l in range(L)]
    for t in range(2):
        order = [(t + s) % tau for s in range(tau)]
        halo_hat = [None]
        for l in range(1, L):
            win = [hist[l][s][ids] for s in order]
            hh = orc.predict(view, omegas[l], win)
            halo_hat.append(hh if store is None else store(hh))
        stale_rows = None
        if stale:
            stale_rows = [None] + [gt_host[l][t % 2][view["local_ids"]] for l in range(1, L)]
        ref = gat.gat_partition_step(view, X[view["local_ids"]], X[view["halo_ids"]], halo_hat,
                                     params, y, SLOPE, store=store, stale_grad=stale_rows)
        for l in range(1, L):
            orc.history_push(hist[l][t % tau], view["local_ids"], ref["H"][l].astype(np.float32))
        step.forward_backward()
        gu.sync()
        assert abs(float(step.loss.item()) - ref["loss"]) < (2e-2 if bf16 else 2e-6) * max(1.0, ref["loss"])
        exact = True
        for l in range(L):
            out = step.logits if l == L - 1 else step.Hbar[l + 1][:n_l]
            gu.assert_close(_download(gu, torch, out, dims[l + 1], bf16), ref["H"][l + 1], rtol,
                            "H layer %d step %d" % (l + 1, t))
            if l < L - 1:
                OUT = ref["caches"][l]["OUT"]
                exact = exact and not np.any(np.abs(OUT) < 2e-6 * np.sqrt(np.mean(OUT * OUT)))
        exact = exact and not bf16
        for l in range(L):
            gr = ref["grads"][l]
            K, F = heads[l], dims[l + 1] // heads[l]
            if l == 0:   # the layers share one dZ buffer: layer 0's is what is left after the step
                _compare_grad(gu, _download(gu, torch, step.dZ[l], dims[l + 1], bf16), gr["dZ"], rtol,
                              "dZ layer %d step %d" % (l, t), exact)
            _compare_grad(gu, step.dW[l].cpu().numpy()[:, :dims[l + 1]], gr["dW"], rtol,
                          "dW layer %d step %d" % (l, t), exact)
            # the attention-vector gradients are sums over all rows of terms of either sign
            # (d_el vanishes wherever a row's scores share one LeakyReLU branch): one valid
            # flip of a ReLU decision moves them by far more than rounding does, so under
            # ambiguity they are held to the size of their terms
            Zh = np.abs(ref["caches"][l]["Z"]).reshape(-1, K, F)
            s_dst = np.linalg.norm(np.einsum("nk,nkf->kf", np.abs(gr["d_el"]), Zh[:n_l]))
            s_src = np.linalg.norm(np.einsum("nk,nkf->kf", np.abs(gr["d_er"]), Zh))
            _compare_grad(gu, step.da_dst[l].cpu().numpy().reshape(K, F), gr["da_dst"], rtol,
                          "da_dst layer %d" % l, exact, s_dst)
            _compare_grad(gu, step.da_src[l].cpu().numpy().reshape(K, F), gr["da_src"], rtol,
                          "da_src layer %d" % l, exact, s_src)
            if l >= 1:
                _compare_grad(gu, _download(gu, torch, step.dH[l], dims[l], bf16), ref["dH_in"][l],
                              rtol, "dH_in layer %d step %d" % (l, t), exact)
        if stale:
            wr = (t + 1) % 2
            others = np.setdiff1d(np.arange(g.N), view["halo_ids"])
            for l in range(1, L):
                got_halo = _download(gu, torch, step.dH_halo[l], dims[l], bf16)
                _compare_grad(gu, got_halo, ref["dH_halo"][l], rtol, "dH_halo layer %d step %d" % (l, t), exact)
                tab = _download(gu, torch, gt[l][wr], dims[l], bf16)
                assert np.array_equal(tab[view["halo_ids"]], got_halo)
                assert np.array_equal(tab[others], gt_host[l][wr][others][:, :dims[l]])
                # the next step reads what the oracle says this one wrote
                w_rows = np.asarray(ref["dH_halo"][l], np.float32)
                gt_host[l][wr][view["halo_ids"], :dims[l]] = orc.round_bf16(w_rows) if bf16 else w_rows
        # the ring received this step's embeddings
        for l in range(1, L):
            got = _download(gu, torch, hist_d[l][t % tau], dims[l], bf16)[view["local_ids"]]
            gu.assert_close(got, ref["H"][l], rtol, "pushed layer %d" % l)


@pytest.mark.parametrize("name,chunk", [("tiny", None), ("medium", None), ("medium", 20_000)])
def test_gat_step_with_a_coded_ring_equals_the_dense_ring_of_stored_values(env, name, chunk):
    """The graph attention step reads its predictor window from a CODED ring (decoded whole, or
    `chunk` rows at a time) and codes what it pushes. A coded ring is a dense ring that holds
    the codec's stored values (orc.polyline_stored_value, pinned byte by byte elsewhere), so
    the step must leave, bit for bit, what the dense-ring step leaves when its tables hold
    those values - over two steps, the second one reading what the first one pushed."""
    sat, gu, torch = env
    from paper_2308_13466_amd.workload import build_workload
    from tests.test_gpu_coded_step import _decode_part
    prec = 2
    _say("gat step, coded ring, %s, chunk=%s" % (name, chunk))
    wc = build_workload(name, backbone="gat", coded_ring=prec, coded_chunk_rows=chunk)
    wd = build_workload(name, backbone="gat")
    sc, sd = wc.step, wd.step
    n_l, dims, L, tau = sc.n_local, wc.dims, wc.L, wc.tau
    local_ids = torch.from_numpy(wc.view["local_ids"].astype(np.int64)).to(gu.DEV)
    for l in range(1, L):       # the dense ring starts from the stored values of the same tables
        for s in range(tau):
            stored = orc.polyline_stored_value(wd.hist_host[l][s][:, :dims[l]], prec)
            sd.hist[l][s][:, :dims[l]] = torch.from_numpy(stored).to(gu.DEV)

    def same(a, b):
        return a.shape == b.shape and torch.equal(a.view(torch.int32), b.view(torch.int32))
    for t in range(2):
        sc.forward_backward()
        sd.forward_backward()
        gu.sync()
        assert sc.coded_overflow() == []
        assert same(sc.loss, sd.loss) and same(sc.logits, sd.logits), "step %d" % t
        for l in range(L):
            assert same(sc.dW[l], sd.dW[l]) and same(sc.da_dst[l], sd.da_dst[l]) and same(sc.da_src[l], sd.da_src[l])
            if l >= 1:
                assert same(sc.Hbar[l], sd.Hbar[l]), "Hbar %d step %d" % (l, t)
                assert same(sc.dH[l], sd.dH[l]), "dH %d step %d" % (l, t)
        # the push: the `own` part of the write slot decodes to the stored values of the fresh
        # rows; the dense ring is then given those values, as a coded table would hand them back
        for l in range(1, L):
            slot = wc.coded.slots[l][t % tau]
            got = _decode_part(sat, gu, slot.own_codes, slot.own_off, n_l, dims[l], sc.ld[l], prec)
            fresh = gu.to_host(sc.Hbar[l], dims[l])[:n_l]
            want = orc.polyline_stored_value(fresh, prec)
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
            tab = sd.hist[l][t % tau]
            tab[local_ids, :dims[l]] = torch.from_numpy(want).to(gu.DEV)
