"""GPU parity of the bf16 storage mode (features, activations and history in
bfloat16, sums in fp32): the oracle sees exactly the bf16 values the GPU sees
(widened to fp64) and results are held to 2e-2; copies are bit-exact."""
import numpy as np
import pytest

import sat_synth as syn
from oracle import sat_oracle as orc

pytestmark = pytest.mark.gpu
RTOL_BF16 = 2e-2


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available()
    import paper_2308_13466_amd as sat
    sat.lib()
    from tests import gpu_util as gu
    return sat, gu, torch


def _say(msg):
    print("[case] " + msg, flush=True)


def _bf16(a):
    """(bit patterns, the exact fp32 values they stand for)"""
    bits = syn.bf16_bits_from_f32(a)
    return bits, syn.f32_from_bf16_bits(bits)


@pytest.mark.parametrize("d,ld_t,ld_o", [(1, 1, 1), (3, 5, 3), (8, 8, 16), (128, 128, 128),
                                         (100, 104, 128), (256, 256, 264), (13, 17, 15)])
def test_bf16_gather_push_bit_exact(env, d, ld_t, ld_o):
    sat, gu, torch = env
    _say("bf16 gather/push d=%d ld_t=%d ld_o=%d" % (d, ld_t, ld_o))
    rng = np.random.default_rng(d)
    n_rows, n = 3000, 2222
    table = rng.integers(0, 65536, size=(n_rows, ld_t)).astype(np.uint16)
    ids = rng.integers(0, n_rows, size=n).astype(np.int32)
    t_d, i_d = gu.to_dev_bits(table), gu.to_dev(ids)
    out = torch.full((n, ld_o), 77, dtype=torch.int16, device=gu.DEV)
    sat.history_gather(t_d, n_rows, ld_t, i_d, n, d, out, ld_o, dtype=sat.BF16, stream=gu.stream_ptr())
    gu.sync()
    got = gu.bits_to_host(out)
    assert np.array_equal(got[:, :d], orc.history_gather(table, ids)[:, :d])
    assert np.all(got[:, d:] == 77)
    pid = rng.permutation(n_rows)[:n].astype(np.int32)
    H = rng.integers(0, 65536, size=(n, ld_o)).astype(np.uint16)
    ref = orc.history_push(table.copy(), pid, H[:, :d])
    sat.history_push(t_d, n_rows, ld_t, gu.to_dev(pid), n, d, gu.to_dev_bits(H), ld_o,
                     dtype=sat.BF16, stream=gu.stream_ptr())
    gu.sync()
    assert np.array_equal(gu.bits_to_host(t_d), ref)


def _graph(kind):
    from tests.test_gpu_parity import _graph as g
    return g(kind)


@pytest.mark.parametrize("kind,d", [("tiny", 64), ("tiny", 8), ("powerlaw", 128), ("powerlaw", 256),
                                    ("hub", 256), ("hub", 128), ("powerlaw", 100), ("tiny", 1),
                                    ("onepart", 600), ("tiny", 2056)])
def test_bf16_spmm_parity(env, kind, d):
    sat, gu, torch = env
    _say("bf16 spmm %s d=%d" % (kind, d))
    g = _graph(kind)
    v = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, 0)
    n_l, n_h = v["n_local"], v["n_halo"]
    rng = np.random.default_rng(d)
    hb_bits, hb = _bf16(rng.standard_normal((n_l + n_h, d)).astype(np.float32))
    g_bits, gv = _bf16(rng.standard_normal((n_l, d)).astype(np.float32))
    ld = gu.ld_for(d, 8)
    pv = gu.upload_view(v)
    agg = torch.full((n_l, ld), 77, dtype=torch.int16, device=gu.DEV)
    sat.spmm_fwd(pv, gu.to_dev_bits(hb_bits, ld), ld, d, agg, ld, dtype=sat.BF16, stream=gu.stream_ptr())
    dl = torch.full((n_l, ld), 77, dtype=torch.int16, device=gu.DEV)
    dh = torch.full((max(n_h, 1), ld), 77, dtype=torch.int16, device=gu.DEV)
    sat.spmm_bwd(pv, gu.to_dev_bits(g_bits, ld), ld, d, dl, ld, dh if n_h else None, ld,
                 dtype=sat.BF16, stream=gu.stream_ptr())
    gu.sync()
    got = syn.f32_from_bf16_bits(gu.bits_to_host(agg, d))
    gu.assert_close(got, orc.spmm_fwd(v, hb), RTOL_BF16, "bf16 spmm_fwd")
    assert np.all(gu.bits_to_host(agg)[:, d:] == 77)
    # the result is the fp32 sum rounded once: it must sit within one bf16 step of the oracle
    ref = orc.spmm_fwd(v, hb)
    rms = np.sqrt(np.mean(ref * ref))
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-5 * rms)
    rl, rh = orc.spmm_bwd(v, gv, want_halo=True)
    gu.assert_close(syn.f32_from_bf16_bits(gu.bits_to_host(dl, d)), rl, RTOL_BF16, "bf16 spmm_bwd")
    if n_h:
        gu.assert_close(syn.f32_from_bf16_bits(gu.bits_to_host(dh, d))[:n_h], rh, RTOL_BF16,
                        "bf16 spmm_bwd halo")


@pytest.mark.parametrize("n,d_in,d_out,act", [(2048, 64, 32, 1), (1000, 128, 256, 1),
                                              (777, 256, 256, 1), (513, 256, 176, 0),
                                              (300, 600, 256, 1), (129, 104, 48, 0), (5, 8, 8, 1),
                                              (1500, 256, 47, 0), (4100, 128, 172, 0),
                                              (70001, 256, 256, 1), (33, 16, 300, 1)])
def test_bf16_dense_fwd_bwd_parity(env, n, d_in, d_out, act):
    sat, gu, torch = env
    _say("bf16 dense n=%d %d->%d act=%d" % (n, d_in, d_out, act))
    rng = np.random.default_rng(n + d_in)
    a_bits, A = _bf16(rng.standard_normal((n, d_in)).astype(np.float32))
    w_bits, W = _bf16(syn.glorot_uniform_f32(np.random.SeedSequence(n), d_in, d_out))
    g_bits, dH = _bf16(rng.standard_normal((n, d_out)).astype(np.float32))
    ld_a, ld_w, ld_h = gu.ld_for(d_in, 8), gu.ld_for(d_out, 8), gu.ld_for(d_out, 32)
    A_d, W_d, dH_d = gu.to_dev_bits(a_bits, ld_a), gu.to_dev_bits(w_bits, ld_w), gu.to_dev_bits(g_bits, ld_h)
    H_d = torch.full((n, ld_h), 77, dtype=torch.int16, device=gu.DEV)
    sat.dense_fwd(A_d, ld_a, n, d_in, d_out, W_d, ld_w, act, H_d, ld_h, dtype=sat.BF16,
                  stream=gu.stream_ptr())
    gu.sync()
    Z, H = orc.dense_fwd(A, W, act)
    got = syn.f32_from_bf16_bits(gu.bits_to_host(H_d, d_out))
    gu.assert_close(got, H, RTOL_BF16, "bf16 dense_fwd")
    rms = np.sqrt(np.mean(H * H))
    assert np.all(np.abs(got - H) <= 2.0 ** -8 * np.abs(H) + 1e-5 * rms)   # one rounding of an fp32 sum
    assert np.all(gu.bits_to_host(H_d)[:, d_out:] == 77)
    # backward: mask from the oracle's forward output rounded to bf16 (both sides see the same mask)
    h_bits, H16 = _bf16(H.astype(np.float32))
    Hm_d = gu.to_dev_bits(h_bits, ld_h)
    dW_d = gu.dev_empty(d_in, ld_w, fill=-3.0)
    dA_d = torch.full((n, ld_a), 77, dtype=torch.int16, device=gu.DEV)
    wsb = sat.dense_bwd_workspace_bytes(n, d_in, d_out)
    ws = gu.workspace(wsb)
    sat.dense_bwd(dH_d, ld_h, Hm_d, ld_h, A_d, ld_a, W_d, ld_w, n, d_in, d_out, act, dW_d, ld_w,
                  dA_d, ld_a, dtype=sat.BF16, workspace=ws, workspace_bytes=wsb, stream=gu.stream_ptr())
    gu.sync()
    dW, dA, _ = orc.dense_bwd(dH, H16, A, W, act)
    gu.assert_close(gu.to_host(dW_d, d_out), dW, 1e-5, "bf16 dW (fp32 out, exact bf16 products)")
    gu.assert_close(syn.f32_from_bf16_bits(gu.bits_to_host(dA_d, d_in)), dA, RTOL_BF16, "bf16 dAGG")


@pytest.mark.parametrize("n,C", [(2048, 8), (1001, 40), (70, 172), (333, 47), (90, 700)])
def test_bf16_loss_grad_parity(env, n, C):
    sat, gu, torch = env
    _say("bf16 loss n=%d C=%d" % (n, C))
    rng = np.random.default_rng(C)
    h_bits, HL = _bf16((3.0 * rng.standard_normal((n, C))).astype(np.float32))
    y = rng.integers(0, C, size=n).astype(np.int32)
    ld = gu.ld_for(C, 8)
    g_d = torch.full((n, ld), 77, dtype=torch.int16, device=gu.DEV)
    loss_d = torch.zeros(1, dtype=torch.float32, device=gu.DEV)
    wsb = sat.loss_workspace_bytes(n)
    ws = gu.workspace(wsb)
    sat.loss_grad(gu.to_dev_bits(h_bits, ld), ld, n, C, gu.to_dev(y), g_d, ld, loss=loss_d,
                  dtype=sat.BF16, workspace=ws, workspace_bytes=wsb, stream=gu.stream_ptr())
    gu.sync()
    loss, g = orc.loss_and_grad(HL, y)
    gu.assert_close(syn.f32_from_bf16_bits(gu.bits_to_host(g_d, C)), g, RTOL_BF16, "bf16 dH^(L)")
    assert np.all(gu.bits_to_host(g_d)[:, C:] == 77)          # padding columns untouched
    assert abs(float(loss_d.item()) - loss) <= 2e-5 * abs(loss)


@pytest.mark.parametrize("kind,d,d_s,tau,use_ids", [("tiny", 32, 32, 2, False),
                                                    ("powerlaw", 256, 64, 2, True),
                                                    ("powerlaw", 104, 64, 3, False),
                                                    ("hub", 40, 32, 1, True)])
def test_bf16_predict_parity(env, kind, d, d_s, tau, use_ids):
    sat, gu, torch = env
    _say("bf16 predict %s d=%d d_s=%d tau=%d ids=%s" % (kind, d, d_s, tau, use_ids))
    g = _graph(kind)
    v = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, 0)
    n_l, n_h = v["n_local"], v["n_halo"]
    n_bar = n_l + n_h
    rng = np.random.default_rng(d + d_s)
    p = syn.predictor_params_f32(np.random.SeedSequence(d_s), d, d_s)
    ld = gu.ld_for(d, 32)
    if use_ids:
        ids = np.concatenate([v["local_ids"], v["halo_ids"]]).astype(np.int32)
        n_rows = g.N
    else:
        ids, n_rows = None, n_bar
    base = np.maximum(rng.standard_normal((n_rows, d)), 0).astype(np.float32)
    tabs = [_bf16((base + 0.05 * rng.standard_normal((n_rows, d))).astype(np.float32))
            for _ in range(tau)]
    win = [t[1][ids] if use_ids else t[1] for t in tabs]
    ref = orc.predict(v, p, win)
    pv = gu.upload_view(v)
    pd = {k: gu.to_dev(p[k]) for k in p}
    w = sat.Predictor(pd["Wx"], pd["Wh"], pd["b"], pd["Wg"], d, d_s, tau)
    slots_d = [gu.to_dev_bits(t[0], ld) for t in tabs]
    Hbar = torch.full((n_bar, ld), 77, dtype=torch.int16, device=gu.DEV)
    wsb = sat.predict_workspace_bytes(n_l, n_h, d, d_s, tau)
    ws = gu.workspace(wsb)
    ids_d = gu.to_dev(ids) if use_ids else None
    sat.predict(pv, w, slots_d, n_rows, ld, ids_d, Hbar, ld, dtype=sat.BF16, workspace=ws,
                workspace_bytes=wsb, stream=gu.stream_ptr())
    gu.sync()
    got = gu.bits_to_host(Hbar)
    assert np.all(got[:n_l] == 77) and np.all(got[:, d:] == 77)
    gu.assert_close(syn.f32_from_bf16_bits(got[n_l:, :d]), ref, RTOL_BF16, "bf16 predict")
    # the only rounding is the final store: within one bf16 step of the oracle
    out = syn.f32_from_bf16_bits(got[n_l:, :d])
    rms = np.sqrt(np.mean(ref * ref))
    assert np.all(np.abs(out - ref) <= 2.0 ** -8 * np.abs(ref) + 2e-5 * rms)
    wb = sat.Predictor(pd["Wx"], pd["Wh"], pd["b"], pd["Wg"], d, d_s, tau, bypass=True)
    Hb2 = torch.full((n_bar, ld), 77, dtype=torch.int16, device=gu.DEV)
    sat.predict(pv, wb, slots_d, n_rows, ld, ids_d, Hb2, ld, dtype=sat.BF16, stream=gu.stream_ptr())
    gu.sync()
    newest_bits = (tabs[-1][0][ids] if use_ids else tabs[-1][0])[n_l:]
    assert np.array_equal(gu.bits_to_host(Hb2)[n_l:, :d], newest_bits)
