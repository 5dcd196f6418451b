"""GPU parity of the embedding predictor's training (Eq. 11 / 12, Alg. 1
"embedding predictor update"): loss and the four gradients of
sat_predictor_grad against the oracle's back-propagation, and a short run of
plain gradient steps (sat_sgd_update) whose loss curve must follow the
oracle's run of the same steps."""
import numpy as np
import pytest

import sat_synth as syn
from oracle import sat_oracle as orc
from tests.test_gpu_parity import _graph

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


def _problem(kind, d, d_s, tau, use_ids, seed):
    g = _graph(kind)
    rng = np.random.default_rng(seed)
    return g, rng, syn.predictor_params_f32(np.random.SeedSequence(seed), d, d_s)


def _setup(env, kind, d, d_s, tau, use_ids, masked, seed, bf16=False):
    sat, gu, torch = env
    g, rng, p = _problem(kind, d, d_s, tau, use_ids, seed)
    v = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, 0)
    n_l, n_h = v["n_local"], v["n_halo"]
    n_bar = n_l + n_h
    ld = gu.ld_for(d, 32)
    if use_ids:
        ids = np.concatenate([v["local_ids"], v["halo_ids"]]).astype(np.int32)
        n_rows = g.N
    else:
        ids, n_rows = None, n_bar
    base = np.maximum(rng.standard_normal((n_rows, d)), 0).astype(np.float32)
    tables = [(base + 0.05 * rng.standard_normal((n_rows, d))).astype(np.float32) for _ in range(tau)]
    win = [t[ids] if use_ids else t for t in tables]
    # "fresh" embeddings of the local nodes: the shared base moved a little further
    target = (win[-1][:n_l] + 0.1 * rng.standard_normal((n_l, d))).astype(np.float32)
    weight = (rng.random(n_l) < 0.3).astype(np.float32) if masked else None

    def up(a):
        if not bf16:
            return gu.to_dev(a, ld)
        return gu.to_dev_bits(syn.bf16_bits_from_f32(a), ld).view(torch.bfloat16)

    if bf16:   # the tables and the target hold bfloat16: both sides start from the rounded values
        tables = [syn.f32_from_bf16_bits(syn.bf16_bits_from_f32(t)) for t in tables]
        target = syn.f32_from_bf16_bits(syn.bf16_bits_from_f32(target))
        win = [t[ids] if use_ids else t for t in tables]
    dev = dict(pv=gu.upload_view(v), slots=[up(t) for t in tables],
               ids=gu.to_dev(ids) if use_ids else None, target=up(target),
               weight=gu.to_dev(weight) if masked else None,
               p={k: gu.to_dev(p[k]) for k in p})
    wsb = sat.predictor_train_workspace_bytes(n_l, n_h, d, d_s, tau)
    dev["ws"], dev["wsb"] = gu.workspace(wsb), wsb
    dev["g"] = dict(Wx=gu.dev_empty(4 * d_s, d), Wh=gu.dev_empty(4 * d_s, d_s),
                    b=torch.full((4 * d_s,), float("nan"), device=gu.DEV),
                    Wg=gu.dev_empty(d_s, d))
    dev["loss"] = torch.full((1,), float("nan"), device=gu.DEV)
    return v, p, win, target, weight, n_rows, ld, dev


def _grad(env, v, dev, d, d_s, tau, n_rows, ld, bf16=False):
    sat, gu, torch = env
    w = sat.Predictor(dev["p"]["Wx"], dev["p"]["Wh"], dev["p"]["b"], dev["p"]["Wg"], d, d_s, tau)
    sat.predictor_grad(dev["pv"], w, dev["slots"], n_rows, ld, dev["ids"], dev["target"], ld,
                       dev["weight"], dev["g"]["Wx"], dev["g"]["Wh"], dev["g"]["b"], dev["g"]["Wg"],
                       dev["loss"], dtype=sat.BF16 if bf16 else sat.F32, workspace=dev["ws"],
                       workspace_bytes=dev["wsb"], stream=gu.stream_ptr())
    gu.sync()


@pytest.mark.parametrize("kind,d,d_s,tau,use_ids,masked,bf16", [
    ("tiny", 32, 32, 2, False, False, False), ("tiny", 32, 32, 1, True, True, False),
    ("powerlaw", 256, 64, 2, True, False, False), ("powerlaw", 100, 64, 3, False, True, False),
    ("hub", 40, 32, 2, True, False, False),
    # d_s = 128: the forward as two transform products and an element-wise step per time step
    ("powerlaw", 100, 128, 2, True, False, False), ("hub", 40, 128, 3, False, True, False),
    ("tiny", 32, 128, 1, False, False, False),
    # bfloat16 tables and target: the same arithmetic (fp32 inside) on the rounded inputs
    ("tiny", 32, 32, 2, True, False, True), ("powerlaw", 256, 64, 2, True, True, True),
    ("hub", 40, 32, 3, False, False, True)])
def test_predictor_grad_parity(env, kind, d, d_s, tau, use_ids, masked, bf16):
    sat, gu, torch = env
    print("[case] predictor_grad %s d=%d d_s=%d tau=%d ids=%s masked=%s bf16=%s" % (
        kind, d, d_s, tau, use_ids, masked, bf16), flush=True)
    v, p, win, target, weight, n_rows, ld, dev = _setup(env, kind, d, d_s, tau, use_ids, masked,
                                                        seed=d + d_s + tau, bf16=bf16)
    _grad(env, v, dev, d, d_s, tau, n_rows, ld, bf16)
    loss, grads = orc.predictor_train_loss_and_grad(v, p, win, target, weight)
    got_loss = float(dev["loss"].item())
    assert abs(got_loss - loss) <= 2 * RTOL * abs(loss), (got_loss, loss)
    for name in ("Wg", "b", "Wx", "Wh"):
        got = dev["g"][name].cpu().numpy()
        # the gradients go through the LSTM's gates (hardware exp2 / reciprocal in the
        # forward, ~2e-7 absolute): same bound as the predictor's forward parity
        gu.assert_close(got, grads[name], 2 * RTOL, "d" + name)
    if tau == 1:
        assert np.all(dev["g"]["Wh"].cpu().numpy() == 0.0)


def test_predictor_training_run_follows_the_oracle(env):
    """Six plain gradient steps on the GPU and in the oracle from the same start:
    the loss falls and the two curves agree."""
    sat, gu, torch = env
    print("[case] predictor training run, tiny", flush=True)
    d, d_s, tau = 32, 32, 2
    v, p, win, target, weight, n_rows, ld, dev = _setup(env, "tiny", d, d_s, tau, True, False, seed=5)
    om = {k: p[k].astype(np.float64) for k in p}
    lr = 0.5
    curve_gpu, curve_orc = [], []
    for it in range(6):
        _grad(env, v, dev, d, d_s, tau, n_rows, ld)
        curve_gpu.append(float(dev["loss"].item()))
        for k in ("Wx", "Wh", "b", "Wg"):
            sat.sgd_update(dev["p"][k], dev["g"][k], dev["p"][k].numel(), lr, stream=gu.stream_ptr())
        l, gr = orc.predictor_train_loss_and_grad(v, om, win, target)
        curve_orc.append(l)
        for k in om:
            om[k] -= lr * gr[k]
    gu.sync()
    print("[case] loss curve gpu %s" % ["%.6f" % x for x in curve_gpu], flush=True)
    assert curve_gpu[-1] < curve_gpu[0]
    np.testing.assert_allclose(curve_gpu, curve_orc, rtol=1e-4)
    for k in om:
        gu.assert_close(dev["p"][k].cpu().numpy(), om[k], 1e-4, "parameter %s after the run" % k)


def test_trained_predictor_alleviates_staleness_on_drifting_embeddings(env):
    """Embeddings that keep moving from epoch to epoch: twenty gradient steps of the
    predictor on the partition's fresh local rows (sat_predictor_grad + sat_sgd_update), then
    sat_predict on the halo rows. The run must follow the oracle's run of the same steps, and
    the predicted halo rows must be less stale than the newest cached ones (Eq. 8')."""
    sat, gu, torch = env
    print("[case] predictor trained on drifting embeddings, tiny", flush=True)
    g = _graph("tiny")
    v = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, 0)
    n_l, n_h = v["n_local"], v["n_halo"]
    n_bar = n_l + n_h
    d, d_s, tau, lr, steps = 16, 32, 2, 2.0, 20
    ld = gu.ld_for(d, 32)
    H = syn.drifting_history_f32(np.random.SeedSequence(3), n_bar, d, tau + 1)
    win, fresh = H[:tau], H[tau]
    p = syn.predictor_params_f32(np.random.SeedSequence(3), d, d_s)
    om = {k: p[k].astype(np.float64) for k in p}
    pv = gu.upload_view(v)
    st = gu.stream_ptr()
    slots_d = [gu.to_dev(t, ld) for t in win]
    target_d = gu.to_dev(fresh[:n_l], ld)
    pd = {k: gu.to_dev(p[k]) for k in p}
    gd = dict(Wx=gu.dev_empty(4 * d_s, d), Wh=gu.dev_empty(4 * d_s, d_s),
              b=torch.full((4 * d_s,), float("nan"), device=gu.DEV), Wg=gu.dev_empty(d_s, d))
    loss_d = torch.full((1,), float("nan"), device=gu.DEV)
    wsb = max(sat.predictor_train_workspace_bytes(n_l, n_h, d, d_s, tau),
              sat.predict_workspace_bytes(n_l, n_h, d, d_s, tau))
    ws = gu.workspace(wsb)
    w = sat.Predictor(pd["Wx"], pd["Wh"], pd["b"], pd["Wg"], d, d_s, tau)
    curve_gpu, curve_orc = [], []
    for it in range(steps):
        sat.predictor_grad(pv, w, slots_d, n_bar, ld, None, target_d, ld, None, gd["Wx"], gd["Wh"],
                           gd["b"], gd["Wg"], loss_d, workspace=ws, workspace_bytes=wsb, stream=st)
        gu.sync()
        curve_gpu.append(float(loss_d.item()))
        for k in ("Wx", "Wh", "b", "Wg"):
            sat.sgd_update(pd[k], gd[k], pd[k].numel(), lr, stream=st)
        l, gr = orc.predictor_train_loss_and_grad(v, om, win, fresh[:n_l])
        curve_orc.append(l)
        for k in om:
            om[k] -= lr * gr[k]
    Hbar = gu.dev_empty(n_bar, ld, fill=-3.0)
    sat.predict(pv, w, slots_d, n_bar, ld, None, Hbar, ld, workspace=ws, workspace_bytes=wsb, stream=st)
    gu.sync()
    print("[case] loss %.6f -> %.6f" % (curve_gpu[0], curve_gpu[-1]), flush=True)
    np.testing.assert_allclose(curve_gpu, curve_orc, rtol=2e-4)
    pred_gpu = Hbar.cpu().numpy()[n_l:, :d]
    pred_orc = orc.predict(v, om, win)
    gu.assert_close(pred_gpu, pred_orc, 1e-4, "predicted halo rows after the run")
    truth = fresh[n_l:].astype(np.float64)
    cached = orc.staleness(truth, win[-1][n_l:])
    after = orc.staleness(truth, pred_gpu)
    print("[case] halo staleness: cached %.3f, predicted %.3f" % (cached, after), flush=True)
    assert curve_gpu[-1] < 0.1 * curve_gpu[0]
    assert after < 0.8 * cached


def test_predictor_grad_rejects_what_it_does_not_do(env):
    sat, gu, torch = env
    from paper_2308_13466_amd import binding as B
    v, p, win, target, weight, n_rows, ld, dev = _setup(env, "tiny", 32, 32, 2, False, False, seed=1)
    w = sat.Predictor(dev["p"]["Wx"], dev["p"]["Wh"], dev["p"]["b"], dev["p"]["Wg"], 32, 32, 2)
    args = (dev["pv"], w, dev["slots"], n_rows, ld, dev["ids"], dev["target"], ld, None,
            dev["g"]["Wx"], dev["g"]["Wh"], dev["g"]["b"], dev["g"]["Wg"], dev["loss"])
    # bfloat16 rows are read in 16-byte chunks: widths that are not a multiple of 8 are refused
    w36 = sat.Predictor(dev["p"]["Wx"], dev["p"]["Wh"], dev["p"]["b"], dev["p"]["Wg"], 36, 32, 2)
    with pytest.raises(sat.SatError) as e:
        sat.predictor_grad(*((args[0], w36) + args[2:]), dtype=B.BF16, workspace=dev["ws"],
                           workspace_bytes=dev["wsb"])
    assert e.value.status == -2
    with pytest.raises(sat.SatError) as e:
        sat.predictor_grad(*args, workspace=dev["ws"], workspace_bytes=dev["wsb"] - 1024)
    assert e.value.status == -4
