"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the HIP library. Each one compares the oracle
with something that is not the oracle: a hand-derived fixture, a dense brute
force, a closed form, a library routine, or central finite differences.
"""
import os

import numpy as np
import pytest
import scipy.sparse as sp

import sat_synth as syn
from oracle import sat_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ helpers
def small_graph(seed=3, N=120, n_parts=3):
    rng = np.random.default_rng(seed)
    return syn.sbm_graph(N, n_comm=n_parts, n_parts=n_parts, intra_deg=4.0,
                         cross_deg=1.5, rng=rng)


def dense_a_hat(g):
    """Brute force: dense boolean adjacency -> D^-1/2 (A+I) D^-1/2 in fp64."""
    A = np.zeros((g.N, g.N))
    for i in range(g.N):
        for j in g.col[g.rowptr[i]:g.rowptr[i + 1]]:
            A[i, j] = 1.0
    At = A + np.eye(g.N)
    dt = At.sum(axis=1)
    return A, At / np.sqrt(np.outer(dt, dt)), dt


def view_to_dense(view):
    n_l, n_h = view["n_local"], view["n_halo"]
    P = np.zeros((n_l, n_l + n_h))
    for i in range(n_l):
        for k in range(view["rowptr"][i], view["rowptr"][i + 1]):
            assert P[i, view["col"][k]] == 0.0, "duplicate column in a row"
            P[i, view["col"][k]] = view["val"][k]
    return P


def tiny_problem():
    cfg = syn.get_config("tiny")
    ss = syn.substreams(cfg["seed"])
    g = syn.make_graph(cfg, np.random.default_rng(ss["graph"]))
    return cfg, ss, g


# --------------------------------------------------- propagation matrix pins
def test_path4_matches_hand_derived_fixture():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "path4_a_hat.txt"))
            if l.strip() and not l.startswith("#")]
    expect = np.zeros((4, 4))
    for i, j, v in rows:
        expect[int(i), int(j)] = float(v)
    rowptr = np.array([0, 1, 3, 5, 6], dtype=np.int64)
    col = np.array([1, 0, 2, 1, 3, 2], dtype=np.int32)
    part = np.array([0, 0, 1, 1], dtype=np.int32)
    for m, loc in ((0, [0, 1]), (1, [2, 3])):
        v = orc.partition_view(4, rowptr, col, part, m)
        P = view_to_dense(v)
        ids = np.concatenate([v["local_ids"], v["halo_ids"]])
        assert list(v["local_ids"]) == loc
        np.testing.assert_allclose(P, expect[np.ix_(loc, ids)], rtol=2e-7)
        # worked aggregate for features x = (1, 2, 3, 4): row 0 of partition 0
        # is 1/2 * 1 + 1/sqrt(6) * 2
        x = np.arange(1.0, 5.0)[:, None].astype(np.float32)
        agg = orc.spmm_fwd(v, x[ids])
        np.testing.assert_allclose(agg[:, 0], expect[loc] @ x[:, 0], rtol=2e-7)


def test_partition_view_against_dense_brute_force():
    g = small_graph()
    A, Ahat, dt = dense_a_hat(g)
    for m in range(g.n_parts):
        v = orc.partition_view(g.N, g.rowptr, g.col, g.part, m)
        loc = np.flatnonzero(g.part == m)
        out = np.flatnonzero(g.part != m)
        halo = out[np.flatnonzero(A[np.ix_(loc, out)].sum(axis=0) > 0)]
        assert np.array_equal(v["local_ids"], loc)
        assert np.array_equal(v["halo_ids"], halo)
        assert v["local_ids"].dtype == np.int32 and v["halo_ids"].dtype == np.int32
        P = view_to_dense(v)
        np.testing.assert_allclose(P[:, :loc.size], Ahat[np.ix_(loc, loc)], rtol=3e-7, atol=0)
        np.testing.assert_allclose(P[:, loc.size:], Ahat[np.ix_(loc, halo)], rtol=3e-7, atol=0)
        # canonical order: columns ascending in every row, split = first halo column
        for i in range(loc.size):
            c = v["col"][v["rowptr"][i]:v["rowptr"][i + 1]]
            assert np.all(np.diff(c) > 0)
            k = v["split"][i] - v["rowptr"][i]
            assert np.all(c[:k] < loc.size) and np.all(c[k:] >= loc.size)
        # nnz(P_in) + nnz(P_out) = sum of d_tilde over the partition
        assert v["nnz"] == int(dt[loc].sum())
        # transposed halo block is exactly the transpose of P_out
        PT = np.zeros((halo.size, loc.size))
        for u in range(halo.size):
            r = v["h_row"][v["h_colptr"][u]:v["h_colptr"][u + 1]]
            assert np.all(np.diff(r) > 0)
            PT[u, r] = v["h_val"][v["h_colptr"][u]:v["h_colptr"][u + 1]]
        assert np.array_equal(PT, P[:, loc.size:].T)
        assert v["nnz_halo"] == int((P[:, loc.size:] != 0).sum())
        np.testing.assert_allclose(v["h_self"], np.diag(Ahat)[halo], rtol=3e-7)


def test_values_are_one_fp32_product_in_unit_interval():
    g = small_graph(seed=5)
    v = orc.partition_view(g.N, g.rowptr, g.col, g.part, 1)
    isd = (1.0 / np.sqrt(1.0 + np.diff(g.rowptr).astype(np.float64))).astype(np.float32)
    ids = np.concatenate([v["local_ids"], v["halo_ids"]])
    rows = np.repeat(np.arange(v["n_local"]), np.diff(v["rowptr"]))
    expect = isd[v["local_ids"][rows]] * isd[ids[v["col"]]]
    assert expect.dtype == np.float32
    assert np.array_equal(v["val"].view(np.uint32), expect.view(np.uint32))
    assert np.all(v["val"] > 0) and np.all(v["val"] <= 1)


def test_sqrt_degree_is_a_fixed_vector():
    # A_hat sqrt(d_tilde) = sqrt(d_tilde)  =>  on a partition
    # [P_in | P_out] sqrt(d_tilde)[local ++ halo] = sqrt(d_tilde)[local]
    cfg, ss, g = tiny_problem()
    v = orc.partition_view(g.N, g.rowptr, g.col, g.part, 0)
    sd = np.sqrt(1.0 + np.diff(g.rowptr).astype(np.float64))
    ids = np.concatenate([v["local_ids"], v["halo_ids"]])
    agg = orc.spmm_fwd(v, sd[ids][:, None])
    np.testing.assert_allclose(agg[:, 0], sd[v["local_ids"]], rtol=5e-7)


def test_ring_graph_is_three_point_mean():
    g = syn.ring_graph(64, n_parts=2)
    v = orc.partition_view(g.N, g.rowptr, g.col, g.part, 0)
    assert np.all(v["val"] == np.float32(1.0 / np.sqrt(3.0)) * np.float32(1.0 / np.sqrt(3.0)))
    assert list(v["halo_ids"]) == [32, 63]
    rng = np.random.default_rng(0)
    X = rng.standard_normal((64, 5)).astype(np.float32)
    ids = np.concatenate([v["local_ids"], v["halo_ids"]])
    agg = orc.spmm_fwd(v, X[ids])
    Xd = X.astype(np.float64)
    mean3 = (np.roll(Xd, 1, axis=0) + Xd + np.roll(Xd, -1, axis=0)) / 3.0
    np.testing.assert_allclose(agg, mean3[:32], rtol=1e-6, atol=1e-7)


def test_degree_override_changes_only_values():
    g = small_graph(seed=9)
    v0 = orc.partition_view(g.N, g.rowptr, g.col, g.part, 0)
    deg = np.diff(g.rowptr) + 3
    v1 = orc.partition_view(g.N, g.rowptr, g.col, g.part, 0, g_deg=deg)
    for k in ("rowptr", "split", "col", "halo_ids", "h_colptr", "h_row"):
        assert np.array_equal(v0[k], v1[k])
    assert not np.array_equal(v0["val"], v1["val"])
    isd = (1.0 / np.sqrt(1.0 + deg.astype(np.float64))).astype(np.float32)
    assert np.array_equal(v1["h_self"], isd[v1["halo_ids"]] * isd[v1["halo_ids"]])


# ------------------------------------------------------------ SpMM pins
def test_spmm_fwd_matches_scipy_and_dense():
    cfg, ss, g = tiny_problem()
    v = orc.partition_view(g.N, g.rowptr, g.col, g.part, 0)
    rng = np.random.default_rng(1)
    Hbar = rng.standard_normal((v["n_local"] + v["n_halo"], 9)).astype(np.float32)
    agg = orc.spmm_fwd(v, Hbar)
    M = sp.csr_matrix((v["val"].astype(np.float64), v["col"], v["rowptr"]),
                      shape=(v["n_local"], v["n_local"] + v["n_halo"]))
    np.testing.assert_allclose(agg, M @ Hbar.astype(np.float64), rtol=1e-12, atol=1e-13)
    rows = [0, 5, v["n_local"] - 1]
    np.testing.assert_allclose(orc.spmm_fwd_rows(v, Hbar, rows), agg[rows], rtol=1e-13)
    # linearity
    H2 = rng.standard_normal(Hbar.shape).astype(np.float32)
    lhs = orc.spmm_fwd(v, 2.0 * Hbar.astype(np.float64) - 0.5 * H2)
    np.testing.assert_allclose(lhs, 2.0 * agg - 0.5 * orc.spmm_fwd(v, H2), rtol=1e-11, atol=1e-12)


def test_spmm_bwd_is_the_transpose():
    g = small_graph(seed=11)
    v = orc.partition_view(g.N, g.rowptr, g.col, g.part, 2)
    P = view_to_dense(v)
    rng = np.random.default_rng(2)
    G = rng.standard_normal((v["n_local"], 7)).astype(np.float32)
    dl, dh = orc.spmm_bwd(v, G, want_halo=True)
    full = P.T @ G.astype(np.float64)
    np.testing.assert_allclose(dl, full[:v["n_local"]], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dh, full[v["n_local"]:], rtol=1e-12, atol=1e-13)
    dl2, none = orc.spmm_bwd(v, G)
    assert none is None
    np.testing.assert_allclose(dl2, dl, rtol=1e-13, atol=1e-14)
    rows = np.arange(0, v["n_local"], 3)
    np.testing.assert_allclose(orc.spmm_bwd_rows(v, G, rows), dl[rows], rtol=1e-12, atol=1e-13)
    # inner-product identity <P H, G> = <H, P^T G>
    H = rng.standard_normal((v["n_local"] + v["n_halo"], 7)).astype(np.float32)
    lhs = np.sum(orc.spmm_fwd(v, H) * G)
    rhs = np.sum(H[:v["n_local"]] * dl) + np.sum(H[v["n_local"]:] * dh)
    assert abs(lhs - rhs) <= 1e-10 * abs(lhs)


# ------------------------------------------------ zero-staleness invariant
def test_zero_staleness_equals_full_graph_gcn():
    cfg, ss, g = tiny_problem()
    dims = cfg["dims"]
    X = syn.normal_f32(ss["features"], g.N, dims[0])
    wss = ss["weights"].spawn(len(dims) - 1)
    Ws = [syn.glorot_uniform_f32(wss[l], dims[l], dims[l + 1]) for l in range(len(dims) - 1)]
    Hfull = orc.full_graph_gcn(g.N, g.rowptr, g.col, X, Ws)
    for m in (0, 1):
        v = orc.partition_view(g.N, g.rowptr, g.col, g.part, m)
        y = syn.labels_i32(ss["labels"], v["n_local"], dims[-1])
        halo_hat = [None] + [Hfull[l][v["halo_ids"]] for l in range(1, len(Ws))]
        st = orc.partition_step(v, X[v["local_ids"]], X[v["halo_ids"]], halo_hat, Ws, y)
        for l in range(len(Ws) + 1):
            np.testing.assert_allclose(st["H"][l], Hfull[l][v["local_ids"]],
                                       rtol=1e-11, atol=1e-12)


def test_dropping_halo_breaks_the_invariant():
    # sanity of the pin itself: the halo term matters on this graph
    cfg, ss, g = tiny_problem()
    X = syn.normal_f32(ss["features"], g.N, 4)
    v = orc.partition_view(g.N, g.rowptr, g.col, g.part, 0)
    W = [np.eye(4, dtype=np.float32)]
    Hfull = orc.full_graph_gcn(g.N, g.rowptr, g.col, X, W)
    Hbar = np.concatenate([X[v["local_ids"]], np.zeros((v["n_halo"], 4), np.float32)])
    assert np.abs(orc.spmm_fwd(v, Hbar) - Hfull[1][v["local_ids"]]).max() > 1e-2


# ------------------------------------------------------------ dense pins
def test_dense_fwd_bwd_textbook():
    rng = np.random.default_rng(4)
    A = rng.standard_normal((50, 12)).astype(np.float32)
    W = rng.standard_normal((12, 7)).astype(np.float32)
    dH = rng.standard_normal((50, 7)).astype(np.float32)
    Z, H = orc.dense_fwd(A, W, 1)
    Zb = np.einsum("ik,kj->ij", A.astype(np.float64), W.astype(np.float64))
    np.testing.assert_allclose(Z, Zb, rtol=1e-13, atol=1e-14)
    assert np.array_equal(H, np.where(Zb > 0, Zb, 0.0))
    dW, dA, dZ = orc.dense_bwd(dH, Z, A, W, 1)
    mask = (Zb > 0).astype(np.float64)
    np.testing.assert_allclose(dW, np.einsum("ik,ij->kj", A.astype(np.float64), dH * mask), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dA, np.einsum("ij,kj->ik", dH * mask, W.astype(np.float64)), rtol=1e-12, atol=1e-13)
    Z0, H0 = orc.dense_fwd(A, W, 0)
    assert np.array_equal(Z0, H0)
    dW0, dA0, _ = orc.dense_bwd(dH, Z0, A, W, 0)
    np.testing.assert_allclose(dW0, A.astype(np.float64).T @ dH, rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------- loss pins
def test_loss_gradient_properties_and_fd():
    rng = np.random.default_rng(6)
    HL = rng.standard_normal((13, 5))
    y = rng.integers(0, 5, size=13)
    loss, g = orc.loss_and_grad(HL, y)
    np.testing.assert_allclose(g.sum(axis=1), 0.0, atol=1e-15)
    p = g * 13
    p[np.arange(13), y] += 1.0
    np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=1e-13)
    # uniform logits: loss = log C
    l0, _ = orc.loss_and_grad(np.zeros((4, 5)), np.array([0, 1, 2, 3]))
    assert abs(l0 - np.log(5.0)) < 1e-14
    eps = 1e-6
    for (i, j) in [(0, 0), (3, 2), (12, 4)]:
        Hp, Hm = HL.copy(), HL.copy()
        Hp[i, j] += eps
        Hm[i, j] -= eps
        fd = (orc.loss_and_grad(Hp, y)[0] - orc.loss_and_grad(Hm, y)[0]) / (2 * eps)
        assert abs(fd - g[i, j]) < 1e-8


# ------------------------------------------------ backward: finite differences
def _fd_problem():
    g = small_graph(seed=21, N=90, n_parts=3)
    v = orc.partition_view(g.N, g.rowptr, g.col, g.part, 1)
    rng = np.random.default_rng(8)
    dims = [6, 5, 4, 3]
    X = rng.standard_normal((g.N, dims[0])).astype(np.float32)
    Ws = [(0.7 * rng.standard_normal((dims[l], dims[l + 1]))).astype(np.float32) for l in range(3)]
    halo_hat = [None] + [rng.standard_normal((v["n_halo"], dims[l])).astype(np.float32) for l in (1, 2)]
    y = rng.integers(0, dims[-1], size=v["n_local"])
    return g, v, X, Ws, halo_hat, y


def test_backward_dW_matches_central_differences():
    g, v, X, Ws, halo_hat, y = _fd_problem()
    Xl, Xh = X[v["local_ids"]], X[v["halo_ids"]]
    st = orc.partition_step(v, Xl, Xh, halo_hat, Ws, y)
    eps = 1e-5
    rng = np.random.default_rng(0)
    for l in range(3):
        for _ in range(6):
            i, j = rng.integers(Ws[l].shape[0]), rng.integers(Ws[l].shape[1])
            Wp = [w.astype(np.float64) for w in Ws]
            Wm = [w.astype(np.float64) for w in Ws]
            Wp[l][i, j] += eps
            Wm[l][i, j] -= eps
            fd = (orc.partition_step(v, Xl, Xh, halo_hat, Wp, y)["loss"]
                  - orc.partition_step(v, Xl, Xh, halo_hat, Wm, y)["loss"]) / (2 * eps)
            assert abs(fd - st["dW"][l][i, j]) <= 1e-7 + 1e-5 * abs(fd), (l, i, j)


def _loss_from_layer(v, l0, H_l0, X_halo, halo_hat, Ws, y):
    """Loss as a function of the local rows entering layer l0+1 (forward
    functions only; these are pinned separately)."""
    L = len(Ws)
    H = np.asarray(H_l0, np.float64)
    for l in range(l0, L):
        halo = X_halo if l == 0 else halo_hat[l]
        Hbar = np.concatenate([H, np.asarray(halo, np.float64)])
        _, H = orc.dense_fwd(orc.spmm_fwd(v, Hbar), Ws[l], 1 if l < L - 1 else 0)
    return orc.loss_and_grad(H, y)[0]


def test_backward_dH_in_matches_central_differences():
    g, v, X, Ws, halo_hat, y = _fd_problem()
    Xl, Xh = X[v["local_ids"]], X[v["halo_ids"]]
    st = orc.partition_step(v, Xl, Xh, halo_hat, Ws, y)
    assert st["dH_in"][0] is None          # no gradient w.r.t. input features
    eps = 1e-5
    rng = np.random.default_rng(1)
    for l in (1, 2):
        for _ in range(8):
            i, j = rng.integers(v["n_local"]), rng.integers(st["H"][l].shape[1])
            Hp, Hm = st["H"][l].copy(), st["H"][l].copy()
            Hp[i, j] += eps
            Hm[i, j] -= eps
            fd = (_loss_from_layer(v, l, Hp, Xh, halo_hat, Ws, y)
                  - _loss_from_layer(v, l, Hm, Xh, halo_hat, Ws, y)) / (2 * eps)
            assert abs(fd - st["dH_in"][l][i, j]) <= 1e-8 + 1e-5 * abs(fd), (l, i, j)


def test_halo_rows_change_the_loss_but_get_no_gradient():
    g, v, X, Ws, halo_hat, y = _fd_problem()
    Xl, Xh = X[v["local_ids"]], X[v["halo_ids"]]
    st = orc.partition_step(v, Xl, Xh, halo_hat, Ws, y)
    hh = [None, halo_hat[1] + 0.1, halo_hat[2]]
    assert abs(orc.partition_step(v, Xl, Xh, hh, Ws, y)["loss"] - st["loss"]) > 1e-6
    # the step's own gradient stops at the local rows: dH_in is P_in^T dAGG alone; the
    # halo term P_out^T dAGG is a separate output for the nodes' owners, used nowhere here
    for l in (1, 2):
        assert np.array_equal(st["dH_in"][l], orc.spmm_bwd(v, st["dAGG"][l])[0])
        assert st["dH_halo"][l].shape == (v["n_halo"], st["dAGG"][l].shape[1])


def test_one_layer_dW_equals_masked_full_graph_gradient():
    g = small_graph(seed=31, N=60, n_parts=2)
    A, Ahat, dt = dense_a_hat(g)
    v = orc.partition_view(g.N, g.rowptr, g.col, g.part, 0)
    rng = np.random.default_rng(3)
    X = rng.standard_normal((g.N, 5)).astype(np.float32)
    W = rng.standard_normal((5, 4)).astype(np.float32)
    y = rng.integers(0, 4, size=v["n_local"])
    st = orc.partition_step(v, X[v["local_ids"]], X[v["halo_ids"]], [None], [W], y)
    loc = v["local_ids"]
    # finite differences of the dense full-graph loss restricted to V_m
    def loss_of(Wd):
        return orc.loss_and_grad((Ahat @ X.astype(np.float64) @ Wd)[loc], y)[0]
    eps = 1e-6
    for (i, j) in [(0, 0), (2, 3), (4, 1)]:
        Wp, Wm = W.astype(np.float64), W.astype(np.float64)
        Wp[i, j] += eps
        Wm[i, j] -= eps
        fd = (loss_of(Wp) - loss_of(Wm)) / (2 * eps)
        assert abs(fd - st["dW"][0][i, j]) < 2e-7


# ------------------------------------------------------- gather / push pins
def test_gather_push_roundtrip_and_isolation():
    rng = np.random.default_rng(12)
    table = rng.standard_normal((40, 6)).astype(np.float32)
    ids = np.array([7, 0, 39, 7, 12], dtype=np.int32)
    out = orc.history_gather(table, ids)
    assert out.dtype == np.float32 and np.array_equal(out, table[[7, 0, 39, 7, 12]])
    out[0, 0] = 99.0
    assert table[7, 0] != 99.0             # a copy, not a view
    H = rng.standard_normal((3, 4)).astype(np.float32)
    before = table.copy()
    pid = np.array([5, 1, 30], dtype=np.int32)
    orc.history_push(table, pid, H)
    assert np.array_equal(orc.history_gather(table, pid)[:, :4], H)
    untouched = np.setdiff1d(np.arange(40), pid)
    assert np.array_equal(table[untouched], before[untouched])
    assert np.array_equal(table[pid, 4:], before[pid, 4:])


# ---------------------------------------------------------- predictor pins
def test_lstm_matches_torch_cpu_library_routine():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(14)
    n, d, d_s, tau = 11, 6, 5, 3
    p = syn.predictor_params_f32(np.random.SeedSequence(2), d, d_s)
    slots = [rng.standard_normal((n, d)).astype(np.float32) for _ in range(tau)]
    S = orc.lstm_last_hidden(slots, p["Wx"], p["Wh"], p["b"])
    lstm = torch.nn.LSTM(d, d_s, num_layers=1, batch_first=False).double()
    with torch.no_grad():
        lstm.weight_ih_l0.copy_(torch.from_numpy(p["Wx"].astype(np.float64)))
        lstm.weight_hh_l0.copy_(torch.from_numpy(p["Wh"].astype(np.float64)))
        lstm.bias_ih_l0.copy_(torch.from_numpy(p["b"].astype(np.float64)))
        lstm.bias_hh_l0.zero_()
        x = torch.from_numpy(np.stack(slots).astype(np.float64))   # [tau, n, d]
        _, (hN, _) = lstm(x)
    np.testing.assert_allclose(S, hN[0].numpy(), rtol=1e-12, atol=1e-13)
    assert np.all(np.abs(S) < 1.0)


def test_lstm_tau1_closed_form():
    rng = np.random.default_rng(15)
    n, d, d_s = 9, 4, 3
    p = syn.predictor_params_f32(np.random.SeedSequence(5), d, d_s)
    x = rng.standard_normal((n, d)).astype(np.float32)
    S = orc.lstm_last_hidden([x], p["Wx"], p["Wh"], p["b"])
    sig = lambda t: 1.0 / (1.0 + np.exp(-t))
    for r in range(n):
        for j in range(d_s):
            pre = [float(p["Wx"][k * d_s + j].astype(np.float64) @ x[r].astype(np.float64)
                         + p["b"][k * d_s + j]) for k in range(4)]
            c = sig(pre[0]) * np.tanh(pre[2])          # f * c_0 vanishes
            assert abs(S[r, j] - sig(pre[3]) * np.tanh(c)) < 1e-14


def test_predictor_hop_against_dense_brute_force():
    g = small_graph(seed=17)
    A, Ahat, dt = dense_a_hat(g)
    v = orc.partition_view(g.N, g.rowptr, g.col, g.part, 0)
    rng = np.random.default_rng(16)
    d_s, d = 4, 6
    S = rng.standard_normal((v["n_local"] + v["n_halo"], d_s)).astype(np.float32)
    Wg = rng.standard_normal((d_s, d)).astype(np.float32)
    loc, halo = v["local_ids"], v["halo_ids"]
    S64 = S.astype(np.float64)
    expect = (Ahat[np.ix_(halo, loc)] @ S64[:loc.size]
              + np.diag(Ahat)[halo][:, None] * S64[loc.size:]) @ Wg.astype(np.float64)
    np.testing.assert_allclose(orc.predictor_hop(v, S, Wg), expect, rtol=2e-6, atol=1e-7)


def test_predictor_identity_cases():
    g = small_graph(seed=19)
    v = orc.partition_view(g.N, g.rowptr, g.col, g.part, 1)
    rng = np.random.default_rng(18)
    d, d_s, tau = 6, 4, 2
    p = syn.predictor_params_f32(np.random.SeedSequence(7), d, d_s)
    slots = [rng.standard_normal((v["n_local"] + v["n_halo"], d)).astype(np.float32)
             for _ in range(tau)]
    newest = slots[-1][v["n_local"]:].astype(np.float64)
    assert np.array_equal(orc.predict(v, p, slots, bypass=True), newest)
    p0 = dict(p, Wg=np.zeros_like(p["Wg"]))
    assert np.array_equal(orc.predict(v, p0, slots), newest)
    out = orc.predict(v, p, slots)
    assert out.shape == newest.shape and np.abs(out - newest).max() > 1e-3
    # the correction is bounded: |S| < 1 and rows of [P_out^T | diag] sum below sqrt-degree bounds
    S = orc.lstm_last_hidden(slots, p["Wx"], p["Wh"], p["b"])
    np.testing.assert_allclose(out - newest, orc.predictor_hop(v, S, p["Wg"]), rtol=1e-13, atol=1e-15)


def test_staleness_norm_is_frobenius():
    a = np.array([[3.0, 0.0], [0.0, 4.0]])
    assert orc.staleness(a, np.zeros((2, 2))) == 5.0


def test_round_bf16_matches_library_conversion():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(30)
    x = np.concatenate([rng.standard_normal(50000), 1e-3 * rng.standard_normal(1000),
                        [0.0, 1.0, -1.0, 1.00390625, 1.01171875, 3.0e38]]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(orc.round_bf16(x), ref)
    # halfway cases go to the even neighbour: 1 + 2^-8 -> 1, 1 + 3 * 2^-8 -> 1 + 2^-6
    assert orc.round_bf16(np.float32(1.00390625)) == 1.0
    assert orc.round_bf16(np.float32(1.01171875)) == 1.015625


def test_partition_step_store_hook_only_rounds_storage():
    g, v, X, Ws, halo_hat, y = _fd_problem()
    Xl, Xh = X[v["local_ids"]], X[v["halo_ids"]]
    a = orc.partition_step(v, Xl, Xh, halo_hat, Ws, y)
    b = orc.partition_step(v, Xl, Xh, halo_hat, Ws, y, store=lambda t: t)
    assert a["loss"] == b["loss"] and all(np.array_equal(p, q) for p, q in zip(a["dW"], b["dW"]))
    c = orc.partition_step(v, Xl, Xh, halo_hat, Ws, y, store=orc.round_bf16)
    assert abs(c["loss"] - a["loss"]) < 2e-2 * abs(a["loss"])
    for l in range(len(Ws)):
        assert np.array_equal(c["AGG"][l], orc.round_bf16(c["AGG"][l]))
        rel = np.linalg.norm(c["dW"][l] - a["dW"][l]) / np.linalg.norm(a["dW"][l])
        assert rel < 3e-2


def test_partition_view_sample_agrees_with_the_full_view():
    """The sampled form used for graphs too large for the per-node loops gives
    the same id lists, offsets and entries as the full view (scattered and
    contiguous partitions, explicit degrees)."""
    rng = np.random.default_rng(5)
    g = syn.make_graph(syn.get_config("tiny"), rng)
    part_scattered = rng.integers(0, 3, size=g.N).astype(np.int32)
    deg = (np.diff(g.rowptr) + rng.integers(0, 4, size=g.N)).astype(np.int32)
    for part, m, gd in ((g.part, 1, None), (part_scattered, 2, deg)):
        full = orc.partition_view(g.N, g.rowptr, g.col, part, m, g_deg=gd)
        rows = rng.choice(full["n_local"], size=40, replace=False)
        hs = rng.choice(full["n_halo"], size=40, replace=False)
        smp = orc.partition_view_sample(g.N, g.rowptr, g.col, part, m, rows, hs, g_deg=gd)
        for k in ("n_local", "n_halo", "nnz", "nnz_halo"):
            assert smp[k] == full[k]
        for k in ("local_ids", "halo_ids", "rowptr", "h_colptr"):
            assert np.array_equal(smp[k], full[k]), k
        assert np.array_equal(smp["h_self"].view(np.uint32), full["h_self"].view(np.uint32))
        for i in rows:
            c, v, sp_off = smp["row_entries"][int(i)]
            s0, e0 = full["rowptr"][i], full["rowptr"][i + 1]
            assert np.array_equal(c, full["col"][s0:e0])
            assert np.array_equal(v.view(np.uint32), full["val"][s0:e0].view(np.uint32))
            assert s0 + sp_off == full["split"][i]
        for u in hs:
            r, v = smp["halo_entries"][int(u)]
            s0, e0 = full["h_colptr"][u], full["h_colptr"][u + 1]
            assert np.array_equal(r, full["h_row"][s0:e0])
            assert np.array_equal(v.view(np.uint32), full["h_val"][s0:e0].view(np.uint32))


def test_partition_rows_generator_is_a_valid_partition_view_input():
    """The partition-only generator: symmetric local block, no loops, ascending
    duplicate-free rows, empty rows outside the partition, degrees >= what the
    partition sees; and the oracle's view of it has P_in symmetric."""
    cfg = syn.get_config("scale_rows_small")
    cfg["N"] = 80_000
    g = syn.make_graph(cfg, np.random.default_rng(1))
    n_l = g.N // cfg["n_parts"]
    assert g.deg is not None and np.all(np.diff(g.rowptr)[n_l:] == 0)
    assert np.array_equal(g.deg[:n_l], np.diff(g.rowptr)[:n_l])
    for i in (0, 1, n_l // 2, n_l - 1):
        r = g.col[g.rowptr[i]:g.rowptr[i + 1]]
        assert np.all(np.diff(r) > 0) and i not in r
    v = orc.partition_view(g.N, g.rowptr, g.col, g.part, 0, g_deg=g.deg)
    assert v["n_local"] == n_l and v["n_halo"] > 0
    import scipy.sparse as sp
    P = sp.csr_matrix((v["val"], v["col"], v["rowptr"]), shape=(n_l, n_l + v["n_halo"]))
    P_in = P[:, :n_l]
    assert abs(P_in - P_in.T).max() == 0
    cross = g.col[g.col >= n_l]
    assert np.all(g.deg[cross] >= 1)
    frac = cross.size / g.nnz
    assert 0.07 < frac < 0.13          # about the 10 % cut of the recipe


def test_stale_gradient_term_completes_the_full_graph_backward():
    """Appendix, SAT backward: G_H = P_in^T D W^T + P_out^T D~ W^T. With nothing stale
    (true halo embeddings, the other partition's term taken from the same step) the
    two partitions' backward passes, after exchanging their P_out^T terms, must give
    the unpartitioned GCN's gradients: G_H^(1) row by row and dW summed over the
    partitions. Dropping, transposing or mis-routing the second term breaks it."""
    cfg = syn.get_config("tiny")
    ss = syn.substreams(3)
    g = syn.make_graph(cfg, np.random.default_rng(ss["graph"]))
    dims = cfg["dims"]
    X = syn.normal_f32(ss["features"], g.N, dims[0])
    wss = ss["weights"].spawn(2)
    Ws = [syn.glorot_uniform_f32(wss[l], dims[l], dims[l + 1]) for l in range(2)]
    y_all = syn.labels_i32(ss["labels"], g.N, dims[-1])
    Hfull = orc.full_graph_gcn(g.N, g.rowptr, g.col, X, Ws)
    G_H, dW_full = orc.full_graph_backward(g.N, g.rowptr, g.col, X, Ws, y_all, g.part)
    views = [orc.partition_view(g.N, g.rowptr, g.col, g.part, m) for m in (0, 1)]

    def run(m, stale):
        v = views[m]
        return orc.partition_step(v, X[v["local_ids"]], X[v["halo_ids"]],
                                  [None, Hfull[1][v["halo_ids"]]], Ws, y_all[v["local_ids"]],
                                  stale_grad=stale)

    first = [run(m, None) for m in (0, 1)]
    second = []
    for m in (0, 1):
        v, other = views[m], views[1 - m]
        # rows of this partition's local nodes in the other partition's halo gradient
        recv = np.zeros((v["n_local"], dims[1]))
        pos = np.searchsorted(v["local_ids"], other["halo_ids"])
        recv[pos] = first[1 - m]["dH_halo"][1]
        second.append(run(m, [None, recv]))
        np.testing.assert_allclose(second[m]["dH_in"][1], G_H[1][v["local_ids"]], rtol=1e-9, atol=1e-12)
        # without the second term the rows that have outside neighbours are wrong
        touched = np.zeros(v["n_local"], bool)
        touched[pos] = True
        err = np.abs(first[m]["dH_in"][1] - G_H[1][v["local_ids"]]).max(axis=1)
        assert err[touched].min() > 0 and err[~touched].max() < 1e-12
    for l in range(2):
        np.testing.assert_allclose(second[0]["dW"][l] + second[1]["dW"][l], dW_full[l],
                                   rtol=1e-9, atol=1e-12)


# ---------------------------------------------------------------- predictor training (Eq. 11, 12)
def _train_problem(seed=0, tau=3, d=6, d_s=4):
    g = small_graph(seed=seed, N=70, n_parts=2)
    v = orc.partition_view(g.N, g.rowptr, g.col, g.part, 0)
    rng = np.random.default_rng(seed + 100)
    n_bar = v["n_local"] + v["n_halo"]
    omega = {k: a.astype(np.float64) for k, a in
             syn.predictor_params_f32(np.random.SeedSequence(seed), d, d_s).items()}
    slots = [rng.standard_normal((n_bar, d)) for _ in range(tau)]
    target = rng.standard_normal((v["n_local"], d))
    weight = rng.integers(0, 2, size=v["n_local"]).astype(np.float64)
    return v, omega, slots, target, weight


def test_predictor_training_gradients_by_finite_differences():
    """Every parameter tensor of the predictor, tau = 1, 2, 3, with and without a
    mini-batch mask: central differences of the loss itself."""
    for tau in (1, 2, 3):
        v, omega, slots, target, weight = _train_problem(seed=tau, tau=tau)
        for wgt in (None, weight):
            loss, grads = orc.predictor_train_loss_and_grad(v, omega, slots, target, wgt)
            rng = np.random.default_rng(tau)
            eps = 1e-6
            for name in ("Wx", "Wh", "b", "Wg"):
                if tau == 1 and name == "Wh":
                    assert np.all(grads["Wh"] == 0)       # h_0 = 0: no recurrent term yet
                    continue
                for _ in range(6):
                    idx = tuple(rng.integers(0, n) for n in omega[name].shape)
                    op = {k: a.copy() for k, a in omega.items()}
                    om = {k: a.copy() for k, a in omega.items()}
                    op[name][idx] += eps
                    om[name][idx] -= eps
                    fd = (orc.predictor_train_loss_and_grad(v, op, slots, target, wgt)[0]
                          - orc.predictor_train_loss_and_grad(v, om, slots, target, wgt)[0]) / (2 * eps)
                    assert abs(fd - grads[name][idx]) <= 1e-9 + 2e-6 * abs(fd), (tau, name, idx)


def test_predictor_training_special_cases():
    v, omega, slots, target, weight = _train_problem(seed=7, tau=2)
    n_l = v["n_local"]
    # Wg = 0: the prediction is the newest cached embedding, the LSTM gets no gradient
    o0 = dict(omega, Wg=np.zeros_like(omega["Wg"]))
    loss, grads = orc.predictor_train_loss_and_grad(v, o0, slots, target)
    assert abs(loss - np.mean((slots[-1][:n_l] - target) ** 2)) < 1e-14
    assert np.all(grads["Wx"] == 0) and np.all(grads["Wh"] == 0) and np.all(grads["b"] == 0)
    assert np.abs(grads["Wg"]).max() > 0
    # the local-row hop is the same propagation as the halo-row hop of inference: a
    # target equal to the prediction gives zero loss and zero gradients
    S = orc.lstm_last_hidden(slots, omega["Wx"], omega["Wh"], omega["b"])
    pred = slots[-1][:n_l] + orc.spmm_fwd(v, S) @ omega["Wg"]
    loss, grads = orc.predictor_train_loss_and_grad(v, omega, slots, pred)
    assert loss < 1e-28 and all(np.abs(gr).max() < 1e-13 for gr in grads.values())
    # a 0/1 mask is the same as dropping the rows from the mean
    loss_m, _ = orc.predictor_train_loss_and_grad(v, omega, slots, target, weight)
    keep = weight > 0
    assert abs(loss_m - np.mean(((pred - target) ** 2)[keep])) < 1e-12
    # a few plain gradient steps lower the loss (Alg. 1, predictor update)
    om = {k: a.copy() for k, a in omega.items()}
    l0 = None
    for it in range(5):
        l, gr = orc.predictor_train_loss_and_grad(v, om, slots, target)
        l0 = l if l0 is None else l0
        for k in om:
            om[k] -= 0.05 * gr[k]
    assert orc.predictor_train_loss_and_grad(v, om, slots, target)[0] < l0


# ---------------------------------------------------------------- compression codec
def test_polyline_codes_match_the_published_examples():
    path = os.path.join(os.path.dirname(__file__), "golden", "polyline_examples.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 3
    for value, prec, code in rows:
        q = orc.polyline_quantise(np.array([float(value)]), int(prec), arith=np.float64)[0]
        assert orc.polyline_encode_value(q) == code.encode("ascii"), (value, q)
    # two values in a row are the concatenation of their codes
    codes, off = orc.polyline_encode_rows(np.array([[38.5, -120.2]]), 5, arith=np.float64)
    assert codes.tobytes() == b"_p~iF~ps|U" and list(off) == [0, 10]


def test_polyline_round_trip_error_bound_and_lengths():
    rng = np.random.default_rng(4)
    H = np.maximum(rng.standard_normal((50, 37)), 0).astype(np.float32) * 3.0   # relu-like: half zeros
    H[3, 5], H[7, 0] = -123.456, 1e-9
    for prec in (1, 2, 4):
        codes, off = orc.polyline_encode_rows(H, prec)
        assert codes.min() >= 63 and codes.max() <= 126             # printable ASCII, as the format says
        back = orc.polyline_decode_rows(codes, off, np.arange(50), 37, prec)
        # lossy by at most half a unit of the kept decimal place (plus fp32 rounding of the product)
        assert np.abs(back.astype(np.float64) - H).max() <= 0.5 * 10.0 ** -prec * (1 + 1e-5) + 1e-6
        # coding what was decoded gives the same bytes: the codec is idempotent
        codes2, off2 = orc.polyline_encode_rows(back, prec)
        assert np.array_equal(codes, codes2) and np.array_equal(off, off2)
        # zero takes one byte ('?'), and the row offsets add up
        assert orc.polyline_encode_value(0) == b"?"
        assert off[-1] == codes.size and np.all(np.diff(off) >= 37)
        # gather by id decodes the right rows
        ids = np.array([49, 0, 7, 7])
        assert np.array_equal(orc.polyline_decode_rows(codes, off, ids, 37, prec), back[ids])
        # the whole-table shortcut returns bit for bit what goes through the bytes
        assert np.array_equal(orc.polyline_stored_value(H, prec).view(np.uint32), back.view(np.uint32))
    # fewer decimals, fewer bytes; relu-shaped rows at one decimal beat 3x against fp32
    sizes = [orc.polyline_encode_rows(H, p)[1][-1] for p in (1, 2, 4)]
    assert sizes[0] < sizes[1] < sizes[2]
    base = np.maximum(rng.standard_normal((200, 256)), 0).astype(np.float32)
    assert 4.0 * base.size / orc.polyline_encode_rows(base, 1)[1][-1] > 3.0


def test_polyline_out_of_range_values_saturate_and_nan_codes_as_zero():
    """The edge clauses of the quantiser (the paper's compression section says nothing about
    them; reading: hold |q| at 2^30, the largest magnitude whose shifted code fits 32 bits
    for either sign, and code NaN as 0). The byte strings below are derived by hand from the
    format's rules: 2^30 shifts to 2^31 = six zero groups with a successor (0x20 + 63 = '_')
    and a last group 2 (+ 63 = 'A'); -2^30 shifts to 2^31 and inverts to 2^31 - 1 = six
    all-ones groups with a successor (31 + 32 + 63 = '~') and a last group 1 ('@')."""
    QM = 1 << 30
    assert orc.POLYLINE_Q_MAX == QM
    assert orc.polyline_encode_value(QM) == b"______A"
    assert orc.polyline_encode_value(-QM) == b"~~~~~~@"
    big = np.float32(QM)
    for prec in (0, 2, 5):
        sc = np.float32(10.0 ** prec)
        edge = big / sc                          # v * 10^p lands on (or within rounding of) 2^30
        H = np.array([[edge, -edge, 4.0 * edge, -4.0 * edge, 1e30, -1e30, np.inf, -np.inf,
                       np.nan, -0.0, 0.0, 3.4e38, -3.4e38]], dtype=np.float32)
        q = orc.polyline_quantise(H, prec)[0]
        assert list(q[2:8]) == [QM, -QM, QM, -QM, QM, -QM], (prec, q)
        assert abs(int(q[0])) <= QM and abs(int(q[1])) <= QM and q[0] > 0 > q[1]
        assert list(q[8:11]) == [0, 0, 0]                      # NaN, -0.0, 0.0
        assert list(q[11:]) == [QM, -QM]                       # the product overflows to +-inf in fp32
        codes, off = orc.polyline_encode_rows(H, prec)
        assert codes.min() >= 63 and codes.max() <= 126 and np.all(np.diff(off) <= 7 * H.shape[1])
        back = orc.polyline_decode_rows(codes, off, [0], H.shape[1], prec)[0]
        assert np.array_equal(back[2:8], np.float32(QM) / sc * np.array([1, -1, 1, -1, 1, -1], np.float32))
        assert np.all(back[8:11] == 0) and not np.signbit(back[8:11]).any()
        assert np.array_equal(orc.polyline_stored_value(H, prec)[0].view(np.uint32), back.view(np.uint32))
    # just inside the range nothing is clipped: the largest fp32 below 2^30 keeps its own code
    below = np.nextafter(big, np.float32(0))
    assert orc.polyline_quantise(np.array([[below, -below]], np.float32), 0).tolist() == [[int(below), -int(below)]]
    # fp64 arithmetic (the published examples' path) takes the same clauses
    assert orc.polyline_quantise(np.array([1e300, -1e300, np.nan]), 5, arith=np.float64).tolist() == [QM, -QM, 0]


# ------------------------------------------------ what the predictor is for
def test_trained_predictor_alleviates_staleness_on_drifting_embeddings():
    """The method's premise (Sec. "Embedding Predictor", the constraint of Eq. 8': the predicted
    embedding must be less stale than the cached one): on embeddings that keep moving from
    epoch to epoch, a predictor trained on the partition's own fresh embeddings (local rows,
    Eq. 11) must bring the HALO rows, which it never saw a target for, closer to their true
    next value than the newest cached rows are. Plain gradient steps, the oracle alone."""
    cfg = syn.get_config("tiny")
    g = syn.make_graph(cfg, np.random.default_rng(syn.substreams(0)["graph"]))
    v = orc.partition_view(g.N, g.rowptr, g.col, g.part, 0)
    n_l, n_bar = v["n_local"], v["n_local"] + v["n_halo"]
    d, d_s, tau = 16, 32, 2
    H = syn.drifting_history_f32(np.random.SeedSequence(3), n_bar, d, tau + 1)
    win, fresh = H[:tau], H[tau].astype(np.float64)
    p = syn.predictor_params_f32(np.random.SeedSequence(3), d, d_s)
    om = {k: p[k].astype(np.float64) for k in p}
    cached = orc.staleness(fresh[n_l:], win[-1][n_l:])
    before = orc.staleness(fresh[n_l:], orc.predict(v, om, win))
    losses = []
    for _ in range(20):
        loss, gr = orc.predictor_train_loss_and_grad(v, om, win, fresh[:n_l])
        losses.append(loss)
        for k in om:
            om[k] -= 2.0 * gr[k]
    after = orc.staleness(fresh[n_l:], orc.predict(v, om, win))
    assert losses[-1] < 0.1 * losses[0]
    assert after < 0.8 * cached and after < before       # delta(H_hat) < delta(H): Eq. 8'
    # the untrained predictor (random parameters) is no better than the cached rows
    assert before > 0.95 * cached
    # and without drift there is nothing to gain: the loss starts at the noise floor
    still = [H[0]] * tau
    l0, _ = orc.predictor_train_loss_and_grad(v, {k: p[k] * 0 for k in p}, still, H[0][:n_l])
    assert l0 == 0.0
