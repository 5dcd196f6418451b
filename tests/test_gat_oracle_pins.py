"""Pins of the GAT oracle against things that are not the oracle: a dense
masked-softmax formulation on torch's CPU softmax and autograd, closed forms,
invariants of the softmax, central finite differences, and the zero-staleness
invariant against an unpartitioned dense GAT. No HIP code is touched.
"""
import numpy as np
import pytest
import torch

import sat_synth as syn
from oracle import gat_oracle as gat
from oracle import sat_oracle as orc

SLOPE = 0.2


def small_graph(seed=5, N=90, n_parts=3):
    rng = np.random.default_rng(seed)
    return syn.sbm_graph(N, n_comm=n_parts, n_parts=n_parts, intra_deg=4.0, cross_deg=1.5, rng=rng)


def make_params(rng, dims, heads):
    ps = []
    for l in range(len(dims) - 1):
        K = heads[l]
        F = dims[l + 1] // K
        ps.append(dict(W=rng.normal(0, 0.4, (dims[l], K * F)),
                       a_dst=rng.normal(0, 0.5, (K, F)), a_src=rng.normal(0, 0.5, (K, F))))
    return ps


def dense_mask(view):
    """[n_local, n_bar] boolean: entry (i, j) of the partition view's CSR."""
    n_l, n_bar = view["n_local"], view["n_local"] + view["n_halo"]
    M = np.zeros((n_l, n_bar), dtype=bool)
    for i in range(n_l):
        M[i, view["col"][view["rowptr"][i]:view["rowptr"][i + 1]]] = True
    return M


def torch_gat_layer(mask, Hbar, W, a_dst, a_src, act, slope=SLOPE):
    """Dense formulation with library routines: masked scores, torch.softmax."""
    n_l = mask.shape[0]
    K, F = a_dst.shape
    Z = Hbar @ W
    Zh = Z.reshape(-1, K, F)
    el = (Zh * a_dst).sum(-1)[:n_l]                     # [n_l, K]
    er = (Zh * a_src).sum(-1)                           # [n_bar, K]
    e = torch.nn.functional.leaky_relu(el[:, None, :] + er[None, :, :], slope)   # [n_l, n_bar, K]
    e = e.masked_fill(~mask[:, :, None], float("-inf"))
    alpha = torch.softmax(e, dim=1)
    out = torch.einsum("ijk,jkf->ikf", alpha, Zh).reshape(n_l, K * F)
    return torch.relu(out) if act == 1 else out, alpha


def torch_gat_step(mask, X_local, X_halo, halo_hat, params, y, stale=None, halos=None):
    """stale: optional per-layer [n_local, d_l] added to the gradient that reaches the local rows
    of layer l's input - as a term <stale_l, h_l> of the objective, which has exactly that
    gradient. halos: optional list that receives the halo inputs (leaves with gradients)."""
    t = lambda a: torch.tensor(np.asarray(a, np.float64), dtype=torch.float64)
    leaves = []
    for p in params:
        leaves.append({k: t(v).requires_grad_(True) for k, v in p.items()})
    h = t(X_local)
    hs = [h]
    m = torch.tensor(mask)
    L = len(params)
    extra = 0.0
    for l in range(L):
        halo = t(X_halo if l == 0 else halo_hat[l]).requires_grad_(True)
        if halos is not None:
            halos.append(halo)
        if stale is not None and l >= 1:
            extra = extra + (t(stale[l]) * h).sum()
        hbar = torch.cat([h, halo], dim=0)
        h, _ = torch_gat_layer(m, hbar, leaves[l]["W"], leaves[l]["a_dst"], leaves[l]["a_src"],
                               1 if l < L - 1 else 0)
        h.retain_grad()
        hs.append(h)
    loss = torch.nn.functional.cross_entropy(h, torch.tensor(np.asarray(y, np.int64)))
    (loss + extra).backward()
    return loss.item(), leaves, hs


@pytest.fixture(scope="module")
def case():
    g = small_graph()
    view = orc.partition_view(g.N, g.rowptr, g.col, g.part, 1)
    rng = np.random.default_rng(11)
    dims, heads = [10, 12, 8, 5], [3, 2, 1]
    n_l, n_h = view["n_local"], view["n_halo"]
    X = rng.normal(0, 1, (g.N, dims[0]))
    params = make_params(rng, dims, heads)
    halo_hat = [None] + [rng.normal(0, 1, (n_h, dims[l])) for l in range(1, len(dims) - 1)]
    y = rng.integers(0, dims[-1], n_l)
    return dict(g=g, view=view, dims=dims, heads=heads, X_local=X[view["local_ids"]],
                X_halo=X[view["halo_ids"]], params=params, halo_hat=halo_hat, y=y, X=X)


def test_forward_and_all_gradients_match_dense_torch_autograd(case):
    c = case
    st = gat.gat_partition_step(c["view"], c["X_local"], c["X_halo"], c["halo_hat"], c["params"],
                                c["y"], SLOPE)
    loss, leaves, hs = torch_gat_step(dense_mask(c["view"]), c["X_local"], c["X_halo"],
                                      c["halo_hat"], c["params"], c["y"])
    assert abs(st["loss"] - loss) < 1e-12
    L = len(c["params"])
    for l in range(L):
        np.testing.assert_allclose(st["H"][l + 1], hs[l + 1].detach().numpy(), rtol=0, atol=1e-12)
        np.testing.assert_allclose(st["grads"][l]["dW"], leaves[l]["W"].grad.numpy(), rtol=0, atol=1e-12)
        np.testing.assert_allclose(st["grads"][l]["da_dst"], leaves[l]["a_dst"].grad.numpy(),
                                   rtol=0, atol=1e-12)
        np.testing.assert_allclose(st["grads"][l]["da_src"], leaves[l]["a_src"].grad.numpy(),
                                   rtol=0, atol=1e-12)
        if l >= 1:   # gradient reaching the local rows of the layer's input
            np.testing.assert_allclose(st["dH_in"][l], hs[l].grad.numpy(), rtol=0, atol=1e-12)


def test_halo_gradient_and_stale_term_match_dense_torch_autograd(case):
    """What the step returns for its halo inputs is the objective's gradient with respect to
    them, and a stale term added to the gradient at the local rows of a layer's input reaches
    every quantity below it as an extra term <stale_l, h_l> of the objective would."""
    c = case
    L = len(c["params"])
    n_l = c["view"]["n_local"]
    rng = np.random.default_rng(5)
    stale = [None] + [rng.normal(0, 0.3, (n_l, c["dims"][l])) for l in range(1, L)]
    st = gat.gat_partition_step(c["view"], c["X_local"], c["X_halo"], c["halo_hat"], c["params"],
                                c["y"], SLOPE, stale_grad=stale)
    halos = []
    loss, leaves, hs = torch_gat_step(dense_mask(c["view"]), c["X_local"], c["X_halo"],
                                      c["halo_hat"], c["params"], c["y"], stale=stale, halos=halos)
    assert abs(st["loss"] - loss) < 1e-12
    for l in range(L):
        np.testing.assert_allclose(st["grads"][l]["dW"], leaves[l]["W"].grad.numpy(), rtol=0, atol=1e-12)
        np.testing.assert_allclose(st["grads"][l]["da_src"], leaves[l]["a_src"].grad.numpy(),
                                   rtol=0, atol=1e-12)
        if l >= 1:
            # (autograd's h.grad holds the stale term as well: it is part of the objective there)
            np.testing.assert_allclose(st["dH_in"][l], hs[l].grad.numpy(), rtol=0, atol=1e-12)
            np.testing.assert_allclose(st["dH_halo"][l], halos[l].grad.numpy(), rtol=0, atol=1e-12)
    # without the stale term the halo gradient is unchanged at the last hidden layer only
    st0 = gat.gat_partition_step(c["view"], c["X_local"], c["X_halo"], c["halo_hat"], c["params"],
                                 c["y"], SLOPE)
    np.testing.assert_allclose(st0["dH_halo"][L - 1], st["dH_halo"][L - 1], rtol=0, atol=0)
    assert np.abs(st0["dH_halo"][1] - st["dH_halo"][1]).max() > 1e-6


def test_zero_attention_vectors_give_the_neighbourhood_mean(case):
    c = case
    view = c["view"]
    rng = np.random.default_rng(2)
    n_bar = view["n_local"] + view["n_halo"]
    Z = rng.normal(0, 1, (n_bar, 12))
    el = np.zeros((view["n_local"], 3))
    er = np.zeros((n_bar, 3))
    out = gat.gat_aggregate_fwd(view, Z, el, er, SLOPE)
    M = dense_mask(view).astype(np.float64)
    mean = (M / M.sum(axis=1, keepdims=True)) @ Z
    np.testing.assert_allclose(out, mean, rtol=0, atol=1e-13)


def test_alpha_rows_sum_to_one_and_slope_one_ignores_el(case):
    view = case["view"]
    rng = np.random.default_rng(4)
    n_l, n_bar = view["n_local"], view["n_local"] + view["n_halo"]
    el = rng.normal(0, 2, (n_l, 2))
    er = rng.normal(0, 2, (n_bar, 2))
    for i in (0, 3, n_l - 1):
        cols, s, a = gat.gat_row_attention(view, i, el, er, SLOPE)
        np.testing.assert_allclose(a.sum(axis=0), 1.0, atol=1e-14)
        assert a.shape == (len(cols), 2) and np.all(a > 0)
        # slope 1: LeakyReLU is the identity and el_i cancels in the softmax
        _, _, a1 = gat.gat_row_attention(view, i, el, er, 1.0)
        _, _, a2 = gat.gat_row_attention(view, i, el + 7.5, er, 1.0)
        ref = np.exp(er[cols]) / np.exp(er[cols]).sum(axis=0, keepdims=True)
        np.testing.assert_allclose(a1, ref, atol=1e-14)
        np.testing.assert_allclose(a2, ref, atol=1e-13)


def test_single_neighbour_row_copies_its_source():
    # a path 0 - 1 with node 0 alone in the partition: row 0 = {0, 1}; with a huge score
    # for node 1 the output row is Z_1 to rounding, with equal scores the mean of both
    view = dict(n_local=1, n_halo=1, rowptr=np.array([0, 2]), col=np.array([0, 1], np.int32))
    Z = np.array([[1.0, 2.0], [5.0, -3.0]])
    out = gat.gat_aggregate_fwd(view, Z, np.zeros((1, 1)), np.array([[0.0], [50.0]]), SLOPE)
    np.testing.assert_allclose(out[0], Z[1], atol=1e-12)
    out = gat.gat_aggregate_fwd(view, Z, np.zeros((1, 1)), np.zeros((2, 1)), SLOPE)
    np.testing.assert_allclose(out[0], Z.mean(axis=0), atol=1e-15)


def test_scores_against_explicit_concatenation(case):
    # the published form: e_ij = LeakyReLU(a^T [z_i || z_j]) with a = [a_dst ; a_src]
    rng = np.random.default_rng(8)
    K, F = 2, 3
    Z = rng.normal(0, 1, (6, K * F))
    a_dst, a_src = rng.normal(0, 1, (K, F)), rng.normal(0, 1, (K, F))
    el, er = gat.gat_scores(Z, a_dst, a_src)
    for k in range(K):
        a = np.concatenate([a_dst[k], a_src[k]])
        for i in range(6):
            for j in range(6):
                cat = np.concatenate([Z[i, k * F:(k + 1) * F], Z[j, k * F:(k + 1) * F]])
                assert abs(a @ cat - (el[i, k] + er[j, k])) < 1e-13


def test_loss_gradient_by_central_differences(case):
    c = case
    base = gat.gat_partition_step(c["view"], c["X_local"], c["X_halo"], c["halo_hat"], c["params"],
                                  c["y"], SLOPE)
    rng = np.random.default_rng(17)
    h = 1e-6
    for l in range(len(c["params"])):
        for key, gname in (("W", "dW"), ("a_dst", "da_dst"), ("a_src", "da_src")):
            arr = c["params"][l][key]
            for _ in range(3):
                idx = tuple(rng.integers(0, s) for s in arr.shape)
                keep = arr[idx]
                arr[idx] = keep + h
                lp = gat.gat_partition_step(c["view"], c["X_local"], c["X_halo"], c["halo_hat"],
                                            c["params"], c["y"], SLOPE)["loss"]
                arr[idx] = keep - h
                lm = gat.gat_partition_step(c["view"], c["X_local"], c["X_halo"], c["halo_hat"],
                                            c["params"], c["y"], SLOPE)["loss"]
                arr[idx] = keep
                fd = (lp - lm) / (2 * h)
                assert abs(fd - base["grads"][l][gname][idx]) < 1e-7 + 1e-5 * abs(fd)


def test_zero_staleness_equals_unpartitioned_dense_gat(case):
    """Feeding the exact embeddings of the halo nodes reproduces the rows of a GAT
    computed on the whole graph (dense, library softmax)."""
    c = case
    g = c["g"]
    A = np.zeros((g.N, g.N), dtype=bool)
    for i in range(g.N):
        A[i, g.col[g.rowptr[i]:g.rowptr[i + 1]]] = True
        A[i, i] = True
    t = lambda a: torch.tensor(np.asarray(a, np.float64), dtype=torch.float64)
    H = [t(c["X"])]
    L = len(c["params"])
    for l in range(L):
        p = c["params"][l]
        h, _ = torch_gat_layer(torch.tensor(A), H[l], t(p["W"]), t(p["a_dst"]), t(p["a_src"]),
                               1 if l < L - 1 else 0)
        H.append(h)
    view = c["view"]
    exact = [None] + [H[l].numpy()[view["halo_ids"]] for l in range(1, L)]
    st = gat.gat_partition_step(view, c["X_local"], c["X_halo"], exact, c["params"], c["y"], SLOPE)
    for l in range(1, L + 1):
        np.testing.assert_allclose(st["H"][l], H[l].numpy()[view["local_ids"]], rtol=0, atol=1e-12)


def test_store_hook_rounds_what_is_kept(case):
    c = case
    st = gat.gat_partition_step(c["view"], c["X_local"], c["X_halo"], c["halo_hat"], c["params"],
                                c["y"], SLOPE, store=orc.round_bf16)
    for l, cc in enumerate(st["caches"]):
        for k in ("Z", "H"):
            np.testing.assert_array_equal(cc[k], orc.round_bf16(cc[k]))
        np.testing.assert_array_equal(st["grads"][l]["dZ"], orc.round_bf16(st["grads"][l]["dZ"]))
