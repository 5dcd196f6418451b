"""CPU oracle for one partition's SAT step with a GAT backbone. TEST INFRASTRUCTURE ONLY.

The paper evaluates SAT on GCN and GAT backbones (experiment tables, rows "GAT")
and states the layer generically (Eq. 1: an aggregation function over the
neighbourhood followed by an update; Eq. 2 / Eq. 5: the same with the
neighbourhood split into in-subgraph and out-of-subgraph nodes, the latter fed
from predicted embeddings). It does not restate the attention layer, so this file
follows the published definition of the graph attention layer (Velickovic et
al., "Graph Attention Networks", Eq. 1-4), written out as loops over rows in
fp64, sharing no code with the HIP library. Only the tests, the smoke check and
the benchmark's cpu_baseline leg may import it.

One layer on partition m, with Hbar = [H_in ; H_out_hat] (local rows, then the halo
rows, which are constants of the step):
    Z      = Hbar W                                   all local + halo rows
    el_i   = <a_dst^k, Z_i^k>  (local i),  er_j = <a_src^k, Z_j^k>  (all j), per head k
    e_ij   = LeakyReLU(el_i + er_j; slope)            j in N(i) u {i}, i local
    alpha  = softmax over j of e_ij                    per row i and head k
    OUT_i  = sum_j alpha_ij^k Z_j^k                    heads concatenated
    H'     = relu(OUT) on hidden layers, OUT on the last
The neighbourhood of a local node i is row i of the partition view's CSR
[P_in | P_out] (self-loop included); its stored values A_hat are not used.
A row without entries cannot come from a partition view (the self-loop is always
there); for hand-made views it is defined as OUT_i = 0, contributing nothing to
any gradient (an empty sum).

Readings (the paper is silent on all of them): heads are concatenated on every
layer (a last layer with one head is the usual classifier); slope 0.2; no bias, no
dropout; the hidden activation is the ReLU of the GCN path; Z of the halo rows
depends on W, so dW sums over local and halo rows, while no gradient is returned
for the halo embeddings themselves (they are constants, as in the GCN path).

Pins (tests/test_gat_oracle_pins.py): a dense masked-softmax formulation with
torch's softmax and autograd on the CPU (forward values and every gradient),
the closed form for zero attention vectors (uniform attention = neighbourhood
mean), rows of alpha summing to one, slope 1 making alpha independent of el,
central finite differences of the loss, and the zero-staleness invariant against
an unpartitioned dense GAT.
"""
import numpy as np


def leaky_relu(x, slope):
    return np.where(x > 0, x, slope * x)


def gat_scores(Z, a_dst, a_src):
    """el, er [n, K]: per head the inner product of the head's slice of Z with the
    destination / source half of the attention vector. a_dst, a_src: [K, F]."""
    a_dst = np.asarray(a_dst, np.float64)
    a_src = np.asarray(a_src, np.float64)
    K, F = a_dst.shape
    Zh = np.asarray(Z, np.float64).reshape(Z.shape[0], K, F)
    return np.einsum("nkf,kf->nk", Zh, a_dst), np.einsum("nkf,kf->nk", Zh, a_src)


def gat_row_attention(view, i, el, er, slope):
    """(cols, s, alpha) of local row i: s[j, k] = el[i, k] + er[col_j, k],
    alpha[j, k] = softmax over the row's entries of LeakyReLU(s)."""
    rowptr, col = view["rowptr"], view["col"]
    cols = col[rowptr[i]:rowptr[i + 1]]
    s = el[i][None, :] + er[cols]
    e = leaky_relu(s, slope)
    p = np.exp(e - e.max(axis=0, keepdims=True))
    return cols, s, p / p.sum(axis=0, keepdims=True)


def gat_aggregate_fwd(view, Z, el, er, slope, rows=None):
    """OUT[i] = sum_j alpha_ij Z_j per head, for the local rows (or the listed ones)."""
    K = el.shape[1]
    Z = np.asarray(Z, np.float64)
    F = Z.shape[1] // K
    rows = range(view["n_local"]) if rows is None else rows
    out = np.zeros((len(rows), K * F), dtype=np.float64)
    for r, i in enumerate(rows):
        if view["rowptr"][i + 1] == view["rowptr"][i]:
            continue                          # empty sum
        cols, _, alpha = gat_row_attention(view, i, el, er, slope)
        out[r] = np.einsum("jk,jkf->kf", alpha, Z[cols].reshape(-1, K, F)).reshape(-1)
    return out


def gat_aggregate_bwd(view, Z, el, er, slope, dOUT, rows=None):
    """Backward of gat_aggregate_fwd for given el, er (treated as inputs):
    returns (dZ_agg [n_bar, d], d_el [n_local, K], d_er [n_bar, K]).
    rows: only these local rows contribute (all of them by default).

    With dalpha_ij = <dOUT_i, Z_j> per head: de_ij = alpha_ij (dalpha_ij - sum_k
    alpha_ik dalpha_ik) (softmax), ds_ij = de_ij LeakyReLU'(s_ij), d_el_i = sum_j
    ds_ij, d_er_j = sum_i ds_ij, dZ_j += sum_i alpha_ij dOUT_i.
    """
    n_local, n_bar = view["n_local"], view["n_local"] + view["n_halo"]
    K = el.shape[1]
    Z = np.asarray(Z, np.float64)
    F = Z.shape[1] // K
    G = np.asarray(dOUT, np.float64).reshape(n_local, K, F)
    dZ = np.zeros((n_bar, K, F), dtype=np.float64)
    d_el = np.zeros((n_local, K), dtype=np.float64)
    d_er = np.zeros((n_bar, K), dtype=np.float64)
    for i in (range(n_local) if rows is None else rows):
        if view["rowptr"][i + 1] == view["rowptr"][i]:
            continue                          # empty sum
        cols, s, alpha = gat_row_attention(view, i, el, er, slope)
        zc = Z[cols].reshape(-1, K, F)
        dalpha = np.einsum("kf,jkf->jk", G[i], zc)
        de = alpha * (dalpha - (alpha * dalpha).sum(axis=0, keepdims=True))
        ds = de * np.where(s > 0, 1.0, slope)
        d_el[i] = ds.sum(axis=0)
        d_er[cols] += ds                      # column ids are distinct inside a row
        dZ[cols] += alpha[:, :, None] * G[i][None, :, :]
    return dZ.reshape(n_bar, K * F), d_el, d_er


def gat_layer_fwd(view, Hbar, W, a_dst, a_src, slope, act, store=None):
    """One layer forward; returns the tensors the backward needs."""
    if store is None:
        store = lambda t: t
    n_local = view["n_local"]
    Hbar = np.asarray(Hbar, np.float64)
    Z = store(Hbar @ np.asarray(W, np.float64))
    el, er = gat_scores(Z, a_dst, a_src)
    OUT = gat_aggregate_fwd(view, Z, el[:n_local], er, slope)
    H = store(np.maximum(OUT, 0.0) if act == 1 else OUT)
    return dict(Hbar=Hbar, Z=Z, el=el[:n_local], er=er, OUT=OUT, H=H)


def gat_layer_bwd(view, c, W, a_dst, a_src, slope, act, dH, store=None):
    """Backward of one layer from dH = d loss / d H' (local rows).
    Returns dict(dW, da_dst, da_src, dHbar [n_bar, d_in] (rows of the halo nodes
    included: the step drops them), dZ)."""
    if store is None:
        store = lambda t: t
    a_dst = np.asarray(a_dst, np.float64)
    a_src = np.asarray(a_src, np.float64)
    K, F = a_dst.shape
    n_local = view["n_local"]
    dOUT = np.asarray(dH, np.float64)
    if act == 1:
        dOUT = dOUT * (c["H"] > 0)
    dOUT = store(dOUT)
    dZ, d_el, d_er = gat_aggregate_bwd(view, c["Z"], c["el"], c["er"], slope, dOUT)
    n_bar = dZ.shape[0]
    dZ = dZ.reshape(n_bar, K, F)
    dZ[:n_local] += d_el[:, :, None] * a_dst[None, :, :]
    dZ += d_er[:, :, None] * a_src[None, :, :]
    Zh = c["Z"].reshape(n_bar, K, F)
    da_dst = np.einsum("nk,nkf->kf", d_el, Zh[:n_local])
    da_src = np.einsum("nk,nkf->kf", d_er, Zh)
    dZ = store(dZ.reshape(n_bar, K * F))
    dW = c["Hbar"].T @ dZ
    dHbar = dZ @ np.asarray(W, np.float64).T
    return dict(dW=dW, da_dst=da_dst, da_src=da_src, dHbar=dHbar, dZ=dZ, d_el=d_el, d_er=d_er,
                dOUT=dOUT)


def gat_partition_step(view, X_local, X_halo, halo_hat, params, y, slope=0.2, store=None,
                       stale_grad=None):
    """Forward and backward of an L-layer GAT on one partition (Eq. 5 with the
    attention layer as f; Eq. 4 as the loss).

    params[l] = dict(W [d_l, K_l F_l], a_dst [K_l, F_l], a_src [K_l, F_l]).
    halo_hat[l] for l = 1..L-1: halo rows fed to layer l (predicted or plain
    historical embeddings); layer 0 uses the true features X_halo.
    store: applied to every tensor kept in memory between calls (Z, H, the loss
    gradient, the masked gradient, dZ, dH_in); identity for fp32 storage.
    stale_grad: None, or stale_grad[l] for l = 1..L-1 = [n_local, d_l]: what the other
    partitions computed, one step ago, for the gradient reaching this partition's nodes
    through THEIR halo copies (the second term of the appendix's SAT backward, G_H = (local
    term) + P_out^T D~ W^T, carried over to this layer type: whatever the layer is, the term
    is the other partitions' gradient with respect to their halo inputs); added to the local
    term before it is kept and passed down.
    Returns dict with per-layer caches, loss, and per layer dW, da_dst, da_src,
    dH_in (None for layer 0) and dH_halo (this partition's gradient with respect to ITS halo
    inputs of layer l, [n_halo, d_l]: what it would send to their owners; None for layer 0).
    """
    from .sat_oracle import loss_and_grad
    if store is None:
        store = lambda t: t
    n_local = view["n_local"]
    L = len(params)
    H = [np.asarray(X_local, np.float64)]
    caches = []
    for l in range(L):
        halo = X_halo if l == 0 else halo_hat[l]
        Hbar = np.concatenate([H[l], np.asarray(halo, np.float64)], axis=0)
        p = params[l]
        c = gat_layer_fwd(view, Hbar, p["W"], p["a_dst"], p["a_src"], slope,
                          1 if l < L - 1 else 0, store)
        caches.append(c)
        H.append(c["H"])
    loss, g = loss_and_grad(H[L], y)
    g = store(g)
    grads = [None] * L
    dH_in = [None] * L
    dH_halo = [None] * L
    for l in range(L - 1, -1, -1):
        p = params[l]
        b = gat_layer_bwd(view, caches[l], p["W"], p["a_dst"], p["a_src"], slope,
                          1 if l < L - 1 else 0, g, store)
        grads[l] = b
        if l >= 1:
            g = b["dHbar"][:n_local]
            if stale_grad is not None:
                g = store(g) + np.asarray(stale_grad[l], np.float64)
            g = store(g)
            dH_in[l] = g
            dH_halo[l] = store(b["dHbar"][n_local:])
    return dict(caches=caches, H=H, loss=loss, grads=grads, dH_in=dH_in, dH_halo=dH_halo)
