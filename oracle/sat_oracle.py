"""CPU oracle for one partition's SAT GCN layer step. TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 restatement of what the hot path computes, written from
the paper's definitions and sharing no code with the HIP library. Only the
tests, the smoke check and the benchmark's cpu_baseline leg may import it;
the product path never does.

Where the paper defines the quantity exactly (propagation matrix, layer
forward, backward, pull / push) the function below is that definition written
out as loops over rows. The embedding predictor is only named by the paper
(an RNN-GNN built from an LSTM and a GCN, with a window of tau past epochs);
its step list is fixed in `predict` and every choice the paper leaves open is
listed there.

Conventions
-----------
* Inputs arrive in the storage precision (fp32 arrays, int32 / int64 index
  arrays); every product and sum is carried out in fp64; results are fp64.
* Index results (halo list, relabelled CSR, transposed halo block) have one
  canonical form and are meant to be compared bit for bit.
* `view` is the dict returned by `partition_view`.

Pins (see tests/test_oracle_pins.py): dense brute force of A_hat on tiny
graphs, the closed form A_hat * sqrt(d) = sqrt(d), the ring graph's 3-point
mean, scipy's CSR product, the zero-staleness invariant against the
unpartitioned GCN, central finite differences of the loss, torch.nn.LSTM on
the CPU, and the tau = 1 closed form of the LSTM cell.

Parity unpinned: the predictor's architecture constants (hidden size d_s,
window tau, residual output, one GCN hop restricted to local-halo edges) are
readings of a description the paper gives only in words; no printed value
exists to pin them to. Their arithmetic is pinned (LSTM vs library routine,
hop vs dense brute force), the choice of architecture is not.
"""
import numpy as np


# --------------------------------------------------------------------------
# Propagation matrix (appendix "Preliminaries": P is the GCN propagation
# matrix of Kipf & Welling): A_tilde = A + I, d_tilde = 1 + deg,
# A_hat[i, j] = A_tilde[i, j] / sqrt(d_tilde[i] * d_tilde[j]).
# --------------------------------------------------------------------------
def inv_sqrt_degree(deg):
    """fp32( 1 / sqrt(1 + deg) ) per node; deg counts neighbours, no self-loop.

    The division and square root are taken in fp64 and rounded once to fp32;
    an entry of A_hat is then ONE fp32 product of two such factors. This fixes
    the stored values bit for bit.
    """
    d_tilde = 1.0 + np.asarray(deg, dtype=np.float64)
    return (1.0 / np.sqrt(d_tilde)).astype(np.float32)


def a_hat_value(isd_i, isd_j):
    """Stored fp32 value of A_hat[i, j] from the two fp32 factors."""
    return np.float32(isd_i) * np.float32(isd_j)


# --------------------------------------------------------------------------
# Partition view (Eq. 2: in-subgraph vs out-of-subgraph neighbours; appendix:
# P = P_in + P_out; Sec. "Temporal graphs": partition plus 1-hop neighbourhood)
# --------------------------------------------------------------------------
def partition_view(N, g_rowptr, g_col, part, m, g_deg=None):
    """Local view of partition m of a simple undirected graph.

    V_m = nodes with part == m in ascending global id; local id = rank.
    Halo = nodes outside V_m adjacent to some node of V_m, ascending global
    id; relabelled n_local + rank. Rows of the local CSR are the local nodes;
    a row holds the self-loop and every neighbour, sorted by relabelled id,
    so all local columns come before all halo columns; split[i] is the offset
    of the first halo column. Values are A_hat entries with GLOBAL degrees
    (otherwise P_in + P_out would not add up to P). The halo block is also
    given transposed (per halo node: its local neighbours ascending), with
    the halo node's own diagonal entry A_hat[u, u] in h_self.

    g_deg (optional) overrides the neighbour count of every node; by default
    it is the row length of the global CSR.
    """
    part = np.asarray(part)
    if g_deg is None:
        g_deg = np.diff(g_rowptr)
    isd = inv_sqrt_degree(g_deg)
    local_ids = np.flatnonzero(part == m).astype(np.int32)
    n_local = local_ids.size

    halo_mark = np.zeros(N, dtype=bool)
    for g in local_ids:
        nb = g_col[g_rowptr[g]:g_rowptr[g + 1]]
        halo_mark[nb[part[nb] != m]] = True
    halo_ids = np.flatnonzero(halo_mark).astype(np.int32)
    n_halo = halo_ids.size

    relabel = np.full(N, -1, dtype=np.int64)
    relabel[local_ids] = np.arange(n_local)
    relabel[halo_ids] = n_local + np.arange(n_halo)

    rowptr = np.zeros(n_local + 1, dtype=np.int64)
    split = np.zeros(n_local, dtype=np.int64)
    cols, vals = [], []
    for i, g in enumerate(local_ids):
        nb = np.concatenate([g_col[g_rowptr[g]:g_rowptr[g + 1]], [g]])
        c = relabel[nb]
        order = np.argsort(c, kind="stable")
        c = c[order]
        v = isd[g] * isd[nb[order]]          # fp32 * fp32 -> fp32
        rowptr[i + 1] = rowptr[i] + c.size
        split[i] = rowptr[i] + np.searchsorted(c, n_local)
        cols.append(c.astype(np.int32))
        vals.append(v.astype(np.float32))
    col = np.concatenate(cols) if cols else np.zeros(0, np.int32)
    val = np.concatenate(vals) if vals else np.zeros(0, np.float32)

    # transposed halo block: entries (row i, halo column c) grouped by c,
    # rows ascending inside a group
    hr, hc, hv = [], [], []
    for i in range(n_local):
        s, e = split[i], rowptr[i + 1]
        hr.append(np.full(e - s, i, dtype=np.int32))
        hc.append(col[s:e] - n_local)
        hv.append(val[s:e])
    hr = np.concatenate(hr) if hr else np.zeros(0, np.int32)
    hc = np.concatenate(hc) if hc else np.zeros(0, np.int32)
    hv = np.concatenate(hv) if hv else np.zeros(0, np.float32)
    order = np.lexsort((hr, hc))             # by halo column, then row
    h_row = hr[order].astype(np.int32)
    h_val = hv[order].astype(np.float32)
    h_colptr = np.zeros(n_halo + 1, dtype=np.int64)
    np.cumsum(np.bincount(hc, minlength=n_halo), out=h_colptr[1:])
    h_self = (isd[halo_ids] * isd[halo_ids]).astype(np.float32)

    return dict(n_local=n_local, n_halo=n_halo, nnz=int(rowptr[-1]),
                nnz_halo=int(h_colptr[-1]), local_ids=local_ids,
                halo_ids=halo_ids, rowptr=rowptr, split=split, col=col,
                val=val, h_colptr=h_colptr, h_row=h_row, h_val=h_val,
                h_self=h_self)


def partition_view_sample(N, g_rowptr, g_col, part, m, rows, halo_sample, g_deg=None):
    """The parts of partition_view that a graph too large for its per-node
    loops still allows: the complete id lists and row offsets (array
    operations over the partition's entries), and for the sampled local rows
    `rows` and sampled halo nodes `halo_sample` (ranks) their entries exactly
    as partition_view lays them out. Same definitions as partition_view; the
    two are compared on small graphs by the tests.

    Returns dict(local_ids, halo_ids, rowptr, n_local, n_halo, nnz, nnz_halo,
    h_colptr, h_self, row_entries = {i: (col, val, split_offset)},
    halo_entries = {u: (h_row, h_val)}).
    """
    part = np.asarray(part)
    if g_deg is None:
        g_deg = np.diff(g_rowptr)
    isd = inv_sqrt_degree(g_deg)
    local_ids = np.flatnonzero(part == m).astype(np.int32)
    n_local = local_ids.size
    lens = (g_rowptr[1:] - g_rowptr[:-1])[local_ids]
    # every entry of the partition's rows, row by row (runs of consecutive ids are one slice)
    brk = np.flatnonzero(np.diff(local_ids) != 1) + 1
    starts = np.concatenate([[0], brk])
    ends = np.concatenate([brk, [n_local]])
    ent = np.concatenate([g_col[g_rowptr[local_ids[a]]:g_rowptr[local_ids[b - 1] + 1]]
                          for a, b in zip(starts, ends)]) if n_local else np.zeros(0, np.int32)
    outside = ent[part[ent] != m]
    halo_ids = np.unique(outside).astype(np.int32)
    n_halo = halo_ids.size
    rowptr = np.zeros(n_local + 1, dtype=np.int64)
    np.cumsum(lens + 1, out=rowptr[1:])                      # + the self-loop
    h_colptr = np.zeros(n_halo + 1, dtype=np.int64)
    np.cumsum(np.bincount(np.searchsorted(halo_ids, outside), minlength=n_halo), out=h_colptr[1:])
    h_self = (isd[halo_ids] * isd[halo_ids]).astype(np.float32)

    def relabel(ids):
        ids = np.asarray(ids, dtype=np.int64)
        loc = part[ids] == m
        out = np.empty(ids.shape, dtype=np.int64)
        out[loc] = np.searchsorted(local_ids, ids[loc])
        out[~loc] = n_local + np.searchsorted(halo_ids, ids[~loc])
        return out

    row_entries = {}
    for i in rows:
        g = int(local_ids[i])
        nb = np.concatenate([g_col[g_rowptr[g]:g_rowptr[g + 1]], [g]])
        c = relabel(nb)
        order = np.argsort(c, kind="stable")
        c = c[order]
        v = (isd[g] * isd[nb[order]]).astype(np.float32)
        row_entries[int(i)] = (c.astype(np.int32), v, int(np.searchsorted(c, n_local)))
    halo_entries = {}
    if len(halo_sample):
        ent_row = np.repeat(np.arange(n_local, dtype=np.int64), lens)   # local row of every entry
        for u in halo_sample:
            gid = int(halo_ids[u])
            r = np.sort(ent_row[ent == gid])
            v = (isd[local_ids[r]] * isd[gid]).astype(np.float32)
            halo_entries[int(u)] = (r.astype(np.int32), v)
    return dict(n_local=n_local, n_halo=n_halo, nnz=int(rowptr[-1]), nnz_halo=int(h_colptr[-1]),
                local_ids=local_ids, halo_ids=halo_ids, rowptr=rowptr, h_colptr=h_colptr,
                h_self=h_self, row_entries=row_entries, halo_entries=halo_entries)


# --------------------------------------------------------------------------
# bf16 storage mode: tensors kept in HBM as bfloat16 are rounded when they are
# stored; all arithmetic stays fp64 here (fp32 on the GPU).
# --------------------------------------------------------------------------
def round_bf16(a):
    """Nearest bfloat16 value (ties to even) of every element, returned as fp64."""
    u = np.asarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = ((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)) << np.uint64(16)
    return r.astype(np.uint32).view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------
# Pull / push (Alg. 1: "Pull H_out", "Push computed embeddings")
# --------------------------------------------------------------------------
def history_gather(table, ids):
    """out[k, :] = table[ids[k], :]; a pure copy (same dtype as the table)."""
    return np.array(table[np.asarray(ids, dtype=np.int64)], copy=True)


def history_push(table, ids, H):
    """table[ids[k], :d] = H[k, :d] in place; other rows and columns untouched."""
    d = H.shape[1]
    for k, r in enumerate(np.asarray(ids, dtype=np.int64)):
        table[r, :d] = H[k]
    return table


# --------------------------------------------------------------------------
# Aggregation (appendix, SAT forward: P_in H_in + P_out H_out_hat) and its
# transpose (appendix, SAT backward: P_in^T D W^T; P_out^T ... on request)
# --------------------------------------------------------------------------
def spmm_fwd(view, Hbar):
    """AGG = [P_in | P_out] Hbar; Hbar stacks local rows then halo rows."""
    n_local = view["n_local"]
    rowptr, col, val = view["rowptr"], view["col"], view["val"]
    Hb = np.asarray(Hbar, dtype=np.float64)
    out = np.zeros((n_local, Hb.shape[1]), dtype=np.float64)
    for i in range(n_local):
        s, e = rowptr[i], rowptr[i + 1]
        out[i] = val[s:e].astype(np.float64) @ Hb[col[s:e]]
    return out


def spmm_fwd_rows(view, Hbar, rows):
    """Rows `rows` of spmm_fwd (rows are independent of one another)."""
    rowptr, col, val = view["rowptr"], view["col"], view["val"]
    out = np.zeros((len(rows), Hbar.shape[1]), dtype=np.float64)
    for k, i in enumerate(rows):
        s, e = rowptr[i], rowptr[i + 1]
        out[k] = val[s:e].astype(np.float64) @ Hbar[col[s:e]].astype(np.float64)
    return out


def spmm_bwd(view, dAGG, want_halo=False):
    """dH_local = P_in^T dAGG (and dH_halo = P_out^T dAGG when asked).

    Written as the transpose scatter of the forward loop, so it does not rely
    on P_in being symmetric.
    """
    n_local, n_halo = view["n_local"], view["n_halo"]
    rowptr, split, col, val = view["rowptr"], view["split"], view["col"], view["val"]
    G = np.asarray(dAGG, dtype=np.float64)
    d = G.shape[1]
    dH = np.zeros((n_local + n_halo, d), dtype=np.float64)
    for i in range(n_local):
        s, e = rowptr[i], (rowptr[i + 1] if want_halo else split[i])
        # column ids are distinct inside a row, so fancy += is a true scatter
        dH[col[s:e]] += val[s:e].astype(np.float64)[:, None] * G[i][None, :]
    if want_halo:
        return dH[:n_local], dH[n_local:]
    return dH[:n_local], None


def spmm_bwd_rows(view, dAGG, rows):
    """Rows `rows` of P_in^T dAGG via the symmetry P_in^T = P_in (A_hat is
    symmetric and local ids index rows and columns alike)."""
    rowptr, split, col, val = view["rowptr"], view["split"], view["col"], view["val"]
    out = np.zeros((len(rows), dAGG.shape[1]), dtype=np.float64)
    for k, i in enumerate(rows):
        s, e = rowptr[i], split[i]
        out[k] = val[s:e].astype(np.float64) @ dAGG[col[s:e]].astype(np.float64)
    return out


# --------------------------------------------------------------------------
# Feature transform (appendix: Z = (P H) W, H' = sigma(Z)) and its backward
# (G_W = (P H)^T D, D = G_H' o sigma'(Z), gradient to the aggregate D W^T)
# --------------------------------------------------------------------------
def dense_fwd(AGG, W, act):
    """Z = AGG W; H = relu(Z) if act == 1 else Z. No bias, no dropout."""
    Z = np.asarray(AGG, dtype=np.float64) @ np.asarray(W, dtype=np.float64)
    H = np.maximum(Z, 0.0) if act == 1 else Z.copy()
    return Z, H


def dense_bwd(dH, Z, AGG, W, act):
    """dZ = dH o relu'(Z) (relu'(z) = 1 for z > 0, else 0; identity if act == 0);
    dW = AGG^T dZ; dAGG = dZ W^T."""
    dZ = np.asarray(dH, dtype=np.float64)
    if act == 1:
        dZ = dZ * (np.asarray(Z) > 0)
    dW = np.asarray(AGG, dtype=np.float64).T @ dZ
    dAGG = dZ @ np.asarray(W, dtype=np.float64).T
    return dW, dAGG, dZ


# --------------------------------------------------------------------------
# Local loss (Eq. 4 with cross-entropy as Loss)
# --------------------------------------------------------------------------
def loss_and_grad(HL, y):
    """Mean softmax cross-entropy over the local nodes and d loss / d HL."""
    HL = np.asarray(HL, dtype=np.float64)
    n = HL.shape[0]
    z = HL - HL.max(axis=1, keepdims=True)
    logp = z - np.log(np.exp(z).sum(axis=1, keepdims=True))
    loss = -logp[np.arange(n), y].mean()
    g = np.exp(logp)
    g[np.arange(n), y] -= 1.0
    return loss, g / n


# --------------------------------------------------------------------------
# Embedding predictor g_omega (Sec. "Embedding Predictor": RNN-GNN = LSTM over
# a window of tau past epochs, then a GCN over the partition-plus-halo graph;
# its output corrects the newest cached embedding of the halo nodes)
# --------------------------------------------------------------------------
def _sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def lstm_last_hidden(slots, Wx, Wh, b):
    """S = h_tau of a one-layer LSTM run over slots[0..tau-1] (oldest first).

    Per node (row), weights shared by all nodes, h_0 = c_0 = 0:
      [i; f; g; o] = Wx x_s + Wh h_{s-1} + b      (blocks of d_s rows, order i, f, g, o)
      c_s = sigmoid(f) o c_{s-1} + sigmoid(i) o tanh(g)
      h_s = sigmoid(o) o tanh(c_s)
    """
    Wx = np.asarray(Wx, np.float64)
    Wh = np.asarray(Wh, np.float64)
    b = np.asarray(b, np.float64)
    d_s = Wh.shape[1]
    n = slots[0].shape[0]
    h = np.zeros((n, d_s))
    c = np.zeros((n, d_s))
    for x in slots:
        pre = np.asarray(x, np.float64) @ Wx.T + h @ Wh.T + b
        i = _sigmoid(pre[:, 0 * d_s:1 * d_s])
        f = _sigmoid(pre[:, 1 * d_s:2 * d_s])
        g = np.tanh(pre[:, 2 * d_s:3 * d_s])
        o = _sigmoid(pre[:, 3 * d_s:4 * d_s])
        c = f * c + i * g
        h = o * np.tanh(c)
    return h


def predictor_hop(view, S, Wg):
    """Delta[u] = ( A_hat[u,u] S[u] + sum_{v local, v ~ u} A_hat[u,v] S[v] ) Wg
    for every halo node u: one GCN propagation over the edges of the
    partition-plus-halo graph that touch a local node, restricted to halo
    rows, no activation. S stacks local rows then halo rows."""
    n_local, n_halo = view["n_local"], view["n_halo"]
    h_colptr, h_row, h_val, h_self = (view["h_colptr"], view["h_row"],
                                      view["h_val"], view["h_self"])
    S = np.asarray(S, np.float64)
    agg = np.zeros((n_halo, S.shape[1]))
    for u in range(n_halo):
        s, e = h_colptr[u], h_colptr[u + 1]
        agg[u] = float(h_self[u]) * S[n_local + u] \
            + h_val[s:e].astype(np.float64) @ S[h_row[s:e]]
    return agg @ np.asarray(Wg, np.float64)


def predict(view, omega, slots, bypass=False):
    """Predicted halo embeddings H_out_hat [n_halo, d] of one hidden layer.

    slots: tau arrays [n_local + n_halo, d], the cached embeddings of the
    partition's nodes and its halo for the last tau epochs, oldest first.
      1. S = lstm_last_hidden(slots)                    (all n_local + n_halo nodes)
      2. Delta = predictor_hop(S)                       (halo rows only)
      3. H_out_hat = newest slot's halo rows + Delta    (correction of the stale value)
    bypass=True returns the newest slot's halo rows untouched (plain
    historical embeddings, the uncorrected baseline).

    Open points of the paper fixed here: one LSTM layer, zero initial state
    per window, gate order i, f, g, o, a single bias; one parameter set per
    hidden layer; the hop reuses the global A_hat values; the output is a
    residual on the newest cached embedding.
    """
    n_local = view["n_local"]
    newest = np.asarray(slots[-1][n_local:], np.float64)
    if bypass:
        return newest.copy()
    S = lstm_last_hidden(slots, omega["Wx"], omega["Wh"], omega["b"])
    return newest + predictor_hop(view, S, omega["Wg"])


# --------------------------------------------------------------------------
# Whole step of one partition (Alg. 1 inner body; Eq. 7; appendix fwd / bwd)
# --------------------------------------------------------------------------
def predictor_train_loss_and_grad(view, omega, slots, target, weight=None):
    """Loss of the embedding predictor on this partition and its gradient (Eq. 11
    restricted to one partition and one hidden layer; Eq. 12 through `weight`).

    The partition knows this step's fresh embeddings only for its local nodes,
    so that is where the predictor is supervised: for local node v
        pred[v] = newest[v] + ( sum_u A_hat[v,u] S[u] ) Wg
    with the sum over row v of [P_in | P_out] (self-loop, local and halo
    neighbours: one GCN hop over the partition-plus-halo graph, the local-row
    counterpart of predictor_hop) and S the LSTM state of every node of the
    partition and its halo. target [n_local, d] holds the fresh embeddings (a
    constant here). weight [n_local] (default all ones) selects / weights the
    mini-batch:
        loss = sum_v weight[v] |pred[v] - target[v]|^2 / (d * sum_v weight[v]).
    Returns (loss, dict(Wx=, Wh=, b=, Wg=)) with the gradients, by
    back-propagation through the hop and through the LSTM's tau steps.
    """
    Wx = np.asarray(omega["Wx"], np.float64)
    Wh = np.asarray(omega["Wh"], np.float64)
    b = np.asarray(omega["b"], np.float64)
    Wg = np.asarray(omega["Wg"], np.float64)
    d_s = Wh.shape[1]
    n_local, n_halo = view["n_local"], view["n_halo"]
    n_bar = n_local + n_halo
    tau = len(slots)
    xs = [np.asarray(x, np.float64) for x in slots]
    target = np.asarray(target, np.float64)
    d = target.shape[1]
    w = np.ones(n_local) if weight is None else np.asarray(weight, np.float64)

    # forward, keeping every step's gates
    h = [np.zeros((n_bar, d_s))]
    c = [np.zeros((n_bar, d_s))]
    gi, gf, gg, go = [], [], [], []
    for s in range(tau):
        pre = xs[s] @ Wx.T + h[s] @ Wh.T + b
        gi.append(_sigmoid(pre[:, 0 * d_s:1 * d_s]))
        gf.append(_sigmoid(pre[:, 1 * d_s:2 * d_s]))
        gg.append(np.tanh(pre[:, 2 * d_s:3 * d_s]))
        go.append(_sigmoid(pre[:, 3 * d_s:4 * d_s]))
        c.append(gf[s] * c[s] + gi[s] * gg[s])
        h.append(go[s] * np.tanh(c[s + 1]))
    S = h[tau]
    agg = spmm_fwd(view, S)                              # [n_local, d_s]
    pred = xs[-1][:n_local] + agg @ Wg
    diff = pred - target
    norm = d * w.sum()
    loss = float((w[:, None] * diff * diff).sum() / norm)

    # backward
    dpred = 2.0 * w[:, None] * diff / norm
    dWg = agg.T @ dpred
    dagg = dpred @ Wg.T
    dS_loc, dS_halo = spmm_bwd(view, dagg, want_halo=True)
    dh = np.concatenate([dS_loc, dS_halo], axis=0)
    dc = np.zeros((n_bar, d_s))
    dWx = np.zeros_like(Wx)
    dWh = np.zeros_like(Wh)
    db = np.zeros_like(b)
    for s in range(tau - 1, -1, -1):
        tc = np.tanh(c[s + 1])
        do = dh * tc
        dc = dc + dh * go[s] * (1.0 - tc * tc)
        da = np.concatenate([dc * gg[s] * gi[s] * (1.0 - gi[s]),          # i
                             dc * c[s] * gf[s] * (1.0 - gf[s]),           # f
                             dc * gi[s] * (1.0 - gg[s] * gg[s]),          # g
                             do * go[s] * (1.0 - go[s])], axis=1)         # o
        dWx += da.T @ xs[s]
        dWh += da.T @ h[s]
        db += da.sum(axis=0)
        dh = da @ Wh
        dc = dc * gf[s]
    return loss, dict(Wx=dWx, Wh=dWh, b=db, Wg=dWg)


def partition_step(view, X_local, X_halo, halo_hat, Ws, y, store=None, stale_grad=None):
    """Forward and backward of an L-layer GCN on one partition.

    stale_grad (optional): stale_grad[l] for l = 1..L-1, [n_local, d_l]: the second
    term of the appendix's SAT backward, P_out^T D~^(t-1) W^T, as this partition's
    local nodes receive it from the partitions that hold them as halo nodes (it
    was computed there one step earlier); added to dH_in[l]. The matching
    output is dH_halo[l] = P_out^T dAGG_l, this partition's contribution to the
    owners of its halo nodes.

    store (optional): applied to every tensor the step keeps in memory between
    calls (AGG, H, the loss gradient, dAGG, dH_in) - the identity for fp32
    storage, round_bf16 for the bf16 storage mode. dW is an fp32 output and
    is never rounded.

    X_local / X_halo: input features of local / halo nodes (layer 0 uses the
    true features of halo nodes: they are static, nothing is stale).
    halo_hat[l] for l = 1..L-1: the halo rows fed to layer l+1 (predicted or
    plain historical); halo_hat[0] is ignored. They are constants of the step:
    no gradient is returned for them.
    Returns dict with per-layer lists AGG, Z, H (H[0] = X_local), the loss,
    dW per layer, and dH_in per layer (None for layer 0).
    """
    if store is None:
        store = lambda t: t
    L = len(Ws)
    H = [np.asarray(X_local, np.float64)]
    AGG, Z = [], []
    for l in range(L):
        halo = X_halo if l == 0 else halo_hat[l]
        Hbar = np.concatenate([H[l], np.asarray(halo, np.float64)], axis=0)
        a = store(spmm_fwd(view, Hbar))
        z, h = dense_fwd(a, Ws[l], 1 if l < L - 1 else 0)
        AGG.append(a)
        Z.append(z)
        H.append(store(h))
    loss, g = loss_and_grad(H[L], y)
    g = store(g)
    dW = [None] * L
    dH_in = [None] * L
    dZ = [None] * L
    dAGGs = [None] * L
    dH_halo = [None] * L
    for l in range(L - 1, -1, -1):
        # relu'(Z) = [H > 0]: the stored forward output is the mask (for bf16 storage a
        # positive Z never rounds to zero, so this is the same decision)
        dW[l], dAGG, dZ[l] = dense_bwd(g, H[l + 1] if l < L - 1 else Z[l], AGG[l], Ws[l],
                                       1 if l < L - 1 else 0)
        dAGG = store(dAGG)
        dAGGs[l] = dAGG
        if l >= 1:
            g, gh = spmm_bwd(view, dAGG, want_halo=True)
            dH_halo[l] = store(gh)
            if stale_grad is not None and stale_grad[l] is not None:
                g = g + np.asarray(stale_grad[l], np.float64)
            g = store(g)
            dH_in[l] = g
    return dict(AGG=AGG, Z=Z, H=H, loss=loss, dW=dW, dH_in=dH_in, dZ=dZ, dAGG=dAGGs,
                dH_halo=dH_halo)


def full_graph_gcn(N, g_rowptr, g_col, X, Ws):
    """Unpartitioned L-layer GCN on all N nodes: H^(l+1) = sigma(A_hat H^(l) W^(l)),
    relu on hidden layers, identity on the last. Returns [H^(0), ..., H^(L)].
    Written directly on the global CSR (self-loop added per row), independent
    of partition_view."""
    isd = inv_sqrt_degree(np.diff(g_rowptr))
    H = [np.asarray(X, np.float64)]
    L = len(Ws)
    for l in range(L):
        agg = np.zeros_like(H[l])
        for i in range(N):
            nb = g_col[g_rowptr[i]:g_rowptr[i + 1]]
            w = (isd[i] * isd[nb]).astype(np.float64)      # fp32 product, then widened
            agg[i] = w @ H[l][nb] + np.float64(isd[i] * isd[i]) * H[l][i]
        z = agg @ np.asarray(Ws[l], np.float64)
        H.append(np.maximum(z, 0.0) if l < L - 1 else z)
    return H


def full_graph_backward(N, g_rowptr, g_col, X, Ws, y, part):
    """Backward of the unpartitioned GCN for the loss sum over partitions m of
    (mean cross-entropy over V_m): the appendix's G_H = P^T D W^T, G_W = (P H)^T D,
    D = G_H o sigma'(Z), written on the global CSR. y: labels of all N nodes;
    part: partition id of every node (it only sets each node's loss weight
    1 / |V_part(v)|). Returns (G_H list indexed by layer, dW list)."""
    isd = inv_sqrt_degree(np.diff(g_rowptr))
    part = np.asarray(part)

    def propagate(M):          # A_hat M (A_hat is symmetric, so this is also A_hat^T M)
        out = np.zeros_like(M)
        for i in range(N):
            nb = g_col[g_rowptr[i]:g_rowptr[i + 1]]
            w = (isd[i] * isd[nb]).astype(np.float64)
            out[i] = w @ M[nb] + np.float64(isd[i] * isd[i]) * M[i]
        return out

    L = len(Ws)
    H = [np.asarray(X, np.float64)]
    PH, Z = [], []
    for l in range(L):
        a = propagate(H[l])
        z = a @ np.asarray(Ws[l], np.float64)
        PH.append(a)
        Z.append(z)
        H.append(np.maximum(z, 0.0) if l < L - 1 else z)
    zmax = H[L].max(axis=1, keepdims=True)
    p = np.exp(H[L] - zmax)
    p /= p.sum(axis=1, keepdims=True)
    p[np.arange(N), y] -= 1.0
    sizes = np.bincount(part)
    G = p / sizes[part][:, None]
    G_H = [None] * (L + 1)
    G_H[L] = G
    dW = [None] * L
    for l in range(L - 1, -1, -1):
        D = G_H[l + 1] * (Z[l] > 0) if l < L - 1 else G_H[l + 1]
        dW[l] = PH[l].T @ D
        G_H[l] = propagate(D @ np.asarray(Ws[l], np.float64).T)
    return G_H, dW


# --------------------------------------------------------------------------
# Compression of stored embeddings (Sec. "Data Compression for Historical
# Embedding Storage"): decimal rounding + the published Encoded Polyline
# Algorithm Format's variable-length character coding, every value on its own.
# --------------------------------------------------------------------------

POLYLINE_Q_MAX = 1 << 30


def polyline_quantise(H, precision, arith=np.float32):
    """q = floor(v * 10^precision + 1/2) per element, as int64. `arith` is the
    floating type the three operations run in: float32 is what the GPU path uses
    (the quantised code is an integer decision, so both sides take it in that
    precision); float64 serves the published worked examples."""
    v = np.asarray(H).astype(arith)
    scale = arith(10.0) ** arith(precision) if arith is np.float64 else np.float32(10.0 ** precision)
    with np.errstate(over="ignore", invalid="ignore"):
        x = np.floor(v * scale + arith(0.5))
    # Out of range (the section is silent; reading): the character coding is defined on
    # signed 32-bit integers after the left shift, so |q| is held at POLYLINE_Q_MAX = 2^30,
    # the largest magnitude whose shifted code fits 32 bits for either sign (+-inf and
    # overflowing products land there too); a NaN has no decimal rounding and codes as 0.
    x = np.where(np.isnan(x), arith(0.0), x)
    x = np.clip(x, -float(POLYLINE_Q_MAX), float(POLYLINE_Q_MAX))
    return x.astype(np.int64)


def polyline_encode_value(q):
    """Bytes of one signed integer: shift left one bit, invert all bits if the
    value is negative, cut into 5-bit groups from the low end, set bit 0x20 on
    every group that has a successor, add 63 to each group."""
    u = (int(q) << 1) ^ (-1 if q < 0 else 0)          # ~(q << 1) for negative q
    out = bytearray()
    while True:
        chunk = u & 0x1F
        u >>= 5
        if u:
            out.append((chunk | 0x20) + 63)
        else:
            out.append(chunk + 63)
            return bytes(out)


def polyline_encode_rows(H, precision, arith=np.float32):
    """Every row of H as the concatenation of its values' codes. Returns
    (codes uint8 [total], row_off int64 [n + 1])."""
    q = polyline_quantise(H, precision, arith)
    rows = [b"".join(polyline_encode_value(x) for x in r) for r in q]
    row_off = np.zeros(len(rows) + 1, dtype=np.int64)
    np.cumsum([len(r) for r in rows], out=row_off[1:])
    codes = np.frombuffer(b"".join(rows), dtype=np.uint8).copy() if rows else np.zeros(0, np.uint8)
    return codes, row_off


def polyline_decode_rows(codes, row_off, ids, d, precision):
    """out[k, :] = decoded row ids[k] (d values each): q / 10^precision in fp32
    (one correctly rounded division, which is what the GPU path does)."""
    scale = np.float32(10.0 ** precision)
    out = np.zeros((len(ids), d), dtype=np.float32)
    for k, r in enumerate(ids):
        pos = int(row_off[r])
        for c in range(d):
            u, shift = 0, 0
            while True:
                b = int(codes[pos]) - 63
                pos += 1
                u |= (b & 0x1F) << shift
                shift += 5
                if not (b & 0x20):
                    break
            q = ~(u >> 1) if (u & 1) else (u >> 1)
            out[k, c] = np.float32(q) / scale
        assert pos == row_off[r + 1], "row %d does not hold exactly %d values" % (r, d)
    return out


def polyline_stored_value(H, precision):
    """What a reader of a coded table gets back for every element of H: the value
    quantised as in polyline_quantise and divided by 10^precision as in
    polyline_decode_rows, without building the byte strings (the coding of the
    integers is lossless). For whole tables, where the byte-by-byte functions are
    too slow; pinned against them on small matrices."""
    q = polyline_quantise(H, precision)
    return (q.astype(np.float32) / np.float32(10.0 ** precision)).astype(np.float32)


def staleness(H_ref, H_approx):
    """Frobenius norm of the difference (Eq. 6 with the Frobenius norm)."""
    return float(np.linalg.norm(np.asarray(H_ref, np.float64) - np.asarray(H_approx, np.float64)))
