"""Per-call checks of the last layer when the step evaluates it as P (Hbar W)
(PartitionStep.transform_first), for the full-size tests: the inputs of every call are read
back from the device for sampled outputs and the oracle computes those outputs from them;
the weight gradient, a sum over ALL local and halo rows, is recomputed in full."""
import numpy as np

from oracle import sat_oracle as orc


def check_last_layer_transform_first(gu, torch, wl, rows, halo_sample, rtol, rounder=None, say=print):
    """rows: sampled local rows; halo_sample: sampled halo nodes. rounder: the storage rounding
    (bf16 mode) or None. Must be called right after one forward_backward()."""
    v, step, dims = wl.view, wl.step, wl.dims
    L = len(dims) - 1
    n_l, n_h = v["n_local"], v["n_halo"]
    C, d = dims[L], dims[L - 1]
    rd = rounder or (lambda a: a)
    W = wl.Ws[L - 1]

    def fetch(t, idx, width):
        i = torch.from_numpy(np.asarray(idx, dtype=np.int64)).to(gu.DEV)
        return t[i].float().cpu().numpy()[:, :width]

    assert step.transform_first and step.AGG[L - 1] is None
    # Zbar rows of sampled local and halo nodes (incl. the last row of the buffer)
    nodes = np.unique(np.concatenate([rows, n_l + halo_sample, [n_l + n_h - 1]]))
    zb = orc.dense_fwd(fetch(step.Hbar[L - 1], nodes, d), W, 0)[0]
    gu.assert_close(fetch(step.Zbar, nodes, C), rd(zb), rtol, "Zbar rows")
    # logits rows from the stored Zbar
    segs = [(int(v["rowptr"][i]), int(v["rowptr"][i + 1])) for i in rows]
    cols = np.concatenate([v["col"][a:b] for a, b in segs])
    uniq, inv = np.unique(cols, return_inverse=True)
    rowptr = np.concatenate([[0], np.cumsum([b - a for a, b in segs])]).astype(np.int64)
    split = rowptr[:-1] + np.array([int(v["split"][i]) - a for i, (a, b) in zip(rows, segs)], dtype=np.int64)
    mini = dict(rowptr=rowptr, split=split, col=inv.astype(np.int32),
                val=np.concatenate([v["val"][a:b] for a, b in segs]))
    ar = np.arange(len(rows))
    lg = orc.spmm_fwd_rows(mini, fetch(step.Zbar, uniq, C), ar)
    gu.assert_close(fetch(step.logits, rows, C), rd(lg), rtol, "logits rows")
    # G = [P_in | P_out]^T dH^(L): local rows through the symmetry of P_in, halo rows through
    # the transposed halo block, both from the stored dH^(L)
    loc = uniq < n_l
    Gin = np.zeros((len(uniq), C), dtype=np.float32)
    Gin[loc] = fetch(step.dH[L], uniq[loc], C)
    gu.assert_close(fetch(step.G, rows, C), rd(orc.spmm_bwd_rows(mini, Gin, ar)), rtol, "G local rows")
    cp = v["h_colptr"]
    ref = np.zeros((len(halo_sample), C))
    for k, u in enumerate(halo_sample):
        a, b = int(cp[u]), int(cp[u + 1])
        ref[k] = v["h_val"][a:b].astype(np.float64) @ fetch(step.dH[L], v["h_row"][a:b], C).astype(np.float64)
    gu.assert_close(fetch(step.G, n_l + halo_sample, C), rd(ref), rtol, "G halo rows")
    # dH^(L-1) rows = G_local W^T
    dh = orc.dense_bwd(fetch(step.G, rows, C), None, np.zeros((len(rows), d)), W, 0)[1]
    gu.assert_close(fetch(step.dH[L - 1], rows, d), rd(dh), rtol, "dH^(L-1) rows")
    # dW = Hbar^T G over all local + halo rows, in row chunks
    n_bar = n_l + n_h
    dW = np.zeros((d, C))
    for a in range(0, n_bar, 1 << 19):
        b = min(a + (1 << 19), n_bar)
        dW += orc.dense_bwd(step.G[a:b, :C].double().cpu().numpy(), None,
                            step.Hbar[L - 1][a:b, :d].double().cpu().numpy(), W, 0)[0]
    got = step.dW[L - 1][:, :C].cpu().numpy()
    gu.assert_close(got, dW, rtol, "dW of the last layer over all local + halo rows")
    say("last layer as P (Hbar W): Zbar, logits, G, dH, dW ok (dW norm-wise error %.2e)" % gu.normwise(got, dW))
