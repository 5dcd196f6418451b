"""One partition's SAT GCN training step as a sequence of libsat calls.

Orchestration only: this module owns the device buffers (torch tensors, used
as plain memory) and issues the C-ABI calls in the order of the paper's inner
loop (Alg. 1): pull / predict, forward per layer, push, local loss, backward.
No arithmetic happens here.

Order inside a step t (history ring of tau slots per hidden layer):
  1. predictions for every hidden layer l = 1..L-1 from the tau slots as they
     stood at the end of step t-1 (so no push of step t is visible to them);
  2. for l = 0..L-1: halo rows of layer 0 are the static features (pull);
     AGG_l = [P_in | P_out] Hbar_l; H_{l+1} = act(AGG_l W_l), written straight
     into the local rows of Hbar_{l+1}; push H_{l+1} into slot t mod tau of the
     layer's ring (it overwrites the oldest epoch);
  3. dH_L from the cross-entropy; for l = L-1..0: dW_l, dAGG_l; dH_l = P_in^T dAGG_l
     for l >= 1 (halo rows are constants of the step: no gradient for them).
     With gradient tables (the second term of the appendix's SAT backward): also
     dH_halo_l = P_out^T dAGG_l, pushed into the write table of the layer's gradient
     ring for the owners of the halo nodes, and the rows the local nodes find in the
     read table (written one step earlier by the partitions that hold them as halo
     nodes) are added to dH_l.

With a coded ring (CodedRing; the paper's section on compressing the stored historical
embeddings) the slots hold the variable-length codes instead of dense rows: step 1 decodes
the window of every hidden layer into dense scratch rows first (pull and decode in one
pass) and the push of step 2 codes the fresh rows straight from the layer's output.
"""
import numpy as np
import torch

from . import binding as B


def _ld(d, mult=32):
    return (d + mult - 1) // mult * mult


class CodedSlot:
    """One epoch of one hidden layer, stored coded, in the two parts the owner-sharded ring
    has: `own` - the rows of the partition's local nodes in local order, rewritten whole by
    every push (rows of variable length cannot be replaced in place) - and `remote` - the
    rows of its halo nodes in halo order, as their owners pushed them. Each part is
    (codes uint8 [capacity], row_off int64 [rows + 1]) on the device."""

    def __init__(self, own_codes, own_off, remote_codes, remote_off):
        self.own_codes, self.own_off = own_codes, own_off
        self.remote_codes, self.remote_off = remote_codes, remote_off

    def coded_bytes(self):
        """Bytes of code the two parts hold now (reads two offsets back: synchronises)."""
        return int(self.own_off[-1].item()), int(self.remote_off[-1].item())


class CodedRing:
    """slots[l][s] for l = 1..L-1, s = 0..tau-1: CodedSlot; precision: decimals kept."""

    def __init__(self, precision, slots):
        self.precision, self.slots = int(precision), slots


def encode_rows(H, ld_h, n, d, precision, dtype, capacity=None, headroom=1.0, stream=None):
    """Code the dense rows H [n, ld_h] into a new (codes, row_off) pair. capacity None: the
    size these rows need (read back after the sizing pass, which synchronises) times
    `headroom` (room for later pushes into the same part); else the bytes to allocate (rows
    that would end beyond it are not written; row_off still tells)."""
    dev = H.device
    row_off = torch.zeros(n + 1, dtype=torch.int64, device=dev)
    wsb = B.history_compress_workspace_bytes(n)
    ws = torch.empty((wsb + 7) // 8, dtype=torch.int64, device=dev)
    B.history_compress_plan(H, ld_h, n, d, precision, row_off, dtype=dtype, workspace=ws,
                            workspace_bytes=wsb, stream=stream)
    if capacity is None:
        capacity = int(int(row_off[-1].item()) * headroom) + 1
    codes = torch.zeros(max(int(capacity), 16), dtype=torch.uint8, device=dev)
    B.history_compress_encode(H, ld_h, n, d, precision, row_off, codes, int(capacity), dtype=dtype,
                              stream=stream)
    return codes, row_off


class PartitionStep:
    """Buffers and call sequence for one partition.

    view: dict of host arrays from binding.partition_view_build.
    X_table: device [n_rows_x, ld_x] input features of all nodes the ids refer to.
    hist: hist[l] for l = 1..L-1 is a list of tau device tables [n_rows_h, ld_l]
          (hist[0] unused); ring position is tracked here.
    table_ids: device int32 [n_bar]; row of each local-then-halo node in X_table
          and in every history table.
    Ws: device weights, Ws[l] is [d_l, ld_w_l] (ld_w_l a multiple of 4 floats / 8 bf16).
    dtype: binding.F32 or binding.BF16 - element type of features, activations,
          history tables and Ws (dW, the loss and the predictor parameters are fp32).
    predictors: predictors[l] a binding.Predictor for l = 1..L-1 (None: bypass).
    y: device int32 [n_local] labels.
    predict_ahead: the predictions of step t + 1 only need the ring as step t's pushes leave
          it, and nothing in step t's backward reads the halo rows they write: with this
          flag they are enqueued on a second stream (same priority) right after step t's
          last push, beside step t's loss and backward, and step t + 1 waits for them before
          its first use of a predicted row and before its first push into a slot they read.
          Results are identical to the sequential order. Dense ring, fused pull only.
    transform_first: the appendix writes a layer as Z = P H W without saying which product
          comes first. The last layer has no activation between the two and usually narrows
          (256 -> 47 classes), so with this flag it is evaluated as P (Hbar W): the transform
          runs over all local + halo rows, and the aggregation and its transpose then gather
          rows of n_classes instead of d_{L-1} elements. Backward accordingly: G = [P_in |
          P_out]^T dH^(L) (local and halo rows), dW = Hbar^T G over all rows, dH^(L-1) =
          G_local W^T. AGG_{L-1} and dAGG_{L-1} are then never formed. "auto": when the last
          layer narrows to half or less. Not with gradient tables.
    projection_cache: keep the LSTM's input projection x Wx^T of every ring slot (one
          [n_bar, 4 d_s] fp32 matrix per slot and hidden layer) and let the predictor read it
          for the slots it has already seen (sat_predict_cached): consecutive windows share
          all but their newest slot, so with tau = 2 the input products of a step halve.
          Bit-identical results. A push into a slot invalidates its matrix; after an update of
          the predictor's parameters call invalidate_projection_cache(). Dense ring, fused
          pull, d_s <= 64 only.
    predict_every: Delta T of Alg. 1 - the predicted halo rows are refreshed on steps
          t = 0, Delta T, 2 Delta T, ... and reused (they stay in the halo rows of Hbar_l) in between.
    grad_tables: None, or grad_tables[l] for l = 1..L-1 a pair [table_a, table_b] of
          device tables [n_rows_g, ld_l] (row of a node as in the history tables): step
          t reads pair[t % 2] (stale term for the local rows) and writes pair[(t+1) % 2]
          (this partition's term for its halo nodes).
    coded: None, or a CodedRing that replaces hist (hist is then ignored): the window is
          decoded into dense scratch rows before the predictions and every push codes the
          layer's fresh rows into the `own` part of the write slot. A push whose codes do
          not fit the part's capacity leaves the rows beyond it unwritten: coded_overflow()
          tells (the caller sizes the parts; see encode_rows).
    coded_chunk_rows: with a coded ring, None (the whole window of a layer is decoded into
          tau dense matrices of n_bar rows) or a row count: the window is decoded that many
          rows at a time, each range goes through the LSTM at once (sat_predict_states; the
          LSTM is row-wise) and only its d_s states are kept; the newest slot's halo rows are
          decoded straight into the halo rows of Hbar_l, where the hop (sat_predict_hop) adds
          its term in place. The dense scratch shrinks from tau * n_bar rows to tau * chunk
          rows (at full Scale: 34 GB to 1 GB); every result keeps its bits.
    """

    def __init__(self, view, dims, X_table, hist, table_ids, Ws, predictors, y, tau,
                 fused_pull=True, timers=None, dtype=B.F32, grad_tables=None, predict_every=1,
                 coded=None, predict_ahead=False, transform_first=False, projection_cache=False,
                 coded_chunk_rows=None):
        dev = X_table.device
        self.coded_chunk_rows = int(coded_chunk_rows) if (coded is not None and coded_chunk_rows) else None
        self.predict_ahead = bool(predict_ahead)
        L_ = len(dims) - 1
        if transform_first == "auto":     # worth it when the last layer narrows to half or less
            transform_first = 2 * dims[L_] <= dims[L_ - 1]
        self.transform_first = bool(transform_first) and grad_tables is None
        self.dtype = dtype
        self.dims = list(dims)
        self.L = len(dims) - 1
        self.tau = tau
        self.view = view
        self.n_local, self.n_halo = view["n_local"], view["n_halo"]
        self.n_bar = self.n_local + self.n_halo
        self.nnz = view["nnz"]
        self.nnz_local = int(np.sum(view["split"] - view["rowptr"][:-1]))
        t = {k: torch.from_numpy(np.ascontiguousarray(view[k])).to(dev)
             for k in ("rowptr", "split", "col", "val", "h_colptr", "h_row", "h_val", "h_self")}
        self.pv = B.PartView(view["n_local"], view["n_halo"], view["nnz"], view["nnz_halo"], **t)
        self.X_table, self.hist, self.table_ids = X_table, hist, table_ids
        self.halo_table_ids = table_ids[self.n_local:]
        self.local_table_ids = table_ids[:self.n_local]
        # None stands for plain historical embeddings: a predictor in bypass mode (no parameters)
        predictors = [None] + [w if w is not None else B.Predictor(None, None, None, None, dims[l], 0, tau,
                                                                   bypass=True)
                               for l, w in enumerate(predictors) if l >= 1]
        self.Ws, self.predictors, self.y = Ws, predictors, y
        self.coded = coded
        self.fused_pull = fused_pull and coded is None
        fused_pull = self.fused_pull
        self.grad_tables = grad_tables
        self.predict_every = max(1, int(predict_every))
        self.t = 0
        self.timers = timers

        f32 = dict(dtype=torch.float32, device=dev)
        act = dict(dtype=torch.bfloat16 if dtype == B.BF16 else torch.float32, device=dev)
        L, n_l, n_bar = self.L, self.n_local, self.n_bar
        self.ld = [_ld(d) for d in dims]
        self.ld_w = [Ws[l].shape[1] for l in range(L)]
        self.Hbar = [torch.zeros((n_bar, self.ld[l]), **act) for l in range(L)]
        self.logits = torch.zeros((n_l, self.ld[L]), **act)
        tf = self.transform_first
        self.AGG = [torch.zeros((n_l, self.ld[l]), **act) if not (tf and l == L - 1) else None
                    for l in range(L)]
        self.dH = [torch.zeros((n_l, self.ld[l]), **act) if l >= 1 else None for l in range(L + 1)]
        self.dAGG = [torch.zeros((n_l, self.ld[l]), **act) if l >= 1 and not (tf and l == L - 1) else None
                     for l in range(L)]
        # transform first: Zbar = Hbar_{L-1} W over all rows, G = P^T dH^(L) over all rows
        self.Zbar = torch.zeros((n_bar, self.ld[L]), **act) if tf else None
        self.G = torch.zeros((n_bar, self.ld[L]), **act) if tf else None
        self.ld_dw = [_ld(dims[l + 1], 4) for l in range(L)]
        self.dW = [torch.zeros((dims[l], self.ld_dw[l]), **f32) for l in range(L)]   # always fp32
        self.dH_halo = [None] * L
        if grad_tables is not None:
            self.dH_halo = [torch.zeros((self.n_halo, self.ld[l]), **act) if l >= 1 else None
                            for l in range(L)]
        self.loss = torch.zeros(1, **f32)
        ws_bytes = [B.loss_workspace_bytes(n_l)]
        ws_bytes += [B.dense_bwd_workspace_bytes(n_bar if (tf and l == L - 1) else n_l, dims[l], dims[l + 1])
                     for l in range(L)]
        for l in range(1, L):
            if not predictors[l].bypass and not self.coded_chunk_rows:   # (else: the two halves' own, below)
                ws_bytes.append(B.predict_workspace_bytes(n_l, self.n_halo, dims[l],
                                                          predictors[l].d_s, tau))
        if coded is not None:
            ws_bytes.append(B.history_compress_workspace_bytes(n_l))
        if self.coded_chunk_rows:
            for l in range(1, L):
                if not predictors[l].bypass:
                    ws_bytes.append(B.predict_states_workspace_bytes(dims[l], predictors[l].d_s))
                    ws_bytes.append(B.predict_hop_workspace_bytes(self.n_halo, predictors[l].d_s))
        self.ws_bytes = max(ws_bytes + [256])
        self.ws = torch.empty((self.ws_bytes + 3) // 4, **f32)
        self.proj = None
        if projection_cache and L >= 2:
            assert coded is None and self.fused_pull, "the projection cache goes with the dense ring and the fused pull"
            self.proj = [None] + [[torch.zeros((n_bar, 4 * predictors[l].d_s), **f32) for _ in range(tau)]
                                  if (not predictors[l].bypass and predictors[l].d_s <= 64) else None
                                  for l in range(1, L)]
            self._proj_valid = [None] + [[False] * tau for _ in range(1, L)]
        self._side = None
        if self.predict_ahead:
            assert coded is not None or self.fused_pull, "predict_ahead goes with the fused pull (or the coded ring)"
            self._side = torch.cuda.Stream(device=dev)          # default priority
            self._ws_side = torch.empty((self.ws_bytes + 3) // 4, **f32)   # the predictor's own scratch
            self._pred_done = None      # event: predictions for step self.t are in place
        if not fused_pull and L >= 2:
            # dense rows of one layer's window, shared by the hidden layers (a layer's pull
            # and prediction are over before the next layer's pull starts); with
            # coded_chunk_rows: of one range of rows
            n_win = min(n_bar, self.coded_chunk_rows) if self.coded_chunk_rows else n_bar
            flat = [torch.zeros(n_win * max(self.ld[1:L]), **act) for _ in range(tau)]
            self.window = [[f[:n_win * self.ld[l]].view(n_win, self.ld[l]) for f in flat]
                           if l >= 1 else None for l in range(L)]
            if self.coded_chunk_rows:      # LSTM states of all rows of one layer
                ds_max = max([predictors[l].d_s for l in range(1, L) if not predictors[l].bypass] + [1])
                self.S = torch.zeros(n_bar * ds_max, **f32)
        # local rows of layer 0 are static: pulled once
        B.history_gather(X_table, X_table.shape[0], X_table.shape[1], self.local_table_ids,
                         n_l, dims[0], self.Hbar[0], self.ld[0], dtype=dtype, stream=self._stream())

    @staticmethod
    def _stream():
        return torch.cuda.current_stream().cuda_stream

    def _timed(self, name, fn):
        if self.timers is None:
            fn()
        else:
            self.timers.record(name, fn)

    def invalidate_projection_cache(self):
        """After the predictor's parameters changed: every kept projection is stale."""
        if self.proj is not None:
            for l in range(1, self.L):
                self._proj_valid[l] = [False] * self.tau

    def _predict_in_place(self, l, order, ws, stream):
        """sat_predict of hidden layer l straight from the ring (slots in window order), with the
        kept input projections where there are any."""
        w = self.predictors[l]
        slots = [self.hist[l][s] for s in order]
        n_rows, ld_t = slots[0].shape
        if self.proj is None or self.proj[l] is None:
            B.predict(self.pv, w, slots, n_rows, ld_t, self.table_ids, self.Hbar[l], self.ld[l],
                      dtype=self.dtype, workspace=ws, workspace_bytes=self.ws_bytes, stream=stream)
            return
        valid = self._proj_valid[l]
        n_valid = 0
        while n_valid < len(order) - 1 and valid[order[n_valid]]:
            n_valid += 1
        B.predict_cached(self.pv, w, slots, n_rows, ld_t, self.table_ids, self.Hbar[l], self.ld[l],
                         [self.proj[l][s] for s in order], n_valid, dtype=self.dtype, workspace=ws,
                         workspace_bytes=self.ws_bytes, stream=stream)
        for pos, s in enumerate(order):      # every slot but the window's first now has its matrix
            if pos >= 1:
                valid[s] = True

    def slot_order(self):
        """Ring slots oldest -> newest as seen by step t's predictions."""
        return [(self.t + s) % self.tau for s in range(self.tau)]

    def forward_backward(self):
        L, dims, ld, n_l, n_h, n_bar = self.L, self.dims, self.ld, self.n_local, self.n_halo, self.n_bar
        st = self._stream()
        dt = self.dtype
        order = self.slot_order()
        if self.predict_ahead:
            return self._forward_backward_predict_ahead(st)
        # 1. predicted halo embeddings of every hidden layer (every Delta T steps)
        for l in range(1, L if self.t % self.predict_every == 0 else 1):
            w = self.predictors[l]
            if self.coded is not None:
                self._predict_coded(l, order, self.ws, st)
                continue
            slots = [self.hist[l][s] for s in order]
            n_rows, ld_t = slots[0].shape
            if self.fused_pull or w.bypass:
                self._timed("predict_l%d" % l, lambda: self._predict_in_place(l, order, self.ws, st))
            else:
                for k, s in enumerate(slots):
                    self._timed("gather_l%d" % l, lambda: B.history_gather(
                        s, n_rows, ld_t, self.table_ids, n_bar, dims[l], self.window[l][k],
                        ld[l], dtype=dt, stream=st))
                self._timed("predict_l%d" % l, lambda: B.predict(
                    self.pv, w, self.window[l], n_bar, ld[l], None, self.Hbar[l], ld[l], dtype=dt,
                    workspace=self.ws, workspace_bytes=self.ws_bytes, stream=st))
        # 2. forward
        w_slot = self.t % self.tau
        for l in range(L):
            if l == 0 and n_h > 0:
                halo0 = self.Hbar[0][n_l:]
                self._timed("gather_l0", lambda: B.history_gather(
                    self.X_table, self.X_table.shape[0], self.X_table.shape[1],
                    self.halo_table_ids, n_h, dims[0], halo0, ld[0], dtype=dt, stream=st))
            self._layer_forward(l, st)
            last = l == L - 1
            if not last and self.coded is not None:
                self._push_coded(l + 1, w_slot, st)
            elif not last:
                tab = self.hist[l + 1][w_slot]
                if self.proj is not None:
                    self._proj_valid[l + 1][w_slot] = False      # the slot's rows change
                self._timed("push_l%d" % (l + 1), lambda: B.history_push(
                    tab, tab.shape[0], tab.shape[1], self.local_table_ids, n_l, dims[l + 1],
                    self.Hbar[l + 1], ld[l + 1], dtype=dt, stream=st))
        self._backward(st)
        self.t += 1

    def _layer_forward(self, l, st):
        """AGG_l = [P_in | P_out] Hbar_l, H_{l+1} = act(AGG_l W_l); on the last layer with
        transform_first: Zbar = Hbar_l W_l over all rows, logits = [P_in | P_out] Zbar."""
        L, dims, ld, n_l, n_bar, dt = self.L, self.dims, self.ld, self.n_local, self.n_bar, self.dtype
        last = l == L - 1
        if last and self.transform_first:
            self._timed("dense_fwd_l%d" % l, lambda: B.dense_fwd(
                self.Hbar[l], ld[l], n_bar, dims[l], dims[L], self.Ws[l], self.ld_w[l],
                B.ACT_IDENTITY, self.Zbar, ld[L], dtype=dt, stream=st))
            self._timed("spmm_fwd_l%d" % l, lambda: B.spmm_fwd(
                self.pv, self.Zbar, ld[L], dims[L], self.logits, ld[L], dtype=dt, stream=st))
            return
        self._timed("spmm_fwd_l%d" % l, lambda: B.spmm_fwd(
            self.pv, self.Hbar[l], ld[l], dims[l], self.AGG[l], ld[l], dtype=dt, stream=st))
        out = self.logits if last else self.Hbar[l + 1]
        self._timed("dense_fwd_l%d" % l, lambda: B.dense_fwd(
            self.AGG[l], ld[l], n_l, dims[l], dims[l + 1], self.Ws[l], self.ld_w[l],
            B.ACT_IDENTITY if last else B.ACT_RELU, out, ld[l + 1], dtype=dt, stream=st))

    def _backward(self, st, after_last_layer=None):
        """3. loss gradient and backward. after_last_layer: called once the calls of layer
        L - 1 have been enqueued."""
        L, dims, ld, n_l, n_h = self.L, self.dims, self.ld, self.n_local, self.n_halo
        dt = self.dtype
        self._timed("loss_grad", lambda: B.loss_grad(
            self.logits, ld[L], n_l, dims[L], self.y, self.dH[L], ld[L], loss=self.loss, dtype=dt,
            workspace=self.ws, workspace_bytes=self.ws_bytes, stream=st))
        for l in range(L - 1, -1, -1):
            last = l == L - 1
            if last and self.transform_first:
                n_bar = self.n_bar
                g_halo = self.G[n_l:] if n_h > 0 else None
                self._timed("spmm_bwd_l%d" % l, lambda: B.spmm_bwd(
                    self.pv, self.dH[L], ld[L], dims[L], self.G, ld[L], dH_halo=g_halo, ld_halo=ld[L],
                    dtype=dt, stream=st))
                self._timed("dense_bwd_l%d" % l, lambda: B.dense_bwd(
                    self.G, ld[L], None, 0, self.Hbar[l], ld[l], self.Ws[l], self.ld_w[l], n_bar,
                    dims[l], dims[L], B.ACT_IDENTITY, self.dW[l], self.ld_dw[l], None, 0, dtype=dt,
                    workspace=self.ws, workspace_bytes=self.ws_bytes, stream=st))
                if l >= 1:
                    self._timed("dense_bwd_in_l%d" % l, lambda: B.dense_bwd(
                        self.G, ld[L], None, 0, None, 0, self.Ws[l], self.ld_w[l], n_l, dims[l],
                        dims[L], B.ACT_IDENTITY, None, 0, self.dH[l], ld[l], dtype=dt, stream=st))
                if after_last_layer is not None:
                    after_last_layer()
                continue
            hout = None if last else self.Hbar[l + 1]
            self._timed("dense_bwd_l%d" % l, lambda: B.dense_bwd(
                self.dH[l + 1], ld[l + 1], hout, 0 if last else ld[l + 1], self.AGG[l], ld[l],
                self.Ws[l], self.ld_w[l], n_l, dims[l], dims[l + 1],
                B.ACT_IDENTITY if last else B.ACT_RELU, self.dW[l], self.ld_dw[l],
                self.dAGG[l], ld[l] if l >= 1 else 0, dtype=dt,
                workspace=self.ws, workspace_bytes=self.ws_bytes, stream=st))
            if l >= 1 and self.grad_tables is None:
                self._timed("spmm_bwd_l%d" % l, lambda: B.spmm_bwd(
                    self.pv, self.dAGG[l], ld[l], dims[l], self.dH[l], ld[l], dtype=dt, stream=st))
            elif l >= 1:
                rd, wr = self.grad_tables[l][self.t % 2], self.grad_tables[l][(self.t + 1) % 2]
                self._timed("spmm_bwd_l%d" % l, lambda: B.spmm_bwd(
                    self.pv, self.dAGG[l], ld[l], dims[l], self.dH[l], ld[l],
                    dH_halo=self.dH_halo[l], ld_halo=ld[l], dtype=dt, stream=st))
                if n_h > 0:
                    self._timed("grad_push_l%d" % l, lambda: B.history_push(
                        wr, wr.shape[0], wr.shape[1], self.halo_table_ids, n_h, dims[l],
                        self.dH_halo[l], ld[l], dtype=dt, stream=st))
                self._timed("grad_pull_l%d" % l, lambda: B.history_gather_add(
                    rd, rd.shape[0], rd.shape[1], self.local_table_ids, n_l, dims[l],
                    self.dH[l], ld[l], dtype=dt, stream=st))

    # ------------------------------------------------ predictions one step ahead
    def _enqueue_predictions(self, t):
        """Predictions for step t on the side stream, after everything the main stream has
        enqueued so far (the pushes that complete the ring as of the end of step t - 1)."""
        main = torch.cuda.current_stream()
        self._side.wait_stream(main)
        if t % self.predict_every == 0:
            order = [(t + s) % self.tau for s in range(self.tau)]
            with torch.cuda.stream(self._side):
                sp = self._side.cuda_stream
                for l in range(1, self.L):
                    if self.coded is not None:      # decode the window, then predict from the dense rows
                        self._predict_coded(l, order, self._ws_side, sp)
                        continue
                    self._timed("predict_l%d" % l, lambda: self._predict_in_place(l, order, self._ws_side, sp))
        self._pred_done = torch.cuda.Event()
        self._pred_done.record(self._side)

    def _forward_backward_predict_ahead(self, st):
        L, dims, ld, n_l, n_h = self.L, self.dims, self.ld, self.n_local, self.n_halo
        dt = self.dtype
        main = torch.cuda.current_stream()
        if self._pred_done is None:             # first step: nothing was enqueued ahead
            self._enqueue_predictions(self.t)
        w_slot = self.t % self.tau
        for l in range(L):
            if l == 0 and n_h > 0:
                halo0 = self.Hbar[0][n_l:]
                self._timed("gather_l0", lambda: B.history_gather(
                    self.X_table, self.X_table.shape[0], self.X_table.shape[1],
                    self.halo_table_ids, n_h, dims[0], halo0, ld[0], dtype=dt, stream=st))
            self._layer_forward(l, st)
            last = l == L - 1
            if l == 0:
                # the first push overwrites a slot the predictions read, and the next layer
                # reads predicted rows: both wait here (layer 0 itself needs neither)
                main.wait_event(self._pred_done)
            if not last and self.coded is not None:
                self._push_coded(l + 1, w_slot, st)
            elif not last:
                tab = self.hist[l + 1][w_slot]
                if self.proj is not None:
                    self._proj_valid[l + 1][w_slot] = False      # the slot's rows change
                self._timed("push_l%d" % (l + 1), lambda: B.history_push(
                    tab, tab.shape[0], tab.shape[1], self.local_table_ids, n_l, dims[l + 1],
                    self.Hbar[l + 1], ld[l + 1], dtype=dt, stream=st))
        # The ring is complete for step t + 1: its predictions run beside this step's backward.
        # They overwrite the halo rows of every Hbar_l, which the backward reads in one place
        # only: the weight gradient of a last layer evaluated as P (Hbar W) sums over local
        # AND halo rows of Hbar_{L-1}. In that order they are enqueued after that layer.
        if self.transform_first:
            self._backward(st, after_last_layer=lambda: self._enqueue_predictions(self.t + 1))
        else:
            self._enqueue_predictions(self.t + 1)
            self._backward(st)
        self.t += 1

    # ------------------------------------------------------------ coded ring
    def _predict_coded(self, l, order, ws, st):
        """Predicted halo rows of hidden layer l from the coded ring: the whole window decoded
        and sat_predict, or (coded_chunk_rows) a range of rows at a time."""
        w = self.predictors[l]
        if not self.coded_chunk_rows or w.bypass:
            self._pull_coded(l, order, st)
            self._timed("predict_l%d" % l, lambda: B.predict(
                self.pv, w, self.window[l], self.n_bar, self.ld[l], None, self.Hbar[l], self.ld[l],
                dtype=self.dtype, workspace=ws, workspace_bytes=self.ws_bytes, stream=st))
            return
        n_l, n_bar, d, ld, P = self.n_local, self.n_bar, self.dims[l], self.ld[l], self.coded.precision
        C = self.coded_chunk_rows
        S = self.S[:n_bar * w.d_s].view(n_bar, w.d_s)
        # ranges of rows in local-then-halo order, none across the boundary between the two parts
        ranges = [(b, min(b + C, n_l)) for b in range(0, n_l, C)] + \
                 [(b, min(b + C, n_bar)) for b in range(n_l, n_bar, C)]
        for b, e in ranges:
            halo = b >= n_l
            srcs = []
            for k, s in enumerate(order):
                slot = self.coded.slots[l][s]
                codes, off = (slot.remote_codes, slot.remote_off[b - n_l:]) if halo else (slot.own_codes, slot.own_off[b:])
                # the newest slot's halo rows are also the hop's residual: decoded where it adds its term
                out = self.Hbar[l][b:e] if (halo and k == self.tau - 1) else self.window[l][k][:e - b]
                self._timed("pull_l%d" % l, lambda: B.history_decompress(
                    codes, off, e - b, None, e - b, d, P, out, ld, dtype=self.dtype, stream=st))
                srcs.append(out)
            self._timed("predict_l%d" % l, lambda: B.predict_states(
                w, srcs, e - b, ld, None, e - b, S[b:], dtype=self.dtype, workspace=ws,
                workspace_bytes=self.ws_bytes, stream=st))
        self._timed("predict_l%d" % l, lambda: B.predict_hop(
            self.pv, w, S, self.Hbar[l][n_l:], self.n_halo, ld, None, self.Hbar[l], ld, dtype=self.dtype,
            workspace=ws, workspace_bytes=self.ws_bytes, stream=st))

    def _pull_coded(self, l, order, st):
        """Decode the tau slots of layer l, oldest first, into the dense window rows (local
        rows from the `own` part, halo rows from the `remote` part; a bypass predictor reads
        the newest slot's halo rows only)."""
        n_l, n_h, d, P = self.n_local, self.n_halo, self.dims[l], self.coded.precision
        bypass = self.predictors[l].bypass
        for k, s in enumerate(order):
            if bypass and k != self.tau - 1:
                continue
            slot, win = self.coded.slots[l][s], self.window[l][k]
            if n_l > 0 and not bypass:
                self._timed("pull_l%d" % l, lambda: B.history_decompress(
                    slot.own_codes, slot.own_off, n_l, None, n_l, d, P, win, self.ld[l],
                    dtype=self.dtype, stream=st))
            if n_h > 0:
                halo = win[n_l:]
                self._timed("pull_l%d" % l, lambda: B.history_decompress(
                    slot.remote_codes, slot.remote_off, n_h, None, n_h, d, P, halo, self.ld[l],
                    dtype=self.dtype, stream=st))

    def _push_coded(self, l, w_slot, st):
        """Code the fresh local rows of layer l into the `own` part of the write slot: a sizing
        pass (row offsets), then the codes."""
        n_l, d, P = self.n_local, self.dims[l], self.coded.precision
        slot = self.coded.slots[l][w_slot]
        if n_l == 0:
            return

        def push():
            B.history_compress_plan(self.Hbar[l], self.ld[l], n_l, d, P, slot.own_off, dtype=self.dtype,
                                    workspace=self.ws, workspace_bytes=self.ws_bytes, stream=st)
            B.history_compress_encode(self.Hbar[l], self.ld[l], n_l, d, P, slot.own_off, slot.own_codes,
                                      slot.own_codes.numel(), dtype=self.dtype, stream=st)
        self._timed("push_l%d" % l, push)

    def coded_overflow(self):
        """[(layer, slot, bytes needed, capacity)] of the `own` parts whose last push did not fit
        (empty when all did). Reads the offsets back: synchronises."""
        bad = []
        if self.coded is not None:
            for l in range(1, self.L):
                for s, slot in enumerate(self.coded.slots[l]):
                    need = int(slot.own_off[-1].item())
                    if need > slot.own_codes.numel():
                        bad.append((l, s, need, slot.own_codes.numel()))
        return bad

    # ------------------------------------------------------------ HIP graph
    def graph_period(self):
        """Steps after which the call sequence repeats with the same buffers: the history ring
        comes back to the same slots every tau steps, the predictions to the same cadence
        every predict_every steps, the gradient tables every 2 steps."""
        period = int(np.lcm(self.tau, self.predict_every))
        if self.grad_tables is not None:
            period = int(np.lcm(period, 2))
        return period

    def capture(self):
        """Record graph_period() consecutive steps into one HIP graph (every entry point of the
        library only enqueues kernels on the given stream, so the whole step is capturable) and
        return a function that replays them; each replay advances the step counter by the
        period. For the workloads whose step is bound by launch latency. Must be called with
        self.t a multiple of the period and after at least one eager step (so that nothing is
        loaded lazily during capture); per-call timers are off inside the graph."""
        period = self.graph_period()
        assert not self.predict_ahead, "predictions one step ahead cross the graph's boundary: capture the in-step order"
        assert self.t % period == 0 and self.t > 0, "capture after a whole number of periods, not at t = 0"
        timers, self.timers = self.timers, None
        t0 = self.t
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(period):
                self.forward_backward()
        self.t = t0               # capturing ran nothing
        self.timers = timers

        def replay():
            graph.replay()
            self.t += period
        replay.period = period
        replay.graph = graph
        return replay

    # ------------------------------------------------------------ accounting
    def edges_per_step(self):
        """CSR entries walked by the aggregation calls of one step: nnz per
        forward layer plus the local-local entries per backward layer >= 1 (all
        entries when the halo term of the backward is computed too)."""
        bwd = self.nnz if self.grad_tables is not None else self.nnz_local
        return self.nnz * self.L + bwd * (self.L - 1)
