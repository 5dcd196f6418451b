"""One partition's SAT training step with a graph attention backbone, as a
sequence of libsat calls. Orchestration only, like step.py: buffers are torch
tensors used as plain memory, no arithmetic happens here.

Per layer l (Hbar_l = local rows, then the halo rows - static features for l = 0,
predicted embeddings for l >= 1, exactly as in the GCN step):
  forward   Z_l = Hbar_l W_l over all local + halo rows     sat_dense_fwd
            el, er                                           sat_gat_scores
            H_{l+1} = act(edge softmax aggregation of Z_l)   sat_gat_aggregate_fwd
            push H_{l+1} into the history ring               sat_history_push
  backward  dZ_l, da_dst_l, da_src_l                          sat_gat_aggregate_bwd
            dW_l = Hbar_l^T dZ_l over all rows                sat_dense_bwd (dAGG = NULL)
            dH_l = dZ_l[local rows] W_l^T for l >= 1          sat_dense_bwd (dW = NULL)
The halo rows are constants of the step: no gradient flows into them. With gradient
tables (the stale-gradient term of the appendix's SAT backward) the gradient FOR them,
dZ_l[halo rows] W_l^T, is formed as well and pushed into the write table at the halo
nodes' rows, and the read table's rows of the local nodes are added to dH_l.
"""
import torch

from . import binding as B
from .step import PartitionStep


class GatPartitionStep(PartitionStep):
    """attn[l] = (a_dst, a_src, heads): device fp32 vectors [heads * d_head] of layer l,
    d_head = dims[l + 1] / heads. Everything else as PartitionStep (gradient tables, the coded
    ring and its decoding a range of rows at a time, kept input projections included)."""

    def __init__(self, view, dims, X_table, hist, table_ids, Ws, attn, predictors, y, tau,
                 slope=0.2, timers=None, dtype=B.F32, predict_every=1, grad_tables=None, coded=None,
                 coded_chunk_rows=None, projection_cache=False):
        super().__init__(view, dims, X_table, hist, table_ids, Ws, predictors, y, tau,
                         fused_pull=True, timers=timers, dtype=dtype, grad_tables=grad_tables,
                         predict_every=predict_every, coded=coded, coded_chunk_rows=coded_chunk_rows,
                         projection_cache=projection_cache)
        dev = X_table.device
        self.attn = attn
        self.slope = float(slope)
        self.heads = [a[2] for a in attn]
        self.d_head = [dims[l + 1] // self.heads[l] for l in range(self.L)]
        for l in range(self.L):
            assert self.heads[l] * self.d_head[l] == dims[l + 1]
        f32 = dict(dtype=torch.float32, device=dev)
        act = dict(dtype=torch.bfloat16 if dtype == B.BF16 else torch.float32, device=dev)
        L, n_l, n_bar = self.L, self.n_local, self.n_bar
        self.AGG = None          # the GCN step's aggregates are not used
        self.dAGG = None
        self.Z = [torch.zeros((n_bar, self.ld[l + 1]), **act) for l in range(L)]
        # dZ_l lives only between the two backward calls of layer l: one buffer for all layers
        ld_max = max(self.ld[1:])
        self._dZ_buf = torch.zeros(n_bar * ld_max, **act)
        self.dZ = [self._dZ_buf[:n_bar * self.ld[l + 1]].view(n_bar, self.ld[l + 1]) for l in range(L)]
        self.el = [torch.zeros((n_l, self.heads[l]), **f32) for l in range(L)]
        self.er = [torch.zeros((n_bar, self.heads[l]), **f32) for l in range(L)]
        self.stats = [torch.zeros((n_l, self.heads[l], 2), **f32) for l in range(L)]
        self.da_dst = [torch.zeros(dims[l + 1], **f32) for l in range(L)]
        self.da_src = [torch.zeros(dims[l + 1], **f32) for l in range(L)]
        need = [self.ws_bytes]
        for l in range(L):
            need.append(B.dense_bwd_workspace_bytes(n_bar, dims[l], dims[l + 1]))
            need.append(B.gat_aggregate_bwd_workspace_bytes(n_l, self.n_halo, self.heads[l],
                                                            self.d_head[l], dtype))
        self.ws_bytes = max(need)
        self.ws = torch.empty((self.ws_bytes + 3) // 4, **f32)

    def forward_backward(self):
        L, dims, ld, n_l, n_h, n_bar = self.L, self.dims, self.ld, self.n_local, self.n_halo, self.n_bar
        st = self._stream()
        dt = self.dtype
        order = self.slot_order()
        for l in range(1, L if self.t % self.predict_every == 0 else 1):
            if self.coded is not None:      # the window decoded from the codes
                self._predict_coded(l, order, self.ws, st)
                continue
            self._timed("predict_l%d" % l, lambda: self._predict_in_place(l, order, self.ws, st))
        w_slot = self.t % self.tau
        for l in range(L):
            if l == 0 and n_h > 0:
                halo0 = self.Hbar[0][n_l:]
                self._timed("gather_l0", lambda: B.history_gather(
                    self.X_table, self.X_table.shape[0], self.X_table.shape[1],
                    self.halo_table_ids, n_h, dims[0], halo0, ld[0], dtype=dt, stream=st))
            K, F = self.heads[l], self.d_head[l]
            a_dst, a_src, _ = self.attn[l]
            self._timed("dense_fwd_l%d" % l, lambda: B.dense_fwd(
                self.Hbar[l], ld[l], n_bar, dims[l], dims[l + 1], self.Ws[l], self.ld_w[l],
                B.ACT_IDENTITY, self.Z[l], ld[l + 1], dtype=dt, stream=st))
            self._timed("gat_scores_l%d" % l, lambda: B.gat_scores(
                self.Z[l], ld[l + 1], n_bar, n_l, K, F, a_dst, a_src, self.el[l], self.er[l],
                dtype=dt, stream=st))
            last = l == L - 1
            out = self.logits if last else self.Hbar[l + 1]
            self._timed("gat_fwd_l%d" % l, lambda: B.gat_aggregate_fwd(
                self.pv, self.Z[l], ld[l + 1], K, F, self.el[l], self.er[l], self.slope,
                B.ACT_IDENTITY if last else B.ACT_RELU, out, ld[l + 1], self.stats[l], dtype=dt,
                stream=st))
            if not last and self.coded is not None:
                self._push_coded(l + 1, w_slot, st)
            elif not last:
                tab = self.hist[l + 1][w_slot]
                if self.proj is not None:
                    self._proj_valid[l + 1][w_slot] = False      # the slot's rows change
                self._timed("push_l%d" % (l + 1), lambda: B.history_push(
                    tab, tab.shape[0], tab.shape[1], self.local_table_ids, n_l, dims[l + 1],
                    self.Hbar[l + 1], ld[l + 1], dtype=dt, stream=st))
        self._timed("loss_grad", lambda: B.loss_grad(
            self.logits, ld[L], n_l, dims[L], self.y, self.dH[L], ld[L], loss=self.loss, dtype=dt,
            workspace=self.ws, workspace_bytes=self.ws_bytes, stream=st))
        for l in range(L - 1, -1, -1):
            last = l == L - 1
            K, F = self.heads[l], self.d_head[l]
            a_dst, a_src, _ = self.attn[l]
            hout = None if last else self.Hbar[l + 1]
            self._timed("gat_bwd_l%d" % l, lambda: B.gat_aggregate_bwd(
                self.pv, self.Z[l], ld[l + 1], K, F, self.el[l], self.er[l], self.stats[l],
                self.slope, B.ACT_IDENTITY if last else B.ACT_RELU, self.dH[l + 1], ld[l + 1],
                hout, 0 if last else ld[l + 1], a_dst, a_src, self.dZ[l], ld[l + 1],
                self.da_dst[l], self.da_src[l], dtype=dt, workspace=self.ws,
                workspace_bytes=self.ws_bytes, stream=st))
            self._timed("dense_bwd_l%d" % l, lambda: B.dense_bwd(
                self.dZ[l], ld[l + 1], None, 0, self.Hbar[l], ld[l], self.Ws[l], self.ld_w[l], n_bar,
                dims[l], dims[l + 1], B.ACT_IDENTITY, self.dW[l], self.ld_dw[l], None, 0, dtype=dt,
                workspace=self.ws, workspace_bytes=self.ws_bytes, stream=st))
            if l >= 1:
                self._timed("dense_bwd_in_l%d" % l, lambda: B.dense_bwd(
                    self.dZ[l], ld[l + 1], None, 0, None, 0, self.Ws[l], self.ld_w[l], n_l,
                    dims[l], dims[l + 1], B.ACT_IDENTITY, None, 0, self.dH[l], ld[l], dtype=dt,
                    workspace=self.ws, workspace_bytes=self.ws_bytes, stream=st))
                if self.grad_tables is not None:
                    rd, wr = self.grad_tables[l][self.t % 2], self.grad_tables[l][(self.t + 1) % 2]
                    if n_h > 0:
                        dz_halo = self.dZ[l][n_l:]
                        self._timed("dense_bwd_halo_l%d" % l, lambda: B.dense_bwd(
                            dz_halo, ld[l + 1], None, 0, None, 0, self.Ws[l], self.ld_w[l], n_h,
                            dims[l], dims[l + 1], B.ACT_IDENTITY, None, 0, self.dH_halo[l], ld[l], dtype=dt,
                            workspace=self.ws, workspace_bytes=self.ws_bytes, stream=st))
                        self._timed("grad_push_l%d" % l, lambda: B.history_push(
                            wr, wr.shape[0], wr.shape[1], self.halo_table_ids, n_h, dims[l],
                            self.dH_halo[l], ld[l], dtype=dt, stream=st))
                    self._timed("grad_pull_l%d" % l, lambda: B.history_gather_add(
                        rd, rd.shape[0], rd.shape[1], self.local_table_ids, n_l, dims[l],
                        self.dH[l], ld[l], dtype=dt, stream=st))
        self.t += 1

    def edges_per_step(self):
        """Entries walked by the edge kernels of one step: per layer the forward
        aggregation, the destination-side and the source-side backward pass, each
        over all nnz entries of the view."""
        return 3 * self.nnz * self.L
