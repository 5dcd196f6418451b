"""Mini-batches of the predictor's training (Eq. 12): instead of weighting all local nodes
with 0/1 (every node's LSTM still runs), the batch's nodes and their 1-hop neighbourhood are
cut out as a view of their own, so the work of sat_predictor_grad falls with the batch.

The compact view is a partition view like any other and comes from the library's own host
call: the batch B (a subset of partition m's local nodes) is "partition 0" of a two-way split
of the graph, everything else is "partition 1". Its local rows are B (ascending global id), its
halo is every neighbour of B outside B - other local nodes of m and true halo nodes alike -
and the stored values are the same A_hat entries (global degrees). The predictor is supervised
on B: pred[v] = newest[v] + (row v of [P_in | P_out] . S) Wg only needs S of v's neighbours,
and S of a node depends on that node's own window alone, so loss and gradients are exactly
those of the 0/1-weighted call, summed in another order.

Orchestration only: no arithmetic happens here.
"""
import numpy as np

from . import binding as B


def minibatch_view(N, g_rowptr, g_col, part, m, batch, g_deg=None):
    """batch: global ids of nodes of partition m (distinct). Returns (view, node_ids): the
    compact view (dict of host arrays, layout of sat_part_view) and the global id of each of
    its local-then-halo nodes (int32 [n_bar]), i.e. the table rows when tables are indexed by
    global id. g_deg: neighbour count of every node; None = the row lengths of the CSR (then
    the CSR must hold every node's row, not just the partition's)."""
    part = np.asarray(part)
    batch = np.unique(np.asarray(batch, dtype=np.int64))
    if batch.size and (batch[0] < 0 or batch[-1] >= N or np.any(part[batch] != m)):
        raise ValueError("a mini-batch holds local nodes of partition %d only" % m)
    split = np.ones(N, dtype=np.int32)
    split[batch] = 0
    if g_deg is None:
        g_deg = np.diff(np.asarray(g_rowptr, dtype=np.int64)).astype(np.int32)
    view = B.partition_view_build(N, g_rowptr, g_col, split, 0, g_deg=g_deg)
    node_ids = np.concatenate([view["local_ids"], view["halo_ids"]]).astype(np.int32)
    return view, node_ids
