"""Seeded random graphs with a contiguous partition vector.

Every generator returns a simple undirected graph (symmetric CSR, no
self-loops, no multi-edges, columns ascending inside each row) plus a
partition vector made of contiguous id ranges. Self-loops and the
normalisation of the propagation matrix belong to the method and are added by
whoever consumes the graph, not here.
"""
from dataclasses import dataclass

import numpy as np
import scipy.sparse as sp


@dataclass
class Graph:
    N: int
    rowptr: np.ndarray    # int64 [N+1]
    col: np.ndarray       # int32 [nnz], ascending within a row, no self-loops
    part: np.ndarray      # int32 [N], partition id of every node
    n_parts: int
    deg: np.ndarray = None  # int32 [N] neighbour count of every node, when rowptr does not
                            # hold every node's row (see chung_lu_partition_rows)

    @property
    def nnz(self):
        return int(self.rowptr[-1])

    def degrees(self):
        return np.diff(self.rowptr).astype(np.int64)


def _csr_from_pairs(N, u, v):
    """Symmetrise, drop loops, dedup; return (rowptr int64, col int32)."""
    keep = u != v
    u = u[keep].astype(np.int32, copy=False)
    v = v[keep].astype(np.int32, copy=False)
    rows = np.concatenate([u, v])
    cols = np.concatenate([v, u])
    del u, v
    data = np.ones(rows.shape[0], dtype=np.int8)
    m = sp.coo_matrix((data, (rows, cols)), shape=(N, N)).tocsr()
    del rows, cols, data
    m.sum_duplicates()
    m.sort_indices()
    return m.indptr.astype(np.int64), m.indices.astype(np.int32)


def _contiguous_parts(N, n_parts):
    """part[i] for n_parts contiguous ranges whose sizes differ by at most one."""
    bounds = (np.arange(n_parts + 1, dtype=np.int64) * N) // n_parts
    part = np.empty(N, dtype=np.int32)
    for p in range(n_parts):
        part[bounds[p]:bounds[p + 1]] = p
    return part, bounds


def ring_graph(N, n_parts=2):
    """Cycle on N nodes: every node has exactly two neighbours (2-regular)."""
    i = np.arange(N, dtype=np.int64)
    rowptr, col = _csr_from_pairs(N, i, (i + 1) % N)
    part, _ = _contiguous_parts(N, n_parts)
    return Graph(N, rowptr, col, part, n_parts)


def sbm_graph(N, n_comm, n_parts, intra_deg, cross_deg, rng):
    """Stochastic block model with n_comm equal contiguous communities.

    intra_deg / cross_deg are the expected numbers of neighbours a node has
    inside / outside its own community. Edges are drawn as uniformly random
    endpoint pairs (with replacement, then deduplicated), which is the sparse
    limit of independent Bernoulli pairs. Partitions are contiguous groups of
    whole communities.
    """
    cb = (np.arange(n_comm + 1, dtype=np.int64) * N) // n_comm
    csize = np.diff(cb)
    comm_of = np.repeat(np.arange(n_comm), csize)

    n_in = rng.poisson(N * intra_deg / 2.0)
    u = rng.integers(0, N, size=n_in, dtype=np.int64)
    cu = comm_of[u]
    v = cb[cu] + (rng.random(n_in) * csize[cu]).astype(np.int64)
    us, vs = [u], [v]

    n_out = rng.poisson(N * cross_deg / 2.0)
    u = rng.integers(0, N, size=n_out, dtype=np.int64)
    cu = comm_of[u]
    # uniform over the nodes outside u's community: draw in [0, N - size) and
    # jump over the community's id range
    r = (rng.random(n_out) * (N - csize[cu])).astype(np.int64)
    v = np.where(r >= cb[cu], r + csize[cu], r)
    us.append(u)
    vs.append(v)

    rowptr, col = _csr_from_pairs(N, np.concatenate(us), np.concatenate(vs))
    # partitions: contiguous groups of communities
    pb = (np.arange(n_parts + 1, dtype=np.int64) * n_comm) // n_parts
    part = np.empty(N, dtype=np.int32)
    for p in range(n_parts):
        part[cb[pb[p]]:cb[pb[p + 1]]] = p
    return Graph(N, rowptr, col, part, n_parts)


def _powerlaw_weights(N, mean_deg, gamma, rng):
    """Expected degrees w_i ~ rank^(-1/(gamma-1)), mean mean_deg, capped at
    sqrt(sum w) so that w_i w_j / sum w <= 1, then shuffled over node ids."""
    i0 = 1.0
    w = (np.arange(N, dtype=np.float64) + i0) ** (-1.0 / (gamma - 1.0))
    w *= mean_deg * N / w.sum()
    for _ in range(8):
        cap = np.sqrt(w.sum())
        if w.max() <= cap:
            break
        w = np.minimum(w, cap)
        w *= mean_deg * N / w.sum()
    w = np.minimum(w, np.sqrt(w.sum()))
    rng.shuffle(w)
    return w


def _draw_weighted(lo, hi, w, count, rng):
    """count ids in [lo, hi) drawn i.i.d. with probability ~ w, random order."""
    p = w[lo:hi] / w[lo:hi].sum()
    cnt = rng.multinomial(count, p)
    ids = np.repeat(np.arange(lo, hi, dtype=np.int64), cnt)
    rng.shuffle(ids)
    return ids


def chung_lu_planted_graph(N, n_parts, mean_deg, gamma, cut, rng):
    """Power-law (Chung-Lu) graph with planted contiguous partitions.

    N*mean_deg/2 undirected edges are drawn: the first endpoint ~ w over all
    nodes; with probability 1-cut the second endpoint ~ w inside the first
    endpoint's partition, else ~ w outside it. Loops and duplicates are
    dropped afterwards, so realised degrees fall slightly short of w.
    """
    part, pb = _contiguous_parts(N, n_parts)
    w = _powerlaw_weights(N, mean_deg, gamma, rng)
    E = int(round(N * mean_deg / 2.0))
    W_part = np.array([w[pb[p]:pb[p + 1]].sum() for p in range(n_parts)])
    e_part = rng.multinomial(E, W_part / W_part.sum())
    us, vs = [], []
    for p in range(n_parts):
        lo, hi = int(pb[p]), int(pb[p + 1])
        e_p = int(e_part[p])
        u = _draw_weighted(lo, hi, w, e_p, rng)
        n_cut = int(rng.binomial(e_p, cut)) if n_parts > 1 else 0
        v_in = _draw_weighted(lo, hi, w, e_p - n_cut, rng)
        if n_cut:
            # ~ w over the ids outside [lo, hi): draw on the concatenation
            w_out = np.concatenate([w[:lo], w[hi:]])
            r = _draw_weighted(0, N - (hi - lo), w_out, n_cut, rng)
            v_out = np.where(r >= lo, r + (hi - lo), r)
            v = np.concatenate([v_in, v_out])
        else:
            v = v_in
        us.append(u)
        vs.append(v)
    rowptr, col = _csr_from_pairs(N, np.concatenate(us), np.concatenate(vs))
    return Graph(N, rowptr, col, part, n_parts)


def chung_lu_partition_rows(N, n_parts, mean_deg, gamma, cut, rng):
    """Rows of partition 0 only of a planted-partition power-law graph on N nodes.

    For graphs whose other partitions nobody can afford to draw. Partition 0 is
    the id range [0, N // n_parts). Its nodes get n_l * mean_deg * (1 - cut) / 2
    undirected local-local edges (both endpoints ~ w inside the partition, so
    the local block is symmetric) and n_l * mean_deg * cut cross entries (local
    endpoint ~ w inside, outside endpoint ~ w over the other ids); loops and
    duplicates are dropped. Rows of nodes outside the partition are left empty.
    `deg` holds every node's neighbour count: the realised row length for the
    partition's nodes; for an outside node the larger of its rounded expected
    degree w and the number of entries it received from the partition.
    """
    part, pb = _contiguous_parts(N, n_parts)
    n_l = int(pb[1])
    w = _powerlaw_weights(N, mean_deg, gamma, rng)
    n_ll = int(round(n_l * mean_deg * (1.0 - cut) / 2.0))
    n_x = int(round(n_l * mean_deg * cut)) if n_parts > 1 else 0
    u = _draw_weighted(0, n_l, w, n_ll, rng).astype(np.int32)
    v = _draw_weighted(0, n_l, w, n_ll, rng).astype(np.int32)
    keep = u != v
    u, v = u[keep], v[keep]
    xu = _draw_weighted(0, n_l, w, n_x, rng).astype(np.int32)
    xv = _draw_weighted(n_l, N, w, n_x, rng).astype(np.int32)
    rows = np.concatenate([u, v, xu])
    cols = np.concatenate([v, u, xv])
    del u, v, xu
    m = sp.coo_matrix((np.ones(rows.shape[0], dtype=np.int8), (rows, cols)), shape=(n_l, N)).tocsr()
    del rows, cols
    m.sum_duplicates()
    m.sort_indices()
    rowptr = np.full(N + 1, m.indptr[-1], dtype=np.int64)
    rowptr[:n_l + 1] = m.indptr
    col = m.indices.astype(np.int32)
    deg = np.rint(w).astype(np.int32)
    deg[:n_l] = np.diff(m.indptr)
    got = np.bincount(xv, minlength=N).astype(np.int32)   # upper bound on distinct entries received
    np.maximum(deg[n_l:], got[n_l:], out=deg[n_l:])
    np.maximum(deg[n_l:], 1, out=deg[n_l:])
    return Graph(N, rowptr, col, part, n_parts, deg)


def make_graph(cfg, rng):
    """Graph for one entry of configs.CONFIGS."""
    if cfg["kind"] == "sbm":
        if "intra_deg" in cfg:
            intra, cross = cfg["intra_deg"], cfg["cross_deg"]
        else:
            # choose intra/cross-community degrees so that a fraction `cut`
            # of a partition's entries leaves the partition: cross-community
            # neighbours are uniform over the other communities, of which a
            # share (n_comm - n_comm/n_parts)/(n_comm - 1) lies outside it
            nc, npar = cfg["n_comm"], cfg["n_parts"]
            share = (nc - nc / npar) / (nc - 1.0)
            cross = cfg["cut"] * cfg["mean_deg"] / share
            intra = cfg["mean_deg"] - cross
        return sbm_graph(cfg["N"], cfg["n_comm"], cfg["n_parts"], intra, cross, rng)
    if cfg["kind"] == "chung_lu_rows":
        return chung_lu_partition_rows(cfg["N"], cfg["n_parts"], cfg["mean_deg"], cfg["gamma"],
                                       cfg["cut"], rng)
    if cfg["kind"] == "chung_lu":
        return chung_lu_planted_graph(cfg["N"], cfg["n_parts"], cfg["mean_deg"],
                                      cfg["gamma"], cfg["cut"], rng)
    raise ValueError(cfg["kind"])


def cached_graph(cfg, seed_seq, cache_dir=None):
    """make_graph with an on-disk cache (a pure function of cfg and seed).

    Large graphs take about a minute to draw; the cache lets the tests and
    the benchmark of one machine share the result. Set SAT_SYNTH_CACHE to
    move it, or to the empty string to switch it off.
    """
    import hashlib
    import json
    import os
    if cache_dir is None:
        cache_dir = os.environ.get("SAT_SYNTH_CACHE", "/tmp/sat_synth_cache")
    keys = {k: cfg[k] for k in sorted(cfg) if k in (
        "kind", "N", "n_comm", "n_parts", "intra_deg", "cross_deg", "mean_deg",
        "gamma", "cut")}
    keys["entropy"] = [int(x) for x in np.atleast_1d(seed_seq.entropy)]
    keys["spawn_key"] = [int(x) for x in seed_seq.spawn_key]
    tag = hashlib.sha256(json.dumps(keys, sort_keys=True).encode()).hexdigest()[:20]
    path = os.path.join(cache_dir, "graph_%s.npz" % tag) if cache_dir else None
    if path and os.path.exists(path):
        try:
            z = np.load(path)
            return Graph(int(z["N"]), z["rowptr"], z["col"], z["part"], int(z["n_parts"]),
                         z["deg"] if "deg" in z.files else None)
        except Exception:
            pass
    g = make_graph(cfg, np.random.Generator(np.random.PCG64(seed_seq)))
    if path and g.nnz > 5_000_000:
        try:
            os.makedirs(cache_dir, exist_ok=True)
            tmp = path + ".%d.tmp.npz" % os.getpid()
            extra = {} if g.deg is None else {"deg": g.deg}
            np.savez(tmp, N=g.N, rowptr=g.rowptr, col=g.col, part=g.part, n_parts=g.n_parts, **extra)
            os.replace(tmp, path)
        except OSError:
            pass
    return g
