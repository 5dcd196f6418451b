"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, rejects bad arguments before touching a device, and its host
entry points (partition view) match the oracle bit for bit."""
import os
import re

import numpy as np
import pytest

import sat_synth as syn
from oracle import sat_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sat():
    import paper_2308_13466_amd as pkg
    if not os.path.exists(pkg.lib_path()):
        from paper_2308_13466_amd.build import build_library
        build_library()
    pkg.lib()
    return pkg


def test_header_symbols_are_exported(sat):
    text = open(os.path.join(ROOT, "include", "sat.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(sat_[a-z0-9_]+)\s*\(", text))
    assert len(declared) >= 17
    from paper_2308_13466_amd import binding
    assert declared == set(binding.EXPORTS)
    handle = sat.lib()
    for name in declared:
        assert getattr(handle, name) is not None


def test_status_strings_and_version(sat):
    assert sat.status_string(0) == "SAT_OK"
    for code in (-1, -2, -3, -4, -5):
        assert sat.status_string(code).startswith("SAT_E")
    assert sat.version() >= 100
    assert sat.lib().sat_last_hip_error() == 0


def _check_view(sat, g, m, g_deg=None):
    ref = orc.partition_view(g.N, g.rowptr, g.col, g.part, m, g_deg=g_deg)
    got = sat.partition_view_build(g.N, g.rowptr, g.col, g.part, m, g_deg=g_deg)
    for k in ("n_local", "n_halo", "nnz", "nnz_halo"):
        assert got[k] == ref[k], k
    for k in ("local_ids", "halo_ids", "rowptr", "split", "col", "h_colptr", "h_row"):
        assert got[k].dtype == ref[k].dtype, k
        assert np.array_equal(got[k], ref[k]), k
    for k in ("val", "h_val", "h_self"):
        assert got[k].dtype == np.float32
        assert np.array_equal(got[k].view(np.uint32), ref[k].view(np.uint32)), k
    return got


def test_partition_view_bit_exact_tiny_all_partitions(sat):
    cfg = syn.get_config("tiny")
    ss = syn.substreams(cfg["seed"])
    g = syn.make_graph(cfg, np.random.default_rng(ss["graph"]))
    for m in range(g.n_parts):
        v = _check_view(sat, g, m)
        assert v["n_local"] == 2048


def test_partition_view_bit_exact_power_law(sat):
    rng = np.random.default_rng(7)
    g = syn.chung_lu_planted_graph(20_000, 4, 11.0, 2.1, 0.15, rng)
    _check_view(sat, g, 2)
    deg = (np.diff(g.rowptr) + rng.integers(0, 5, size=g.N)).astype(np.int32)
    _check_view(sat, g, 1, g_deg=deg)


def test_partition_view_degenerate_cases(sat):
    # one partition: no halo at all
    g = syn.ring_graph(50, n_parts=1)
    v = _check_view(sat, g, 0)
    assert v["n_halo"] == 0 and v["nnz_halo"] == 0 and v["nnz"] == 150
    # empty partition id
    v = _check_view(sat, g, 3)
    assert v["n_local"] == 0 and v["nnz"] == 0
    # isolated nodes: rows hold the self-loop only, value 1
    rowptr = np.zeros(6, dtype=np.int64)
    col = np.zeros(0, dtype=np.int32)
    part = np.array([0, 1, 0, 1, 0], dtype=np.int32)
    got = sat.partition_view_build(5, rowptr, col, part, 0)
    assert list(got["col"]) == [0, 1, 2] and np.all(got["val"] == 1.0)
    assert list(got["split"]) == [1, 2, 3]


def test_partition_view_rejects_bad_graphs(sat):
    rowptr = np.array([0, 1, 2], dtype=np.int64)
    part = np.zeros(2, dtype=np.int32)
    for bad_col in ([0, 0], [5, 0], [-1, 0]):     # self-loop, out of range, negative
        with pytest.raises(sat.SatError) as e:
            sat.partition_view_build(2, rowptr, np.array(bad_col, dtype=np.int32), part, 0)
        assert e.value.status == -1
    rowptr = np.array([0, 2, 2, 4], dtype=np.int64)          # unsorted row
    with pytest.raises(sat.SatError):
        sat.partition_view_build(3, rowptr, np.array([2, 1, 0, 1], dtype=np.int32),
                                 np.zeros(3, np.int32), 0)


def test_compute_calls_validate_before_launch(sat):
    # all of these must fail on the host; none may touch a device (none exists here)
    L = sat.lib()
    assert L.sat_history_gather(None, 10, 8, None, 4, 8, None, 8, 0, None) == -1
    assert L.sat_history_gather(None, 10, 8, None, 4, 8, None, 8, 7, None) == -1     # no such dtype
    assert L.sat_history_gather(None, 10, 8, None, 0, 8, None, 8, 0, None) == 0      # empty: no-op
    assert L.sat_history_push(None, 10, 4, None, 4, 8, None, 8, 0, None) == -1
    assert L.sat_history_gather_add(None, 10, 8, None, 4, 8, None, 8, 0, None) == -1
    assert L.sat_history_gather_add(None, 10, 8, None, 0, 8, None, 8, 1, None) == 0  # empty: no-op
    # fake but non-null 16-byte aligned addresses: an ld that breaks the row alignment is
    # refused on the host, before anything could dereference them
    assert L.sat_history_gather_add(4096, 10, 9, 8192, 4, 8, 12288, 8, 0, None) == -3
    assert L.sat_history_gather_add(4096, 10, 8, 8192, 4, 8, 12292, 8, 0, None) == -3
    assert L.sat_dense_fwd(None, 8, 4, 8, 8, None, 8, 1, 0, None, 8, None) == -1
    assert L.sat_dense_fwd(None, 8, 0, 8, 8, None, 8, 7, 0, None, 8, None) == -1     # bad act
    assert L.sat_spmm_fwd(None, None, 8, 8, 0, None, 8, None, 0, None) == -1
    assert L.sat_loss_grad(None, 8, 4, 0, None, 0, None, 8, None, None, 0, None) == -1
    # the entry point with static scratch: same checks, and its size limit, all on the host
    assert L.sat_loss_grad_static(None, 8, 4, 0, None, 0, None, 8, None, None) == -1
    assert L.sat_loss_grad_static(None, 8, 0, 8, None, 0, None, 8, None, None) == 0      # empty: no-op
    assert L.sat_loss_grad_static(4096, 8, sat.loss_grad_static_max_rows() + 1, 8, 8192, 0, 12288, 8,
                                  16384, None) == -2
    assert sat.dense_bwd_workspace_bytes(1000, 64, 32) > 0
    assert sat.predict_workspace_bytes(10, 5, 64, 32, 2) >= 15 * 32 * 4
    assert sat.loss_workspace_bytes(9) >= 4


def test_bench_refuses_more_than_one_gpu():
    """One partition on one GPU is all this library does: the benchmark must say so and exit,
    before it touches a device, when asked for more."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr) and "{" not in r.stdout     # no result line
