"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer: the
partition-view builder (csrc/partition_view.cpp, plain C++, no device) is compiled with
g++ -fsanitize=address,undefined together with a small driver and run on the tiny
workload, a power-law graph with explicit degrees, the degenerate cases and graphs it must
refuse. Any out-of-bounds access, overflow or misaligned access inside the library aborts
the driver; its outputs are also compared bit for bit with the oracle's view."""
import os
import shutil
import struct
import subprocess

import numpy as np
import pytest

import sat_synth as syn
from oracle import sat_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path_factory.mktemp("san") / "view_driver")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan",
           os.path.join(ROOT, "tests", "host", "view_driver.cpp"),
           os.path.join(ROOT, "paper_2308_13466_amd", "csrc", "partition_view.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0 and "static-lib" in r.stderr + " ".join(cmd) and ("cannot find" in r.stderr):
        cmd = [c for c in cmd if not c.startswith("-static-lib")]      # only shared runtimes installed
        r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return exe


def _run(driver, tmp_path, N, rowptr, col, part, m, deg=None):
    rowptr = np.ascontiguousarray(rowptr, np.int64)
    col = np.ascontiguousarray(col, np.int32)
    part = np.ascontiguousarray(part, np.int32)
    fin, fout = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(fin, "wb") as f:
        f.write(struct.pack("<qqii", N, col.size, m, 0 if deg is None else 1))
        f.write(rowptr.tobytes())
        f.write(col.tobytes())
        f.write(part.tobytes())
        if deg is not None:
            f.write(np.ascontiguousarray(deg, np.int32).tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)          # the sanitizer runtime must be the first thing loaded
    r = subprocess.run([driver, fin, fout], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, "sanitizer report or driver failure:\n" + r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    raw = open(fout, "rb").read()
    st_sizes, st_build = struct.unpack_from("<ii", raw, 0)
    n_local, n_halo, nnz, nnz_halo = struct.unpack_from("<qqqq", raw, 8)
    out = dict(st_sizes=st_sizes, st_build=st_build, n_local=n_local, n_halo=n_halo, nnz=nnz, nnz_halo=nnz_halo)
    if st_build == 0:
        pos = 40
        for k, dt, n in (("local_ids", np.int32, n_local), ("halo_ids", np.int32, n_halo),
                         ("rowptr", np.int64, n_local + 1), ("split", np.int64, n_local),
                         ("col", np.int32, nnz), ("val", np.float32, nnz),
                         ("h_colptr", np.int64, n_halo + 1), ("h_row", np.int32, nnz_halo),
                         ("h_val", np.float32, nnz_halo), ("h_self", np.float32, n_halo)):
            out[k] = np.frombuffer(raw, dtype=dt, count=n, offset=pos)
            pos += n * np.dtype(dt).itemsize
        assert pos == len(raw)
    return out


def _same_as_oracle(got, g, m, deg=None):
    ref = orc.partition_view(g.N, g.rowptr, g.col, g.part, m, g_deg=deg)
    assert got["st_sizes"] == 0 and got["st_build"] == 0
    for k in ("n_local", "n_halo", "nnz", "nnz_halo"):
        assert got[k] == ref[k], k
    for k in ("local_ids", "halo_ids", "rowptr", "split", "col", "h_colptr", "h_row"):
        assert np.array_equal(got[k], ref[k]), k
    for k in ("val", "h_val", "h_self"):
        assert np.array_equal(got[k].view(np.uint32), ref[k].view(np.uint32)), k


def test_view_builder_is_clean_on_tiny_and_power_law(driver, tmp_path):
    cfg = syn.get_config("tiny")
    g = syn.make_graph(cfg, np.random.default_rng(syn.substreams(cfg["seed"])["graph"]))
    for m in range(g.n_parts):
        _same_as_oracle(_run(driver, tmp_path, g.N, g.rowptr, g.col, g.part, m), g, m)
    rng = np.random.default_rng(7)
    g = syn.chung_lu_planted_graph(20_000, 4, 11.0, 2.1, 0.15, rng)
    _same_as_oracle(_run(driver, tmp_path, g.N, g.rowptr, g.col, g.part, 2), g, 2)
    deg = (np.diff(g.rowptr) + rng.integers(0, 5, size=g.N)).astype(np.int32)
    _same_as_oracle(_run(driver, tmp_path, g.N, g.rowptr, g.col, g.part, 1, deg=deg), g, 1, deg=deg)


def test_view_builder_is_clean_on_degenerate_and_refused_graphs(driver, tmp_path):
    g = syn.ring_graph(50, n_parts=1)
    _same_as_oracle(_run(driver, tmp_path, g.N, g.rowptr, g.col, g.part, 0), g, 0)     # no halo
    got = _run(driver, tmp_path, g.N, g.rowptr, g.col, g.part, 3)                       # empty partition
    assert got["st_build"] == 0 and got["n_local"] == 0 and got["nnz"] == 0
    # no nodes at all; isolated nodes only
    got = _run(driver, tmp_path, 0, np.zeros(1, np.int64), np.zeros(0, np.int32), np.zeros(0, np.int32), 0)
    assert got["st_build"] == 0 and got["n_local"] == 0
    got = _run(driver, tmp_path, 5, np.zeros(6, np.int64), np.zeros(0, np.int32),
               np.array([0, 1, 0, 1, 0], np.int32), 0)
    assert list(got["col"]) == [0, 1, 2] and np.all(got["val"] == 1.0)
    # refused inputs must be refused without a stray access: self-loop, id out of range, negative
    # id, unsorted row, decreasing row offsets, a row offset past the end of the column array
    rp = np.array([0, 1, 2], np.int64)
    for bad in ([0, 0], [5, 0], [-1, 0]):
        got = _run(driver, tmp_path, 2, rp, np.array(bad, np.int32), np.zeros(2, np.int32), 0)
        assert got["st_sizes"] == -1
    got = _run(driver, tmp_path, 3, np.array([0, 2, 2, 4], np.int64), np.array([2, 1, 0, 1], np.int32),
               np.zeros(3, np.int32), 0)
    assert got["st_sizes"] == -1
    got = _run(driver, tmp_path, 2, np.array([0, 2, 1], np.int64), np.array([1, 0], np.int32),
               np.zeros(2, np.int32), 0)
    assert got["st_sizes"] == -1
