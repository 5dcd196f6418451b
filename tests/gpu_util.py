"""Helpers for the GPU parity tests: device buffers (through torch, which is
only plumbing here), padded layouts, the comparison rule."""
import numpy as np
import torch

import paper_2308_13466_amd as sat

DEV = "cuda:0"


def ld_for(d, mult=32):
    """Leading dimension: d rounded up to a multiple of `mult` floats."""
    return (d + mult - 1) // mult * mult


def to_dev(a, ld=None, pad_value=float("nan")):
    """Host matrix -> device [rows, ld] with NaN (by default) in the padding
    columns, so a kernel that lets padding leak into results is caught."""
    a = np.ascontiguousarray(a)
    if a.ndim == 1 or ld is None or ld == a.shape[1]:
        return torch.from_numpy(a).to(DEV)
    out = np.full((a.shape[0], ld), pad_value, dtype=a.dtype)
    out[:, :a.shape[1]] = a
    return torch.from_numpy(out).to(DEV)


def dev_empty(rows, ld, fill=float("nan")):
    return torch.full((rows, ld), fill, dtype=torch.float32, device=DEV)


def to_host(t, d=None):
    a = t.detach().cpu().numpy()
    return a if d is None else a[:, :d]


def upload_view(v):
    """dict from partition_view_build (or the oracle) -> sat.PartView on device."""
    t = {k: torch.from_numpy(np.ascontiguousarray(v[k])).to(DEV)
         for k in ("rowptr", "split", "col", "val", "h_colptr", "h_row", "h_val", "h_self")}
    return sat.PartView(v["n_local"], v["n_halo"], v["nnz"], v["nnz_halo"], **t)


def workspace(nbytes):
    n = max(int(nbytes), 256)
    return torch.empty((n + 3) // 4, dtype=torch.float32, device=DEV)


def stream_ptr():
    return torch.cuda.current_stream().cuda_stream


def sync():
    torch.cuda.synchronize()


def assert_close(got, ref, rtol, what="", max_bad_rows=0):
    """|got - ref| <= rtol * (|ref| + rms(ref)) element-wise.

    max_bad_rows > 0 lets that many rows hold elements outside the bound (used
    only where a valid 0/1 decision upstream may differ between the two sides).

    A pure element-wise relative bound cannot hold for sums that nearly cancel;
    the rms of the reference matrix is the magnitude the rounding error of one
    accumulated element actually scales with.
    """
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    if ref.size == 0:
        return
    assert np.all(np.isfinite(got)), "%s: non-finite values in result" % what
    rms = np.sqrt(np.mean(ref * ref))
    err = np.abs(got - ref)
    bound = rtol * (np.abs(ref) + rms)
    bad = err > bound
    if max_bad_rows and bad.any() and bad.ndim == 2:
        n_rows_bad = int(bad.any(axis=1).sum())
        if n_rows_bad <= max_bad_rows:
            return
        what = "%s [%d rows outside, %d allowed]" % (what, n_rows_bad, max_bad_rows)
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError("%s: %d of %d elements outside rtol=%g; worst at %s: got %r ref %r (rms %g)"
                             % (what, int(bad.sum()), ref.size, rtol, i, got[i], ref[i], rms))


def normwise(got, ref):
    ref = np.asarray(ref, np.float64)
    return float(np.linalg.norm(np.asarray(got, np.float64) - ref) / max(np.linalg.norm(ref), 1e-300))


def to_dev_bits(bits, ld=None, pad_bits=0x7FC0):
    """uint16 bf16 patterns [rows, d] -> device uint16 tensor [rows, ld]; padding
    columns hold a NaN pattern by default."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if ld is None or ld == bits.shape[1]:
        return torch.from_numpy(bits.view(np.int16)).to(DEV)
    out = np.full((bits.shape[0], ld), pad_bits, dtype=np.uint16)
    out[:, :bits.shape[1]] = bits
    return torch.from_numpy(out.view(np.int16)).to(DEV)


def bits_to_host(t, d=None):
    a = t.detach().cpu().numpy().view(np.uint16)
    return a if d is None else a[:, :d]
