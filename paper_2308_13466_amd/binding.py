"""ctypes binding of libsat.so: same names as the C ABI minus the sat_ prefix.

Argument marshalling only. Tensor-like arguments may be anything with a
data_ptr() method (torch tensors), an int address, or None. Leading dimensions
are passed explicitly, exactly as in the C header. If libsat.so has not been
built this module raises on first use: there is no fallback path.
"""
import ctypes as C
import os

import numpy as np

F32, BF16 = 0, 1
ACT_IDENTITY, ACT_RELU = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class SatError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s" % (where, status_string(status)))


def lib_path():
    return os.path.join(_HERE, "libsat.so")


class _PartViewC(C.Structure):
    _fields_ = [("n_local", C.c_int64), ("n_halo", C.c_int64), ("nnz", C.c_int64),
                ("nnz_halo", C.c_int64), ("rowptr", C.c_void_p), ("split", C.c_void_p),
                ("col", C.c_void_p), ("val", C.c_void_p), ("h_colptr", C.c_void_p),
                ("h_row", C.c_void_p), ("h_val", C.c_void_p), ("h_self", C.c_void_p)]


class _PredictorC(C.Structure):
    _fields_ = [("Wx", C.c_void_p), ("Wh", C.c_void_p), ("b", C.c_void_p), ("Wg", C.c_void_p),
                ("d", C.c_int32), ("d_s", C.c_int32), ("tau", C.c_int32), ("bypass", C.c_int32)]


_i32, _i64, _vp = C.c_int32, C.c_int64, C.c_void_p
_SIGNATURES = {
    "sat_status_string": (C.c_char_p, [_i32]),
    "sat_last_hip_error": (_i32, []),
    "sat_version": (_i32, []),
    "sat_partition_view_sizes": (_i32, [_i64, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp]),
    "sat_partition_view_build": (_i32, [_i64, _vp, _vp, _vp, _vp, _i32] + [_vp] * 10),
    "sat_history_gather": (_i32, [_vp, _i64, _i64, _vp, _i64, _i32, _vp, _i64, _i32, _vp]),
    "sat_history_gather_add": (_i32, [_vp, _i64, _i64, _vp, _i64, _i32, _vp, _i64, _i32, _vp]),
    "sat_history_compress_workspace_bytes": (_i64, [_i64]),
    "sat_history_compress_plan": (_i32, [_vp, _i64, _i64, _i32, _i32, _i32, _vp, _vp, _i64, _vp]),
    "sat_history_compress_encode": (_i32, [_vp, _i64, _i64, _i32, _i32, _i32, _vp, _vp, _i64, _vp]),
    "sat_history_decompress": (_i32, [_vp, _vp, _i64, _vp, _i64, _i32, _i32, _i32, _vp, _i64, _vp]),
    "sat_history_push": (_i32, [_vp, _i64, _i64, _vp, _i64, _i32, _vp, _i64, _i32, _vp]),
    "sat_predict_workspace_bytes": (_i64, [_i64, _i64, _i32, _i32, _i32]),
    "sat_predict": (_i32, [_vp, _vp, _vp, _i64, _i64, _vp, _vp, _i64, _i32, _vp, _i64, _vp]),
    "sat_predict_states_workspace_bytes": (_i64, [_i32, _i32]),
    "sat_predict_states": (_i32, [_vp, _vp, _i64, _i64, _vp, _i64, _i32, _vp, _vp, _i64, _vp]),
    "sat_predict_hop_workspace_bytes": (_i64, [_i64, _i32]),
    "sat_predict_hop": (_i32, [_vp, _vp, _vp, _vp, _i64, _i64, _vp, _vp, _i64, _i32, _vp, _i64, _vp]),
    "sat_predict_cached": (_i32, [_vp, _vp, _vp, _i64, _i64, _vp, _vp, _i64, _i32, _vp, _i32, _vp, _i64,
                                  _vp]),
    "sat_predictor_train_workspace_bytes": (_i64, [_i64, _i64, _i32, _i32, _i32]),
    "sat_predictor_grad": (_i32, [_vp, _vp, _vp, _i64, _i64, _vp, _vp, _i64, _vp, _i32, _vp, _vp,
                                  _vp, _vp, _vp, _vp, _i64, _vp]),
    "sat_sgd_update": (_i32, [_vp, _vp, _i64, C.c_float, _vp]),
    "sat_spmm_workspace_bytes": (_i64, [_vp, _i32]),
    "sat_spmm_fwd": (_i32, [_vp, _vp, _i64, _i32, _i32, _vp, _i64, _vp, _i64, _vp]),
    "sat_spmm_bwd": (_i32, [_vp, _vp, _i64, _i32, _i32, _vp, _i64, _vp, _i64, _vp, _i64, _vp]),
    "sat_dense_fwd": (_i32, [_vp, _i64, _i64, _i32, _i32, _vp, _i64, _i32, _i32, _vp, _i64, _vp]),
    "sat_dense_bwd_workspace_bytes": (_i64, [_i64, _i32, _i32]),
    "sat_dense_bwd": (_i32, [_vp, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _i64, _i32, _i32, _i32,
                             _i32, _vp, _i64, _vp, _i64, _vp, _i64, _vp]),
    "sat_gat_scores": (_i32, [_vp, _i64, _i64, _i64, _i32, _i32, _vp, _vp, _i32, _vp, _vp, _vp]),
    "sat_gat_aggregate_fwd": (_i32, [_vp, _vp, _i64, _i32, _i32, _i32, _vp, _vp, C.c_float, _i32,
                                     _vp, _i64, _vp, _vp]),
    "sat_gat_aggregate_bwd_workspace_bytes": (_i64, [_i64, _i64, _i32, _i32, _i32]),
    "sat_gat_aggregate_bwd": (_i32, [_vp, _vp, _i64, _i32, _i32, _i32, _vp, _vp, _vp, C.c_float,
                                     _i32, _vp, _i64, _vp, _i64, _vp, _vp, _vp, _i64, _vp, _vp,
                                     _vp, _i64, _vp]),
    "sat_loss_workspace_bytes": (_i64, [_i64]),
    "sat_loss_grad": (_i32, [_vp, _i64, _i64, _i32, _vp, _i32, _vp, _i64, _vp, _vp, _i64, _vp]),
    "sat_loss_grad_static_max_rows": (_i64, []),
    "sat_loss_grad_static": (_i32, [_vp, _i64, _i64, _i32, _vp, _i32, _vp, _i64, _vp, _vp]),
}
EXPORTS = tuple(sorted(_SIGNATURES))


def lib():
    """The loaded library. Raises if libsat.so is missing or lacks a symbol."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(
                "libsat.so not built (%s); run __graft_entry__.build() or "
                "python paper_2308_13466_amd/build.py" % path)
        handle = C.CDLL(path)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)      # AttributeError if not exported
            fn.restype = res
            fn.argtypes = args
        _LIB = handle
    return _LIB


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    return x.data_ptr()


def _check(status, where):
    if status != 0:
        raise SatError(status, where)


def status_string(status):
    return lib().sat_status_string(int(status)).decode()


def version():
    return lib().sat_version()


class PartView:
    """Device-side sat_part_view. Keeps the tensors it points to alive."""

    def __init__(self, n_local, n_halo, nnz, nnz_halo, rowptr, split, col, val,
                 h_colptr, h_row, h_val, h_self):
        self.tensors = dict(rowptr=rowptr, split=split, col=col, val=val, h_colptr=h_colptr,
                            h_row=h_row, h_val=h_val, h_self=h_self)
        self.n_local, self.n_halo, self.nnz, self.nnz_halo = n_local, n_halo, nnz, nnz_halo
        self.c = _PartViewC(n_local, n_halo, nnz, nnz_halo, _ptr(rowptr), _ptr(split), _ptr(col),
                            _ptr(val), _ptr(h_colptr), _ptr(h_row), _ptr(h_val), _ptr(h_self))

    @property
    def ref(self):
        return C.addressof(self.c)


class Predictor:
    """Device-side sat_predictor (one hidden layer's omega)."""

    def __init__(self, Wx, Wh, b, Wg, d, d_s, tau, bypass=False):
        self.tensors = (Wx, Wh, b, Wg)
        self.d, self.d_s, self.tau, self.bypass = d, d_s, tau, bool(bypass)
        self.c = _PredictorC(_ptr(Wx), _ptr(Wh), _ptr(b), _ptr(Wg), d, d_s, tau, int(bool(bypass)))

    @property
    def ref(self):
        return C.addressof(self.c)


def partition_view_build(N, g_rowptr, g_col, part, m, g_deg=None):
    """Host call. numpy in, dict of numpy arrays out (layout: sat_part_view)."""
    L = lib()
    g_rowptr = np.ascontiguousarray(g_rowptr, dtype=np.int64)
    g_col = np.ascontiguousarray(g_col, dtype=np.int32)
    part = np.ascontiguousarray(part, dtype=np.int32)
    if g_deg is not None:
        g_deg = np.ascontiguousarray(g_deg, dtype=np.int32)
    sizes = [C.c_int64(0) for _ in range(4)]
    _check(L.sat_partition_view_sizes(N, _ptr(g_rowptr), _ptr(g_col), _ptr(part), m,
                                      *[C.addressof(s) for s in sizes]),
           "sat_partition_view_sizes")
    n_local, n_halo, nnz, nnz_halo = [s.value for s in sizes]
    out = dict(n_local=n_local, n_halo=n_halo, nnz=nnz, nnz_halo=nnz_halo,
               local_ids=np.empty(n_local, np.int32), halo_ids=np.empty(n_halo, np.int32),
               rowptr=np.empty(n_local + 1, np.int64), split=np.empty(n_local, np.int64),
               col=np.empty(nnz, np.int32), val=np.empty(nnz, np.float32),
               h_colptr=np.empty(n_halo + 1, np.int64), h_row=np.empty(nnz_halo, np.int32),
               h_val=np.empty(nnz_halo, np.float32), h_self=np.empty(n_halo, np.float32))
    _check(L.sat_partition_view_build(
        N, _ptr(g_rowptr), _ptr(g_col), _ptr(g_deg), _ptr(part), m,
        *[_ptr(out[k]) for k in ("local_ids", "halo_ids", "rowptr", "split", "col", "val",
                                 "h_colptr", "h_row", "h_val", "h_self")]),
        "sat_partition_view_build")
    return out


def history_gather(table, n_rows, ld_table, ids, n, d, out, ld_out, dtype=F32, stream=None):
    _check(lib().sat_history_gather(_ptr(table), n_rows, ld_table, _ptr(ids), n, d, _ptr(out),
                                    ld_out, dtype, stream), "sat_history_gather")


def history_gather_add(table, n_rows, ld_table, ids, n, d, out, ld_out, dtype=F32, stream=None):
    _check(lib().sat_history_gather_add(_ptr(table), n_rows, ld_table, _ptr(ids), n, d, _ptr(out),
                                        ld_out, dtype, stream), "sat_history_gather_add")


def history_compress_workspace_bytes(n):
    return lib().sat_history_compress_workspace_bytes(n)


def history_compress_plan(H, ld_h, n, d, precision, row_off, dtype=F32, workspace=None,
                          workspace_bytes=0, stream=None):
    _check(lib().sat_history_compress_plan(_ptr(H), ld_h, n, d, precision, dtype, _ptr(row_off),
                                           _ptr(workspace), workspace_bytes, stream),
           "sat_history_compress_plan")


def history_compress_encode(H, ld_h, n, d, precision, row_off, codes, capacity, dtype=F32,
                            stream=None):
    _check(lib().sat_history_compress_encode(_ptr(H), ld_h, n, d, precision, dtype, _ptr(row_off),
                                             _ptr(codes), capacity, stream),
           "sat_history_compress_encode")


def history_decompress(codes, row_off, n_rows, ids, n, d, precision, out, ld_out, dtype=F32,
                       stream=None):
    _check(lib().sat_history_decompress(_ptr(codes), _ptr(row_off), n_rows, _ptr(ids), n, d,
                                        precision, dtype, _ptr(out), ld_out, stream),
           "sat_history_decompress")


def history_push(table, n_rows, ld_table, ids, n, d, H, ld_h, dtype=F32, stream=None):
    _check(lib().sat_history_push(_ptr(table), n_rows, ld_table, _ptr(ids), n, d, _ptr(H), ld_h,
                                  dtype, stream), "sat_history_push")


def predict_workspace_bytes(n_local, n_halo, d, d_s, tau):
    return lib().sat_predict_workspace_bytes(n_local, n_halo, d, d_s, tau)


def predict(pv, w, slots, n_rows_slot, ld_slot, ids, Hbar, ld, dtype=F32, workspace=None,
            workspace_bytes=0, stream=None):
    arr = (C.c_void_p * len(slots))(*[_ptr(s) for s in slots])
    _check(lib().sat_predict(pv.ref, w.ref, C.addressof(arr), n_rows_slot, ld_slot, _ptr(ids),
                             _ptr(Hbar), ld, dtype, _ptr(workspace), workspace_bytes, stream),
           "sat_predict")


def predict_states_workspace_bytes(d, d_s):
    return lib().sat_predict_states_workspace_bytes(d, d_s)


def predict_states(w, slots, n_rows_slot, ld_slot, ids, n_nodes, S, dtype=F32, workspace=None,
                   workspace_bytes=0, stream=None):
    arr = (C.c_void_p * len(slots))(*[_ptr(s) for s in slots])
    _check(lib().sat_predict_states(w.ref, C.addressof(arr), n_rows_slot, ld_slot, _ptr(ids), n_nodes,
                                    dtype, _ptr(S), _ptr(workspace), workspace_bytes, stream),
           "sat_predict_states")


def predict_hop_workspace_bytes(n_halo, d_s):
    return lib().sat_predict_hop_workspace_bytes(n_halo, d_s)


def predict_hop(pv, w, S, newest, n_rows_newest, ld_newest, halo_ids, Hbar, ld, dtype=F32,
                workspace=None, workspace_bytes=0, stream=None):
    _check(lib().sat_predict_hop(pv.ref, w.ref, _ptr(S), _ptr(newest), n_rows_newest, ld_newest,
                                 _ptr(halo_ids), _ptr(Hbar), ld, dtype, _ptr(workspace),
                                 workspace_bytes, stream), "sat_predict_hop")


def predict_cached(pv, w, slots, n_rows_slot, ld_slot, ids, Hbar, ld, proj, n_proj_valid, dtype=F32,
                   workspace=None, workspace_bytes=0, stream=None):
    arr = (C.c_void_p * len(slots))(*[_ptr(s) for s in slots])
    parr = (C.c_void_p * len(proj))(*[_ptr(p) for p in proj])
    _check(lib().sat_predict_cached(pv.ref, w.ref, C.addressof(arr), n_rows_slot, ld_slot, _ptr(ids),
                                    _ptr(Hbar), ld, dtype, C.addressof(parr), n_proj_valid,
                                    _ptr(workspace), workspace_bytes, stream), "sat_predict_cached")


def spmm_workspace_bytes(pv, d):
    return lib().sat_spmm_workspace_bytes(pv.ref, d)


def predictor_train_workspace_bytes(n_local, n_halo, d, d_s, tau):
    return lib().sat_predictor_train_workspace_bytes(n_local, n_halo, d, d_s, tau)


def predictor_grad(pv, w, slots, n_rows_slot, ld_slot, ids, target, ld_target, weight, dWx, dWh,
                   db, dWg, loss, dtype=F32, workspace=None, workspace_bytes=0, stream=None):
    arr = (C.c_void_p * len(slots))(*[_ptr(s) for s in slots])
    _check(lib().sat_predictor_grad(pv.ref, w.ref, C.addressof(arr), n_rows_slot, ld_slot, _ptr(ids),
                                    _ptr(target), ld_target, _ptr(weight), dtype, _ptr(dWx),
                                    _ptr(dWh), _ptr(db), _ptr(dWg), _ptr(loss), _ptr(workspace),
                                    workspace_bytes, stream), "sat_predictor_grad")


def sgd_update(param, grad, n, lr, stream=None):
    _check(lib().sat_sgd_update(_ptr(param), _ptr(grad), n, lr, stream), "sat_sgd_update")


def spmm_fwd(pv, Hbar, ld_in, d, AGG, ld_out, dtype=F32, workspace=None, workspace_bytes=0,
             stream=None):
    _check(lib().sat_spmm_fwd(pv.ref, _ptr(Hbar), ld_in, d, dtype, _ptr(AGG), ld_out,
                              _ptr(workspace), workspace_bytes, stream), "sat_spmm_fwd")


def spmm_bwd(pv, dAGG, ld_in, d, dH_local, ld_out, dH_halo=None, ld_halo=0, dtype=F32,
             workspace=None, workspace_bytes=0, stream=None):
    _check(lib().sat_spmm_bwd(pv.ref, _ptr(dAGG), ld_in, d, dtype, _ptr(dH_local), ld_out,
                              _ptr(dH_halo), ld_halo, _ptr(workspace), workspace_bytes, stream),
           "sat_spmm_bwd")


def dense_fwd(AGG, ld_a, n, d_in, d_out, W, ld_w, act, H, ld_h, dtype=F32, stream=None):
    _check(lib().sat_dense_fwd(_ptr(AGG), ld_a, n, d_in, d_out, _ptr(W), ld_w, act, dtype,
                               _ptr(H), ld_h, stream), "sat_dense_fwd")


def dense_bwd_workspace_bytes(n, d_in, d_out):
    return lib().sat_dense_bwd_workspace_bytes(n, d_in, d_out)


def dense_bwd(dH, ld_dh, Hout, ld_ho, AGG, ld_a, W, ld_w, n, d_in, d_out, act, dW, ld_dw,
              dAGG, ld_da, dtype=F32, workspace=None, workspace_bytes=0, stream=None):
    _check(lib().sat_dense_bwd(_ptr(dH), ld_dh, _ptr(Hout), ld_ho, _ptr(AGG), ld_a, _ptr(W), ld_w,
                               n, d_in, d_out, act, dtype, _ptr(dW), ld_dw, _ptr(dAGG), ld_da,
                               _ptr(workspace), workspace_bytes, stream), "sat_dense_bwd")


def gat_scores(Z, ld_z, n, n_dst, heads, d_head, a_dst, a_src, el, er, dtype=F32, stream=None):
    _check(lib().sat_gat_scores(_ptr(Z), ld_z, n, n_dst, heads, d_head, _ptr(a_dst), _ptr(a_src),
                                dtype, _ptr(el), _ptr(er), stream), "sat_gat_scores")


def gat_aggregate_fwd(pv, Z, ld_z, heads, d_head, el, er, slope, act, H, ld_h, stats, dtype=F32,
                      stream=None):
    _check(lib().sat_gat_aggregate_fwd(pv.ref, _ptr(Z), ld_z, heads, d_head, dtype, _ptr(el),
                                       _ptr(er), slope, act, _ptr(H), ld_h, _ptr(stats), stream),
           "sat_gat_aggregate_fwd")


def gat_aggregate_bwd_workspace_bytes(n_local, n_halo, heads, d_head, dtype=F32):
    return lib().sat_gat_aggregate_bwd_workspace_bytes(n_local, n_halo, heads, d_head, dtype)


def gat_aggregate_bwd(pv, Z, ld_z, heads, d_head, el, er, stats, slope, act, dH, ld_dh, H, ld_h,
                      a_dst, a_src, dZ, ld_dz, da_dst, da_src, dtype=F32, workspace=None,
                      workspace_bytes=0, stream=None):
    _check(lib().sat_gat_aggregate_bwd(pv.ref, _ptr(Z), ld_z, heads, d_head, dtype, _ptr(el),
                                       _ptr(er), _ptr(stats), slope, act, _ptr(dH), ld_dh, _ptr(H),
                                       ld_h, _ptr(a_dst), _ptr(a_src), _ptr(dZ), ld_dz,
                                       _ptr(da_dst), _ptr(da_src), _ptr(workspace),
                                       workspace_bytes, stream), "sat_gat_aggregate_bwd")


def loss_workspace_bytes(n):
    return lib().sat_loss_workspace_bytes(n)


def loss_grad(HL, ld_hl, n, n_classes, y, dH, ld_dh, loss=None, dtype=F32, workspace=None,
              workspace_bytes=0, stream=None):
    _check(lib().sat_loss_grad(_ptr(HL), ld_hl, n, n_classes, _ptr(y), dtype, _ptr(dH), ld_dh,
                               _ptr(loss), _ptr(workspace), workspace_bytes, stream),
           "sat_loss_grad")


def loss_grad_static_max_rows():
    return lib().sat_loss_grad_static_max_rows()


def loss_grad_static(HL, ld_hl, n, n_classes, y, dH, ld_dh, loss=None, dtype=F32, stream=None):
    _check(lib().sat_loss_grad_static(_ptr(HL), ld_hl, n, n_classes, _ptr(y), dtype, _ptr(dH),
                                      ld_dh, _ptr(loss), stream), "sat_loss_grad_static")
