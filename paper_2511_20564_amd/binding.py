"""ctypes binding of libe2eg.so: same names and argument order as include/e2eg.h.

Pointer arguments accept a torch tensor (its data_ptr() is passed), an int address or None.
A negative status raises E2egError with the library's message.  Nothing is computed here.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libe2eg.so")

E2EG_OK = 0
E2EG_ERR_INVALID_ARG = -1
E2EG_ERR_NULL_PTR = -2
E2EG_ERR_BAD_DTYPE = -3
E2EG_ERR_CAPACITY = -4
E2EG_ERR_OVERFLOW = -5
E2EG_ERR_WORKSPACE = -6
E2EG_ERR_HIP = -7
E2EG_ERR_BAD_INDEX = -8
E2EG_F32 = 0
E2EG_BF16 = 1
E2EG_ADD_SELF_LOOPS = 1
E2EG_AGG_SYM, E2EG_AGG_MEAN, E2EG_AGG_MEAN_T, E2EG_AGG_SUM = 0, 1, 2, 3
E2EG_TRANSFORM_FWD = 0
E2EG_TRANSFORM_BWD = 1

_vp, _i32, _i64, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t

# name -> (restype, argtypes); the list the header declares
SIGNATURES = {
    "e2eg_status_string": (ctypes.c_char_p, [_i32]),
    "e2eg_last_error": (ctypes.c_char_p, []),
    "e2eg_version": (_i32, []),
    "e2eg_build_csr_workspace_bytes": (_sz, [_i32, _i32, _i64]),
    "e2eg_build_csr": (_i32, [_i32, _i32, _i64, _vp, _vp, _i32, _vp, _vp, _i64, ctypes.POINTER(_i64), _vp, _sz, _vp]),
    "e2eg_sched_bytes": (_sz, [_i32, _i64]),
    "e2eg_normalize_workspace_bytes": (_sz, [_i32, _i64]),
    "e2eg_normalize": (_i32, [_i32, _i64, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _sz, _vp]),
    "e2eg_propagate_workspace_bytes": (_sz, [_i32, _i64, _i32, _i32, _i32]),
    "e2eg_propagate_fwd": (_i32, [_i32, _i64, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _i64, _vp, _i64, _i64, _vp, _sz, _vp]),
    "e2eg_propagate_bwd": (_i32, [_i32, _i64, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _sz, _vp]),
    "e2eg_layer_transform_workspace_bytes": (_sz, [_i32, _i32, _i32, _i32, _i32]),
    "e2eg_layer_transform": (_i32, [_i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "e2eg_layer_transform_noalloc": (_i32, [_i32, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "e2eg_aggregate_workspace_bytes": (_sz, [_i32, _i64, _i32, _i32]),
    "e2eg_aggregate": (_i32, [_i32, _i32, _i64, _vp, _vp, _vp, _i32, _i32, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _sz, _vp]),
    "e2eg_readout_mean": (_i32, [_i32, _i32, _i32, _i32, _vp, _i64, _vp, _i64, _i64, _vp, _i64, _vp]),
    "e2eg_gfae_loss_workspace_bytes": (_sz, [_i32, _i32]),
    "e2eg_gfae_loss": (_i32, [_i32, _i32, _i32, _vp, _i64, _vp, _i64, _vp, _vp, _i64, ctypes.c_float, _vp, _sz, _vp]),
    "e2eg_block_norms_workspace_bytes": (_sz, [_i32, _i32, _i32]),
    "e2eg_block_norms": (_i32, [_i32, _i32, _i32, _i32, _vp, _i64, _vp, _vp, _sz, _vp]),
    "e2eg_gradnorm_step": (_i32, [_i32, _vp, _vp, _vp, ctypes.c_double, ctypes.c_double, _vp, _vp]),
    "e2eg_edge_weights": (_i32, [_i32, _i32, _i64, _vp, _vp, _vp, _i64, _vp, _vp, _vp, _vp]),
    "e2eg_sched_weighted_bytes": (_sz, [_i32, _i64]),
    "e2eg_normalize_weighted": (_i32, [_i32, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp, _sz, _vp]),
    "e2eg_sched_check_symmetric": (_i32, [_vp, _vp]),
    "e2eg_propagate_weighted_fwd": (_i32, [_i32, _i64, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _i64, _vp, _i64, _i64, _vp, _sz, _vp]),
    "e2eg_propagate_weighted_bwd": (_i32, [_i32, _i64, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _sz, _vp]),
    "e2eg_sampling_weights": (_i32, [_i64, _vp, ctypes.c_float, _vp, _vp]),
    "e2eg_sampler_table_bytes": (_sz, [_i64]),
    "e2eg_sampler_prepare_workspace_bytes": (_sz, [_i32, _i64]),
    "e2eg_sampler_prepare": (_i32, [_i32, _i64, _vp, _vp, _vp, _vp, _sz, _vp, _sz, _vp]),
    "e2eg_sample_capacity": (_i64, [_i32, _i32, _i32, ctypes.POINTER(_i32)]),
    "e2eg_sample_subgraph_workspace_bytes": (_sz, [_i32, _i32, _i32, ctypes.POINTER(_i32)]),
    "e2eg_sample_subgraph": (_i32, [_i32, _i32, _i64, _vp, _vp, _vp, _vp, _i32, _vp, _i32, ctypes.POINTER(_i32),
                                    ctypes.c_uint64, _vp, _i64, _vp, _vp, _vp, _i64, ctypes.POINTER(_i32), _vp, _sz,
                                    _vp]),
    "e2eg_profile_begin": (_i32, [_i32]),
    "e2eg_profile_end": (_i32, [ctypes.POINTER(ctypes.c_float), _i32, ctypes.POINTER(_i32)]),
    "e2eg_profile_copy": (_i32, [_vp, _vp, ctypes.c_size_t, _vp]),
}

_lib = None


class E2egError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"e2eg status {status}: {message}")
        self.status = status


def load_library():
    """Loads libe2eg.so from the package directory.  There is no other implementation: if the
    library has not been built (paper_2511_20564_amd/build.py) this raises."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_20564_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def _check(status: int):
    if status != E2EG_OK:
        lib = load_library()
        raise E2egError(status, f"{lib.e2eg_status_string(status).decode()}: {lib.e2eg_last_error().decode()}")


def e2eg_version() -> int:
    return int(load_library().e2eg_version())


def e2eg_status_string(status: int) -> str:
    return load_library().e2eg_status_string(status).decode()


def e2eg_last_error() -> str:
    return load_library().e2eg_last_error().decode()


def e2eg_build_csr_workspace_bytes(n_users, n_items, n_edges) -> int:
    return int(load_library().e2eg_build_csr_workspace_bytes(n_users, n_items, n_edges))


def e2eg_build_csr(n_users, n_items, n_edges, d_user_ids, d_item_ids, flags, d_row_ptr, d_col_idx,
                   col_capacity, ws, ws_bytes=None, stream=0) -> int:
    """-> nnz"""
    nnz = _i64(0)
    _check(load_library().e2eg_build_csr(n_users, n_items, n_edges, _ptr(d_user_ids), _ptr(d_item_ids), flags,
                                         _ptr(d_row_ptr), _ptr(d_col_idx), col_capacity, ctypes.byref(nnz),
                                         _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes, stream or None))
    return int(nnz.value)


def e2eg_sched_bytes(n, nnz) -> int:
    return int(load_library().e2eg_sched_bytes(n, nnz))


def e2eg_normalize_workspace_bytes(n, nnz) -> int:
    return int(load_library().e2eg_normalize_workspace_bytes(n, nnz))


def e2eg_normalize(n, nnz, d_row_ptr, d_col_idx, d_deg, d_dinv_sqrt, d_sched, sched_bytes, ws, ws_bytes=None,
                   stream=0):
    _check(load_library().e2eg_normalize(n, nnz, _ptr(d_row_ptr), _ptr(d_col_idx), _ptr(d_deg), _ptr(d_dinv_sqrt),
                                         _ptr(d_sched),
                                         _nbytes(d_sched) if sched_bytes is None else sched_bytes, _ptr(ws),
                                         _nbytes(ws) if ws_bytes is None else ws_bytes, stream or None))


def e2eg_propagate_workspace_bytes(n, nnz, dtype, F, K) -> int:
    return int(load_library().e2eg_propagate_workspace_bytes(n, nnz, dtype, F, K))


def e2eg_propagate_fwd(n, nnz, d_row_ptr, d_col_idx, d_dinv_sqrt, d_sched, dtype, F, K, d_X0, ldx, d_Xout, ldo,
                       layer_stride, ws, ws_bytes=None, stream=0):
    _check(load_library().e2eg_propagate_fwd(n, nnz, _ptr(d_row_ptr), _ptr(d_col_idx), _ptr(d_dinv_sqrt),
                                             _ptr(d_sched), dtype, F, K, _ptr(d_X0), ldx, _ptr(d_Xout), ldo,
                                             layer_stride, _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes,
                                             stream or None))


def e2eg_propagate_bwd(n, nnz, d_row_ptr, d_col_idx, d_dinv_sqrt, d_sched, dtype, F, K, d_gXK, ldg, d_gLayers,
                       g_layer_stride, d_gX0, ldo, ws, ws_bytes=None, stream=0):
    _check(load_library().e2eg_propagate_bwd(n, nnz, _ptr(d_row_ptr), _ptr(d_col_idx), _ptr(d_dinv_sqrt),
                                             _ptr(d_sched), dtype, F, K, _ptr(d_gXK), ldg, _ptr(d_gLayers),
                                             g_layer_stride, _ptr(d_gX0), ldo, _ptr(ws),
                                             _nbytes(ws) if ws_bytes is None else ws_bytes, stream or None))


def e2eg_edge_weights(n_users, n_items, n_edges, d_user_ids, d_item_ids, d_weights, nnz, d_row_ptr, d_col_idx,
                      d_val, stream=0):
    _check(load_library().e2eg_edge_weights(n_users, n_items, n_edges, _ptr(d_user_ids), _ptr(d_item_ids),
                                            _ptr(d_weights), nnz, _ptr(d_row_ptr), _ptr(d_col_idx), _ptr(d_val),
                                            stream or None))


def e2eg_sched_weighted_bytes(n, nnz) -> int:
    return int(load_library().e2eg_sched_weighted_bytes(n, nnz))


def e2eg_sched_check_symmetric(d_sched, stream=0):
    """Raises E2egError (INVALID_ARG) if the schedule's structure or values are not symmetric."""
    _check(load_library().e2eg_sched_check_symmetric(_ptr(d_sched), stream or None))


def e2eg_normalize_weighted(n, nnz, d_row_ptr, d_col_idx, d_val, d_deg, d_deg_w, d_dinv_sqrt, d_sched, sched_bytes,
                            ws, ws_bytes=None, stream=0):
    _check(load_library().e2eg_normalize_weighted(n, nnz, _ptr(d_row_ptr), _ptr(d_col_idx), _ptr(d_val),
                                                  _ptr(d_deg), _ptr(d_deg_w), _ptr(d_dinv_sqrt), _ptr(d_sched),
                                                  _nbytes(d_sched) if sched_bytes is None else sched_bytes,
                                                  _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes,
                                                  stream or None))


def e2eg_propagate_weighted_fwd(n, nnz, d_row_ptr, d_col_idx, d_dinv_sqrt, d_sched, dtype, F, K, d_X0, ldx, d_Xout,
                                ldo, layer_stride, ws, ws_bytes=None, stream=0):
    _check(load_library().e2eg_propagate_weighted_fwd(n, nnz, _ptr(d_row_ptr), _ptr(d_col_idx), _ptr(d_dinv_sqrt),
                                                      _ptr(d_sched), dtype, F, K, _ptr(d_X0), ldx, _ptr(d_Xout),
                                                      ldo, layer_stride, _ptr(ws),
                                                      _nbytes(ws) if ws_bytes is None else ws_bytes, stream or None))


def e2eg_propagate_weighted_bwd(n, nnz, d_row_ptr, d_col_idx, d_dinv_sqrt, d_sched, dtype, F, K, d_gXK, ldg,
                                d_gLayers, g_layer_stride, d_gX0, ldo, ws, ws_bytes=None, stream=0):
    _check(load_library().e2eg_propagate_weighted_bwd(n, nnz, _ptr(d_row_ptr), _ptr(d_col_idx), _ptr(d_dinv_sqrt),
                                                      _ptr(d_sched), dtype, F, K, _ptr(d_gXK), ldg, _ptr(d_gLayers),
                                                      g_layer_stride, _ptr(d_gX0), ldo, _ptr(ws),
                                                      _nbytes(ws) if ws_bytes is None else ws_bytes, stream or None))


def e2eg_sampling_weights(nnz, d_val, beta, d_p, stream=0):
    _check(load_library().e2eg_sampling_weights(nnz, _ptr(d_val), beta, _ptr(d_p), stream or None))


def e2eg_sampler_table_bytes(nnz) -> int:
    return int(load_library().e2eg_sampler_table_bytes(nnz))


def e2eg_sampler_prepare_workspace_bytes(n, nnz) -> int:
    return int(load_library().e2eg_sampler_prepare_workspace_bytes(n, nnz))


def e2eg_sampler_prepare(n, nnz, d_row_ptr, d_col_idx, d_p, d_table, table_bytes, ws, ws_bytes=None, stream=0):
    _check(load_library().e2eg_sampler_prepare(n, nnz, _ptr(d_row_ptr), _ptr(d_col_idx), _ptr(d_p), _ptr(d_table),
                                               _nbytes(d_table) if table_bytes is None else table_bytes, _ptr(ws),
                                               _nbytes(ws) if ws_bytes is None else ws_bytes, stream or None))


def _fanout_array(fanout):
    return (_i32 * len(fanout))(*[int(k) for k in fanout]) if fanout is not None else None


def e2eg_sample_capacity(n, n_seeds, fanout) -> int:
    """-> the number of draws the fan-outs allow (raises on bad arguments)."""
    cap = int(load_library().e2eg_sample_capacity(n, n_seeds, len(fanout) if fanout is not None else 0,
                                                  _fanout_array(fanout)))
    if cap < 0:
        raise E2egError(E2EG_ERR_INVALID_ARG, e2eg_last_error())
    return cap


def e2eg_sample_subgraph_workspace_bytes(n, n_seeds, fanout) -> int:
    return int(load_library().e2eg_sample_subgraph_workspace_bytes(n, n_seeds, len(fanout), _fanout_array(fanout)))


def e2eg_sample_subgraph(n_users, n, nnz, d_row_ptr, d_col_idx, d_table, d_val, n_seeds, d_seeds, fanout, seed, d_nodes,
                         node_capacity, d_edge_users, d_edge_items, d_edge_w, edge_capacity, ws, ws_bytes=None,
                         stream=0):
    """-> (local users, local items, pairs)"""
    counts = (_i32 * 3)()
    _check(load_library().e2eg_sample_subgraph(n_users, n, nnz, _ptr(d_row_ptr), _ptr(d_col_idx), _ptr(d_table),
                                               _ptr(d_val), n_seeds, _ptr(d_seeds),
                                               len(fanout) if fanout is not None else 0, _fanout_array(fanout),
                                               ctypes.c_uint64(seed), _ptr(d_nodes), node_capacity,
                                               _ptr(d_edge_users), _ptr(d_edge_items), _ptr(d_edge_w), edge_capacity,
                                               counts, _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes,
                                               stream or None))
    return int(counts[0]), int(counts[1]), int(counts[2])


def e2eg_layer_transform_workspace_bytes(mode, n, Fin, Fout, dtype) -> int:
    return int(load_library().e2eg_layer_transform_workspace_bytes(mode, n, Fin, Fout, dtype))


def e2eg_layer_transform(mode, n, Fin, Fout, dtype, relu, d_P, d_W, d_H, d_gH, d_gP, d_gW, ws, ws_bytes=None,
                         stream=0):
    _check(load_library().e2eg_layer_transform(mode, n, Fin, Fout, dtype, relu, _ptr(d_P), _ptr(d_W), _ptr(d_H),
                                               _ptr(d_gH), _ptr(d_gP), _ptr(d_gW), _ptr(ws),
                                               _nbytes(ws) if ws_bytes is None else ws_bytes, stream or None))


def e2eg_layer_transform_noalloc(mode, n, Fin, Fout, dtype, relu, d_P, d_W, d_H, d_gH, d_gP, d_gW, stream=0):
    _check(load_library().e2eg_layer_transform_noalloc(mode, n, Fin, Fout, dtype, relu, _ptr(d_P), _ptr(d_W),
                                                       _ptr(d_H), _ptr(d_gH), _ptr(d_gP), _ptr(d_gW), stream or None))


def e2eg_profile_begin(capacity: int):
    _check(load_library().e2eg_profile_begin(capacity))


def e2eg_profile_end(capacity: int):
    """-> list of per-launch durations in ms"""
    buf = (ctypes.c_float * max(capacity, 1))()
    count = _i32(0)
    _check(load_library().e2eg_profile_end(buf, capacity, ctypes.byref(count)))
    return [float(buf[k]) for k in range(min(capacity, count.value))]


def e2eg_profile_copy(d_dst, d_src, nbytes: int, stream=0):
    _check(load_library().e2eg_profile_copy(_ptr(d_dst), _ptr(d_src), nbytes, stream or None))


def e2eg_readout_mean(n, dtype, F, K, d_X0, ldx, d_layers, ld, layer_stride, d_Y, ldy, stream=0):
    _check(load_library().e2eg_readout_mean(n, dtype, F, K, _ptr(d_X0), ldx, _ptr(d_layers), ld, layer_stride,
                                            _ptr(d_Y), ldy, stream or None))


def e2eg_gfae_loss_workspace_bytes(n, F) -> int:
    return int(load_library().e2eg_gfae_loss_workspace_bytes(n, F))


def e2eg_gfae_loss(n, dtype, F, d_X, ldx, d_Y, ldy, d_loss, d_gY, ldg, grad_scale, ws, ws_bytes=None, stream=0):
    _check(load_library().e2eg_gfae_loss(n, dtype, F, _ptr(d_X), ldx, _ptr(d_Y), ldy, _ptr(d_loss), _ptr(d_gY), ldg,
                                         grad_scale, _ptr(ws), _nbytes(ws) if ws_bytes is None else ws_bytes,
                                         stream or None))


def e2eg_aggregate_workspace_bytes(n, nnz, dtype, F) -> int:
    return int(load_library().e2eg_aggregate_workspace_bytes(n, nnz, dtype, F))


def e2eg_aggregate(mode, n, nnz, d_row_ptr, d_col_idx, d_sched, dtype, F, d_X, ldx, d_addend, ld_add, d_Y, ldy, ws,
                   ws_bytes=None, stream=0):
    _check(load_library().e2eg_aggregate(mode, n, nnz, _ptr(d_row_ptr), _ptr(d_col_idx), _ptr(d_sched), dtype, F,
                                         _ptr(d_X), ldx, _ptr(d_addend), ld_add, _ptr(d_Y), ldy, _ptr(ws),
                                         _nbytes(ws) if ws_bytes is None else ws_bytes, stream or None))


def e2eg_block_norms_workspace_bytes(n, F, T) -> int:
    return int(load_library().e2eg_block_norms_workspace_bytes(n, F, T))


def e2eg_block_norms(n, dtype, F, T, d_G, ld, d_norms, ws, ws_bytes=None, stream=0):
    _check(load_library().e2eg_block_norms(n, dtype, F, T, _ptr(d_G), ld, _ptr(d_norms), _ptr(ws),
                                           _nbytes(ws) if ws_bytes is None else ws_bytes, stream or None))


def e2eg_gradnorm_step(loss, loss0, gnorm, w, gamma=1.0, lr=0.025):
    """Host arrays in (sequences of T floats) -> (meta-loss at `w`, new weights as a list)."""
    T = len(w)
    arr = ctypes.c_double * T
    a_loss, a_loss0, a_gn, a_w = arr(*loss), arr(*loss0), arr(*gnorm), arr(*w)
    meta = ctypes.c_double(0.0)
    _check(load_library().e2eg_gradnorm_step(T, ctypes.addressof(a_loss), ctypes.addressof(a_loss0),
                                             ctypes.addressof(a_gn), gamma, lr, ctypes.addressof(a_w),
                                             ctypes.addressof(meta)))
    return meta.value, list(a_w)
