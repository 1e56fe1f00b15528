"""CPU oracle: the plain definition of normalized-adjacency propagation, in double.

TEST INFRASTRUCTURE ONLY.  Nothing in the GPU package imports this; only tests, the smoke
check and the benchmark's CPU-baseline leg do.  The arithmetic is in `e2eg_oracle.c`
(plain C, built with gcc into `libe2eg_oracle.so`); this file marshals numpy arrays and
strings the layers together in the order the paper writes them:

    H(0) = X,  H(l+1) = A^ H(l)   for l = 0..K-1          (Section 3.1, LightGCN matrix form)
    G(K) = dL/dH(K),  G(l) = A^T G(l+1) [+ dL/dH(l) direct] (Appendix A, GNN backprop factor)

with A^ = D~^-1/2 (A + I) D~^-1/2 (Section 3, "Notation").
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "e2eg_oracle.c")
_LIB = os.path.join(_HERE, "libe2eg_oracle.so")
_LIB_SAN = os.path.join(_HERE, "libe2eg_oracle_san.so")
_lib = None

_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)
_f64p = ctypes.POINTER(ctypes.c_double)
_f32p = ctypes.POINTER(ctypes.c_float)
_u32p = ctypes.POINTER(ctypes.c_uint32)
_u64p = ctypes.POINTER(ctypes.c_uint64)


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP).  Returns the library path.

    sanitize=True builds a second library, instrumented with AddressSanitizer and
    UndefinedBehaviorSanitizer (any report aborts the process); a process that loads it must have
    been started with gcc's libasan.so first in LD_PRELOAD.  The environment variable
    E2EG_ORACLE_SANITIZE=1 makes this module load that library instead of the plain one."""
    lib = _LIB_SAN if sanitize else _LIB
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC):
        opt = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
               "-fno-sanitize-recover=all"] if sanitize else ["-O2"]
        cmd = ["gcc"] + opt + ["-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", lib, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return lib


def _load():
    global _lib
    if _lib is None:
        sanitize = os.environ.get("E2EG_ORACLE_SANITIZE", "") == "1"
        lib = ctypes.CDLL(build(sanitize=sanitize))
        lib.e2eg_oracle_max_threads.restype = ctypes.c_int32
        lib.e2eg_oracle_set_threads.argtypes = [ctypes.c_int32]
        lib.e2eg_oracle_build_csr.restype = ctypes.c_int64
        lib.e2eg_oracle_build_csr.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, _i32p, _i32p,
                                              ctypes.c_int32, _i64p, _i32p]
        lib.e2eg_oracle_build_csr_rows.restype = ctypes.c_int64
        lib.e2eg_oracle_build_csr_rows.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, _i32p, _i32p,
                                                   ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, _i64p, _i32p,
                                                   ctypes.c_int64]
        lib.e2eg_oracle_transposed_to_targets.argtypes = [ctypes.c_int64, ctypes.c_int64, _i64p, _i32p, _i64p,
                                                          ctypes.c_int64, _f64p, ctypes.c_int64, _i64p, _f64p]
        lib.e2eg_oracle_normalize.argtypes = [ctypes.c_int64, _i64p, _i64p, _f64p]
        lib.e2eg_oracle_propagate_layer.argtypes = [ctypes.c_int64, _i64p, _i32p, ctypes.c_int64, _f64p, _f64p]
        lib.e2eg_oracle_propagate_layer_transposed.argtypes = lib.e2eg_oracle_propagate_layer.argtypes
        lib.e2eg_oracle_propagate_rows.argtypes = [ctypes.c_int64, _i64p, _i64p, _i32p, ctypes.c_int64,
                                                   _f64p, _f64p]
        lib.e2eg_oracle_mean_neighbours.argtypes = [ctypes.c_int64, _i64p, _i32p, ctypes.c_int64, _f64p, _f64p]
        lib.e2eg_oracle_mean_neighbours_transposed.argtypes = lib.e2eg_oracle_mean_neighbours.argtypes
        lib.e2eg_oracle_edge_values.argtypes = [ctypes.c_int32, ctypes.c_int64, _i32p, _i32p, _f64p, ctypes.c_int64,
                                                _i64p, _i32p, _f64p]
        lib.e2eg_oracle_weighted_degrees.argtypes = [ctypes.c_int64, _i64p, _f64p, _f64p]
        lib.e2eg_oracle_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
        lib.e2eg_oracle_sampling_weights.argtypes = [ctypes.c_int64, _f64p, ctypes.c_double, _f64p]
        lib.e2eg_oracle_sampling_table.argtypes = [ctypes.c_int64, _i64p, _i32p, _f32p, _u64p]
        lib.e2eg_oracle_sample_subgraph.restype = ctypes.c_int64
        lib.e2eg_oracle_sample_subgraph.argtypes = [ctypes.c_int64, _i64p, _i32p, _u64p, ctypes.c_int64, _i32p,
                                                    ctypes.c_int32, _i32p, ctypes.c_uint64, _i32p, _i32p, _i32p,
                                                    _i64p, ctypes.c_int64]
        lib.e2eg_oracle_propagate_layer_weighted.argtypes = [ctypes.c_int64, _i64p, _i32p, _f64p, _f64p, ctypes.c_int64,
                                                             _f64p, _f64p]
        lib.e2eg_oracle_propagate_layer_weighted_transposed.argtypes = lib.e2eg_oracle_propagate_layer_weighted.argtypes
        lib.e2eg_oracle_block_norms.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, _f64p, _f64p]
        lib.e2eg_oracle_gradnorm_step.restype = ctypes.c_double
        lib.e2eg_oracle_gradnorm_step.argtypes = [ctypes.c_int64, _f64p, _f64p, _f64p, ctypes.c_double, ctypes.c_double,
                                                  _f64p]
        lib.e2eg_oracle_readout_mean.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, _f64p, _f64p, _f64p]
        lib.e2eg_oracle_gfae_loss.restype = ctypes.c_double
        lib.e2eg_oracle_gfae_loss.argtypes = [ctypes.c_int64, ctypes.c_int64, _f64p, _f64p, _f64p]
        lib.e2eg_oracle_transform_fwd.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, _f64p, _f64p,
                                                  ctypes.c_int32, _f64p, _f64p]
        lib.e2eg_oracle_transform_bwd.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, _f64p, _f64p,
                                                  _f64p, _f64p, ctypes.c_int32, _f64p, _f64p]
        _lib = lib
    return _lib


def _p(a, t):
    return a.ctypes.data_as(t)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def max_threads() -> int:
    return int(_load().e2eg_oracle_max_threads())


def set_threads(t: int) -> None:
    _load().e2eg_oracle_set_threads(int(t))


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of bf16 bit patterns (uint16) as doubles."""
    u = _c(bits, np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def as_f64(x: np.ndarray) -> np.ndarray:
    """The exact values of an input array: fp32 values, or bf16 bit patterns if uint16."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return bf16_bits_to_f64(x)
    return _c(x, np.float64)


def build_csr(n_users, n_items, users, items, add_self_loops=True):
    """Canonical CSR of A~ = A + I (of A if not add_self_loops).  -> (row_ptr int64[n+1],
    col_idx int32[nnz])."""
    users = _c(users, np.int32)
    items = _c(items, np.int32)
    if users.shape != items.shape or users.ndim != 1:
        raise ValueError("users/items must be 1-D arrays of equal length")
    n = int(n_users) + int(n_items)
    E = users.size
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    col = np.empty(max(1, 2 * E + n), dtype=np.int32)
    nnz = _load().e2eg_oracle_build_csr(n_users, n_items, E, _p(users, _i32p), _p(items, _i32p),
                                        1 if add_self_loops else 0, _p(row_ptr, _i64p), _p(col, _i32p))
    if nnz < 0:
        raise ValueError("edge id out of range")
    return row_ptr, col[:nnz].copy()


def normalize(row_ptr):
    """-> (deg int64[n] = d~_i, dinv_sqrt float64[n] = d~_i^-1/2)."""
    row_ptr = _c(row_ptr, np.int64)
    n = row_ptr.size - 1
    deg = np.empty(n, dtype=np.int64)
    dinv = np.empty(n, dtype=np.float64)
    _load().e2eg_oracle_normalize(n, _p(row_ptr, _i64p), _p(deg, _i64p), _p(dinv, _f64p))
    return deg, dinv


def propagate_layer(row_ptr, col_idx, X):
    """Y = A^ X for one layer (gather over rows)."""
    row_ptr = _c(row_ptr, np.int64)
    col_idx = _c(col_idx, np.int32)
    X = _c(X, np.float64)
    n, F = X.shape
    assert row_ptr.size == n + 1
    Y = np.empty_like(X)
    _load().e2eg_oracle_propagate_layer(n, _p(row_ptr, _i64p), _p(col_idx, _i32p), F, _p(X, _f64p),
                                        _p(Y, _f64p))
    return Y


def propagate_layer_transposed(row_ptr, col_idx, G):
    """A^T G for one layer (scatter over the rows of the forward CSR)."""
    row_ptr = _c(row_ptr, np.int64)
    col_idx = _c(col_idx, np.int32)
    G = _c(G, np.float64)
    n, F = G.shape
    assert row_ptr.size == n + 1
    out = np.empty_like(G)
    _load().e2eg_oracle_propagate_layer_transposed(n, _p(row_ptr, _i64p), _p(col_idx, _i32p), F,
                                                   _p(G, _f64p), _p(out, _f64p))
    return out


def propagate_rows(row_ptr, col_idx, X, rows):
    """(A^ X)[rows] computed row by row."""
    row_ptr = _c(row_ptr, np.int64)
    col_idx = _c(col_idx, np.int32)
    X = _c(X, np.float64)
    rows = _c(rows, np.int64)
    F = X.shape[1]
    Y = np.empty((rows.size, F), dtype=np.float64)
    _load().e2eg_oracle_propagate_rows(rows.size, _p(rows, _i64p), _p(row_ptr, _i64p), _p(col_idx, _i32p),
                                       F, _p(X, _f64p), _p(Y, _f64p))
    return Y


def build_csr_rows(n_users, n_items, users, items, row_lo, row_hi, add_self_loops=True):
    """Rows row_lo <= r < row_hi of the canonical CSR of A~ -> (row_ptr_local int64 starting at 0,
    col_idx int32), built from the pair list alone."""
    users = _c(users, np.int32)
    items = _c(items, np.int32)
    if users.shape != items.shape or users.ndim != 1:
        raise ValueError("users/items must be 1-D arrays of equal length")
    rows = int(row_hi) - int(row_lo)
    if rows < 0:
        raise ValueError("empty or reversed row range")
    row_ptr = np.zeros(rows + 1, dtype=np.int64)
    # room for every listed entry of the range (repeated pairs make the result shorter)
    listed = (int(np.count_nonzero((users >= row_lo) & (users < row_hi)))
              + int(np.count_nonzero((items >= row_lo - n_users) & (items < row_hi - n_users)))
              + (rows if add_self_loops else 0))
    col = np.empty(max(listed, 1), dtype=np.int32)
    nnz = _load().e2eg_oracle_build_csr_rows(n_users, n_items, users.size, _p(users, _i32p), _p(items, _i32p),
                                             1 if add_self_loops else 0, int(row_lo), int(row_hi),
                                             _p(row_ptr, _i64p), _p(col, _i32p), col.size)
    if nnz < 0 or nnz > col.size:
        raise ValueError("bad row range, user or item id out of range, or out of memory")
    return row_ptr, col[:nnz]


def transposed_to_targets(row_lo, row_ptr_local, col_idx_local, deg, Gnext, targets, out):
    """out += contributions of the source rows [row_lo, row_lo + rows) to (A^T Gnext)[targets];
    `targets` ascending node ids, `deg` = d~ of every node, `out` float64 [len(targets), F]."""
    row_ptr_local, col_idx_local = _c(row_ptr_local, np.int64), _c(col_idx_local, np.int32)
    deg, targets = _c(deg, np.int64), _c(targets, np.int64)
    if Gnext.dtype != np.float64 or not Gnext.flags.c_contiguous or out.dtype != np.float64 or not out.flags.c_contiguous:
        raise ValueError("Gnext and out must be C-contiguous float64 arrays")
    if targets.size > 1 and (np.diff(targets) <= 0).any():
        raise ValueError("targets must be strictly ascending")
    F = Gnext.shape[1]
    assert out.shape == (targets.size, F) and row_ptr_local[-1] == col_idx_local.size
    _load().e2eg_oracle_transposed_to_targets(int(row_lo), row_ptr_local.size - 1, _p(row_ptr_local, _i64p),
                                              _p(col_idx_local, _i32p), _p(deg, _i64p), F, _p(Gnext, _f64p),
                                              targets.size, _p(targets, _i64p), _p(out, _f64p))


def propagate_fwd(row_ptr, col_idx, X0, K):
    """[H(1), ..., H(K)] with H(0) = X0 (fp32 values or bf16 bit patterns), no rounding in
    between."""
    H = as_f64(X0)
    layers = []
    for _ in range(K):
        H = propagate_layer(row_ptr, col_idx, H)
        layers.append(H)
    return layers


def propagate_bwd(row_ptr, col_idx, gHK, K, g_layers=None, g_shared=None):
    """dL/dH(0) given dL/dH(K) and optional direct terms: `g_layers`, dL/dH(1..K-1) (list of
    K-1 arrays, entry l-1 for layer l), or `g_shared`, one array that is the direct term of every
    layer 0..K-1 (a loss that reads all layers with equal weight)."""
    G = as_f64(gHK)
    for l in range(K - 1, -1, -1):
        G = propagate_layer_transposed(row_ptr, col_idx, G)
        if g_layers is not None and l >= 1:
            G = G + as_f64(g_layers[l - 1])
        if g_shared is not None:
            G = G + as_f64(g_shared)
    return G


def readout_mean(X0, layers):
    """Y = 1/(K+1) (H(0) + ... + H(K)) with H(0) = X0 and layers = [H(1), ..., H(K)]."""
    X0 = as_f64(X0)
    K = len(layers)
    n, F = X0.shape
    L = _c(np.stack([as_f64(h) for h in layers]) if K else np.zeros((0, n, F)), np.float64)
    Y = np.empty_like(X0)
    _load().e2eg_oracle_readout_mean(n, F, K, _p(X0, _f64p), _p(L, _f64p), _p(Y, _f64p))
    return Y


def gfae_loss(X, Y):
    """-> (||X - Y||_F^2, dL/dY = 2 (Y - X))."""
    X = as_f64(X)
    Y = as_f64(Y)
    assert X.shape == Y.shape
    n, F = X.shape
    gY = np.empty_like(X)
    loss = _load().e2eg_oracle_gfae_loss(n, F, _p(X, _f64p), _p(Y, _f64p), _p(gY, _f64p))
    return float(loss), gY


def gfae_step(row_ptr, col_idx, X0, K):
    """The self-supervised branch end to end on a LightGCN encoder: Y = mean of the K+1 layers,
    L = ||X0 - Y||_F^2, and dL/dX0 through the readout and the K layers (X0 also enters the loss
    directly).  -> (loss, Y, dL/dX0)."""
    layers = propagate_fwd(row_ptr, col_idx, X0, K)
    Y = readout_mean(X0, layers)
    loss, gY = gfae_loss(X0, Y)
    g = gY / (K + 1)                      # dL/dH(l), the same for every layer l = 0..K
    G0 = propagate_bwd(row_ptr, col_idx, g, K, g_shared=g)
    return loss, Y, G0 - gY               # - gY = 2 (X0 - Y): the direct dependence of the loss on X0


def transform_fwd(P, W, relu=True):
    """Z = P W and H = max(Z, 0) (H = Z if not relu).  -> (Z, H)."""
    P = as_f64(P)
    W = as_f64(W)
    n, Fin = P.shape
    assert W.shape[0] == Fin
    Fout = W.shape[1]
    Z = np.empty((n, Fout), dtype=np.float64)
    H = np.empty((n, Fout), dtype=np.float64)
    _load().e2eg_oracle_transform_fwd(n, Fin, Fout, _p(P, _f64p), _p(W, _f64p), 1 if relu else 0,
                                      _p(Z, _f64p), _p(H, _f64p))
    return Z, H


def transform_bwd(P, W, mask, gH, relu=True):
    """dP = dZ W^T, dW = P^T dZ with dZ = gH * [mask > 0] (dZ = gH if not relu)."""
    P = as_f64(P)
    W = as_f64(W)
    mask = as_f64(mask)
    gH = as_f64(gH)
    n, Fin = P.shape
    Fout = W.shape[1]
    dP = np.empty((n, Fin), dtype=np.float64)
    dW = np.empty((Fin, Fout), dtype=np.float64)
    _load().e2eg_oracle_transform_bwd(n, Fin, Fout, _p(P, _f64p), _p(W, _f64p), _p(mask, _f64p),
                                      _p(gH, _f64p), 1 if relu else 0, _p(dP, _f64p), _p(dW, _f64p))
    return dP, dW


def mean_neighbours(row_ptr, col_idx, X):
    """GraphSAGE mean aggregator: row i -> mean of X over the row's neighbours (0 if none)."""
    row_ptr = _c(row_ptr, np.int64)
    col_idx = _c(col_idx, np.int32)
    X = as_f64(X)
    n, F = X.shape
    M = np.empty_like(X)
    _load().e2eg_oracle_mean_neighbours(n, _p(row_ptr, _i64p), _p(col_idx, _i32p), F, _p(X, _f64p), _p(M, _f64p))
    return M


def mean_neighbours_transposed(row_ptr, col_idx, gM):
    """Transpose of the mean aggregator applied to gM (scatter over the same CSR)."""
    row_ptr = _c(row_ptr, np.int64)
    col_idx = _c(col_idx, np.int32)
    gM = as_f64(gM)
    n, F = gM.shape
    G = np.empty_like(gM)
    _load().e2eg_oracle_mean_neighbours_transposed(n, _p(row_ptr, _i64p), _p(col_idx, _i32p), F, _p(gM, _f64p),
                                                   _p(G, _f64p))
    return G


def sage_layer_fwd(row_ptr, col_idx, H, W, relu=True):
    """GraphSAGE layer: C = CONCAT(H, mean of neighbours), Z = C W (W is [2F][Fout]), H' = relu(Z).
    -> (C, Z, H')."""
    H = as_f64(H)
    C = np.concatenate([H, mean_neighbours(row_ptr, col_idx, H)], axis=1)
    Z, Hn = transform_fwd(C, W, relu)
    return C, Z, Hn


def sage_layer_bwd(row_ptr, col_idx, C, W, mask, gHn, relu=True):
    """Backward of sage_layer_fwd: -> (dL/dH, dL/dW) given dL/dH' and the sign pattern `mask` of Z."""
    F = C.shape[1] // 2
    dC, dW = transform_bwd(C, W, mask, gHn, relu)
    gH = dC[:, :F] + mean_neighbours_transposed(row_ptr, col_idx, np.ascontiguousarray(dC[:, F:]))
    return gH, dW


def block_norms(G, T):
    """2-norms of the T column blocks of G ([n, T*F])."""
    G = as_f64(G)
    n, TF = G.shape
    assert TF % T == 0
    out = np.empty(T, dtype=np.float64)
    _load().e2eg_oracle_block_norms(n, TF // T, T, _p(_c(G, np.float64), _f64p), _p(out, _f64p))
    return out


def gradnorm_step(loss, loss0, gnorm, w, gamma=1.0, lr=0.025):
    """One GradNorm weight update.  -> (meta-loss before the step, new weights)."""
    loss, loss0, gnorm = (_c(np.asarray(a, dtype=np.float64), np.float64) for a in (loss, loss0, gnorm))
    w = _c(np.array(w, dtype=np.float64), np.float64)
    meta = _load().e2eg_oracle_gradnorm_step(w.size, _p(loss, _f64p), _p(loss0, _f64p), _p(gnorm, _f64p),
                                             float(gamma), float(lr), _p(w, _f64p))
    return float(meta), w


def edge_values(n_users, users, items, weights, row_ptr, col_idx):
    """Values of the stored entries of the weighted A~: 1 on the diagonal, the edge weight both
    ways; a repeated pair keeps its largest weight."""
    users, items = _c(users, np.int32), _c(items, np.int32)
    weights = _c(weights, np.float64)
    row_ptr, col_idx = _c(row_ptr, np.int64), _c(col_idx, np.int32)
    val = np.empty(col_idx.size, dtype=np.float64)
    _load().e2eg_oracle_edge_values(n_users, users.size, _p(users, _i32p), _p(items, _i32p), _p(weights, _f64p),
                                    row_ptr.size - 1, _p(row_ptr, _i64p), _p(col_idx, _i32p), _p(val, _f64p))
    return val


def weighted_degrees(row_ptr, val):
    row_ptr, val = _c(row_ptr, np.int64), _c(val, np.float64)
    deg = np.empty(row_ptr.size - 1, dtype=np.float64)
    _load().e2eg_oracle_weighted_degrees(deg.size, _p(row_ptr, _i64p), _p(val, _f64p), _p(deg, _f64p))
    return deg


def propagate_layer_weighted(row_ptr, col_idx, val, X, transposed=False):
    """A^ X (or A^T X) for the weighted operator A^_ij = val_ij / sqrt(d~_i d~_j)."""
    row_ptr, col_idx, val = _c(row_ptr, np.int64), _c(col_idx, np.int32), _c(val, np.float64)
    X = as_f64(X)
    n, F = X.shape
    deg = weighted_degrees(row_ptr, val)
    Y = np.empty_like(X)
    fn = _load().e2eg_oracle_propagate_layer_weighted_transposed if transposed else _load().e2eg_oracle_propagate_layer_weighted
    fn(n, _p(row_ptr, _i64p), _p(col_idx, _i32p), _p(val, _f64p), _p(deg, _f64p), F, _p(X, _f64p), _p(Y, _f64p))
    return Y


def propagate_weighted(row_ptr, col_idx, val, X0, K, transposed=False):
    """K layers of the weighted operator (forward: A^, backward: A^T); -> the last layer."""
    H = as_f64(X0)
    for _ in range(K):
        H = propagate_layer_weighted(row_ptr, col_idx, val, H, transposed)
    return H


# ------------------------------------------------------------------ importance sampling (Section 4.1)
def philox4x32_10(counter, key):
    """One block of Philox4x32-10: counter (4 words), key (2 words) -> 4 words."""
    c, k = _c(counter, np.uint32), _c(key, np.uint32)
    out = np.empty(4, dtype=np.uint32)
    _load().e2eg_oracle_philox4x32_10(_p(c, _u32p), _p(k, _u32p), _p(out, _u32p))
    return out


def sampling_weights(val, beta):
    """w^beta per stored entry, the numerator of the sampling probability; 0 where w is not > 0."""
    val = _c(val, np.float64)
    p = np.empty_like(val)
    _load().e2eg_oracle_sampling_weights(val.size, _p(val, _f64p), float(beta), _p(p, _f64p))
    return p


def sampling_table(row_ptr, col_idx, p):
    """Integer weights q (uint64 [nnz]) of every row's sampling distribution; `p` is taken in float32,
    the precision in which the scaling to integers is decided."""
    row_ptr, col_idx, p = _c(row_ptr, np.int64), _c(col_idx, np.int32), _c(p, np.float32)
    if p.size != col_idx.size or row_ptr[-1] != col_idx.size:
        raise ValueError("one weight per stored entry is needed")
    q = np.empty(col_idx.size, dtype=np.uint64)
    _load().e2eg_oracle_sampling_table(row_ptr.size - 1, _p(row_ptr, _i64p), _p(col_idx, _i32p), _p(p, _f32p),
                                       _p(q, _u64p))
    return q


def sample_picks(row_ptr, col_idx, q, seeds, fanout, seed):
    """-> (hop_of [n], src, dst, entry): every pick of the multi-hop sampler in its defined order."""
    row_ptr, col_idx, q = _c(row_ptr, np.int64), _c(col_idx, np.int32), _c(q, np.uint64)
    seeds, fanout = _c(seeds, np.int32), _c(fanout, np.int32)
    n = row_ptr.size - 1
    cap, width = 0, seeds.size
    for k in fanout:
        width = min(width * int(k), n * int(k))
        cap += width
    hop_of = np.empty(n, dtype=np.int32)
    src, dst = np.empty(cap, dtype=np.int32), np.empty(cap, dtype=np.int32)
    entry = np.empty(cap, dtype=np.int64)
    m = _load().e2eg_oracle_sample_subgraph(n, _p(row_ptr, _i64p), _p(col_idx, _i32p), _p(q, _u64p), seeds.size,
                                            _p(seeds, _i32p), fanout.size, _p(fanout, _i32p), int(seed),
                                            _p(hop_of, _i32p), _p(src, _i32p), _p(dst, _i32p), _p(entry, _i64p), cap)
    assert m <= cap
    return hop_of, src[:m].copy(), dst[:m].copy(), entry[:m].copy()


def sample_subgraph(n_users, row_ptr, col_idx, q, seeds, fanout, seed):
    """The sampled subgraph in local numbering: nodes of the subgraph in ascending global id (users
    come first because they do in the parent), every pick as a (local user, local item) pair in pick
    order, and the index of the parent's stored entry it came from.
    -> dict(nodes, n_users, n_items, users, items, entry, hop_of)"""
    hop_of, src, dst, entry = sample_picks(row_ptr, col_idx, q, seeds, fanout, seed)
    nodes = np.nonzero(hop_of)[0].astype(np.int32)
    nu = int(np.searchsorted(nodes, n_users))
    user_end = np.where(src < n_users, src, dst)      # an edge joins a user and an item
    item_end = np.where(src < n_users, dst, src)
    assert (user_end < n_users).all() and (item_end >= n_users).all()
    return dict(nodes=nodes, n_users=nu, n_items=int(nodes.size - nu),
                users=np.searchsorted(nodes, user_end).astype(np.int32),
                items=(np.searchsorted(nodes, item_end) - nu).astype(np.int32), entry=entry, hop_of=hop_of)
