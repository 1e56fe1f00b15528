"""Buffer management around the C ABI: torch owns device memory and the stream, libe2eg.so does
the work.  Nothing here computes; every function sizes buffers, calls one entry point of
`binding` and hands the tensors back."""
from __future__ import annotations

from dataclasses import dataclass

import torch

from . import binding as B


def _require_gpu():
    if not torch.cuda.is_available():
        raise RuntimeError("paper_2511_20564_amd needs a GPU: there is no CPU implementation")
    B.load_library()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _bytes(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return B.E2EG_F32
    if t.dtype == torch.bfloat16:
        return B.E2EG_BF16
    raise TypeError(f"unsupported feature dtype {t.dtype}")


@dataclass
class Graph:
    """CSR structure of A~ with its degree scaling and launch schedule, all on the device."""
    n_users: int
    n_items: int
    n: int
    nnz: int
    row_ptr: torch.Tensor      # int32 [n+1]
    col_idx: torch.Tensor      # int32 [nnz]
    deg: torch.Tensor          # int32 [n]
    dinv_sqrt: torch.Tensor    # float32 [n]
    sched: torch.Tensor        # uint8, opaque
    val: torch.Tensor | None = None    # float32 [nnz]: entry values of a weighted graph
    deg_w: torch.Tensor | None = None  # float32 [n]: d~ of a weighted graph (then `deg` is the row length)


def normalize(n: int, nnz: int, row_ptr: torch.Tensor, col_idx: torch.Tensor):
    """e2eg_normalize on an existing CSR -> (deg, dinv_sqrt, sched)."""
    _require_gpu()
    dev = row_ptr.device
    deg = torch.empty(n, dtype=torch.int32, device=dev)
    dinv = torch.empty(n, dtype=torch.float32, device=dev)
    sched = _bytes(B.e2eg_sched_bytes(n, nnz), dev)
    ws = _bytes(B.e2eg_normalize_workspace_bytes(n, nnz), dev)
    B.e2eg_normalize(n, nnz, row_ptr, col_idx, deg, dinv, sched, None, ws, None, _stream())
    return deg, dinv, sched


def check_symmetric(sched: torch.Tensor) -> None:
    """e2eg_sched_check_symmetric: raises if the transposed entry points cannot run on `sched`."""
    _require_gpu()
    B.e2eg_sched_check_symmetric(sched, _stream())


def build_graph(n_users: int, n_items: int, users: torch.Tensor, items: torch.Tensor,
                add_self_loops: bool = True) -> Graph:
    """e2eg_build_csr followed by e2eg_normalize.  `users`/`items`: int32 device tensors."""
    _require_gpu()
    assert users.dtype == torch.int32 and items.dtype == torch.int32 and users.is_cuda and items.is_cuda
    assert users.is_contiguous() and items.is_contiguous() and users.numel() == items.numel()
    dev = users.device
    n = n_users + n_items
    n_edges = users.numel()
    flags = B.E2EG_ADD_SELF_LOOPS if add_self_loops else 0
    cap = 2 * n_edges + n
    row_ptr = torch.empty(n + 1, dtype=torch.int32, device=dev)
    col = torch.empty(max(cap, 1), dtype=torch.int32, device=dev)
    ws = _bytes(B.e2eg_build_csr_workspace_bytes(n_users, n_items, n_edges), dev)
    nnz = B.e2eg_build_csr(n_users, n_items, n_edges, users, items, flags, row_ptr, col, cap, ws, None, _stream())
    del ws
    col_idx = col[:nnz]
    deg, dinv, sched = normalize(n, nnz, row_ptr, col_idx)
    return Graph(n_users, n_items, n, nnz, row_ptr, col_idx, deg, dinv, sched)


def normalize_weighted(n: int, nnz: int, row_ptr: torch.Tensor, col_idx: torch.Tensor, val: torch.Tensor):
    """e2eg_normalize_weighted on an existing CSR with values -> (deg, deg_w, dinv_sqrt, sched)."""
    _require_gpu()
    assert val.dtype == torch.float32 and val.is_contiguous() and val.numel() >= nnz
    dev = row_ptr.device
    deg = torch.empty(n, dtype=torch.int32, device=dev)
    deg_w = torch.empty(n, dtype=torch.float32, device=dev)
    dinv = torch.empty(n, dtype=torch.float32, device=dev)
    sched = _bytes(B.e2eg_sched_weighted_bytes(n, nnz), dev)
    ws = _bytes(B.e2eg_normalize_workspace_bytes(n, nnz), dev)
    B.e2eg_normalize_weighted(n, nnz, row_ptr, col_idx, val, deg, deg_w, dinv, sched, None, ws, None, _stream())
    return deg, deg_w, dinv, sched


def build_weighted_graph(n_users: int, n_items: int, users: torch.Tensor, items: torch.Tensor,
                         weights: torch.Tensor) -> Graph:
    """e2eg_build_csr (with self-loops), e2eg_edge_weights, e2eg_normalize_weighted."""
    _require_gpu()
    assert users.dtype == torch.int32 and items.dtype == torch.int32 and weights.dtype == torch.float32
    assert users.is_cuda and items.is_cuda and weights.is_cuda
    assert users.is_contiguous() and items.is_contiguous() and weights.is_contiguous()
    assert users.numel() == items.numel() == weights.numel()
    dev = users.device
    n = n_users + n_items
    n_edges = users.numel()
    cap = 2 * n_edges + n
    row_ptr = torch.empty(n + 1, dtype=torch.int32, device=dev)
    col = torch.empty(max(cap, 1), dtype=torch.int32, device=dev)
    ws = _bytes(B.e2eg_build_csr_workspace_bytes(n_users, n_items, n_edges), dev)
    nnz = B.e2eg_build_csr(n_users, n_items, n_edges, users, items, B.E2EG_ADD_SELF_LOOPS, row_ptr, col, cap, ws,
                           None, _stream())
    del ws
    col_idx = col[:nnz]
    val = torch.empty(max(nnz, 1), dtype=torch.float32, device=dev)[:nnz]
    B.e2eg_edge_weights(n_users, n_items, n_edges, users, items, weights, nnz, row_ptr, col_idx, val, _stream())
    deg, deg_w, dinv, sched = normalize_weighted(n, nnz, row_ptr, col_idx, val)
    return Graph(n_users, n_items, n, nnz, row_ptr, col_idx, deg, dinv, sched, val, deg_w)


def sampler_table(g: Graph, beta: float = 1.0, p: torch.Tensor | None = None) -> torch.Tensor:
    """The sampling table of a weighted graph: e2eg_sampling_weights (unless `p`, float32 [nnz], is
    given) and e2eg_sampler_prepare."""
    _require_gpu()
    dev = g.row_ptr.device
    if p is None:
        assert g.val is not None
        p = torch.empty(max(g.nnz, 1), dtype=torch.float32, device=dev)
        B.e2eg_sampling_weights(g.nnz, g.val, float(beta), p, _stream())
    assert p.dtype == torch.float32 and p.is_contiguous() and p.numel() >= g.nnz
    table = _bytes(B.e2eg_sampler_table_bytes(g.nnz), dev)
    ws = _bytes(B.e2eg_sampler_prepare_workspace_bytes(g.n, g.nnz), dev)
    B.e2eg_sampler_prepare(g.n, g.nnz, g.row_ptr, g.col_idx, p, table, None, ws, None, _stream())
    return table


def sample_subgraph(g: Graph, table: torch.Tensor, seeds: torch.Tensor, fanout, seed: int,
                    with_weights: bool = True, ws: torch.Tensor | None = None) -> dict:
    """e2eg_sample_subgraph -> dict(nodes, n_users, n_items, users, items, weights): global ids of the
    local nodes, and the picks as local (user, item) pairs (with the parent's values)."""
    _require_gpu()
    assert seeds.dtype == torch.int32 and seeds.is_cuda and seeds.is_contiguous()
    dev = g.row_ptr.device
    n_seeds = seeds.numel()
    cap = B.e2eg_sample_capacity(g.n, n_seeds, fanout)
    node_cap = min(g.n, n_seeds + cap)
    nodes = torch.empty(max(node_cap, 1), dtype=torch.int32, device=dev)
    eu = torch.empty(max(cap, 1), dtype=torch.int32, device=dev)
    ei = torch.empty(max(cap, 1), dtype=torch.int32, device=dev)
    ew = torch.empty(max(cap, 1), dtype=torch.float32, device=dev) if with_weights and g.val is not None else None
    if ws is None:
        ws = _bytes(B.e2eg_sample_subgraph_workspace_bytes(g.n, n_seeds, fanout), dev)
    nu, ni, ne = B.e2eg_sample_subgraph(g.n_users, g.n, g.nnz, g.row_ptr, g.col_idx, table,
                                        g.val if ew is not None else None, n_seeds, seeds, fanout, seed, nodes,
                                        node_cap, eu, ei, ew, cap, ws, None, _stream())
    return dict(nodes=nodes[:nu + ni], n_users=nu, n_items=ni, users=eu[:ne], items=ei[:ne],
                weights=ew[:ne] if ew is not None else None)


def propagate_workspace(g: Graph, dtype: torch.dtype, F: int, K: int) -> torch.Tensor:
    code = B.E2EG_F32 if dtype == torch.float32 else B.E2EG_BF16
    return _bytes(B.e2eg_propagate_workspace_bytes(g.n, g.nnz, code, F, K), g.row_ptr.device)


def propagate_fwd(g: Graph, X0: torch.Tensor, K: int, all_layers: bool = False, out: torch.Tensor | None = None,
                  ws: torch.Tensor | None = None) -> torch.Tensor:
    """H(K) as [n, F], or all of H(1..K) as [K, n, F] when all_layers."""
    _require_gpu()
    n, F = X0.shape
    assert n == g.n and X0.stride(1) == 1
    if out is None:
        out = torch.empty((K, n, F) if all_layers else (n, F), dtype=X0.dtype, device=X0.device)
    if ws is None:
        ws = propagate_workspace(g, X0.dtype, F, K)
    fn = B.e2eg_propagate_fwd if g.val is None else B.e2eg_propagate_weighted_fwd
    fn(g.n, g.nnz, g.row_ptr, g.col_idx, g.dinv_sqrt, g.sched, _dtype_code(X0), F, K,
       X0, X0.stride(0), out, F, n * F if all_layers else 0, ws, None, _stream())
    return out


def propagate_bwd(g: Graph, gXK: torch.Tensor, K: int, g_layers: torch.Tensor | None = None,
                  out: torch.Tensor | None = None, ws: torch.Tensor | None = None,
                  g_shared: torch.Tensor | None = None) -> torch.Tensor:
    """dL/dH(0) from dL/dH(K) and optional direct terms: `g_layers`, dL/dH(1..K-1) as [K-1, n, F],
    or `g_shared`, one [n, F] array that is the direct term of every layer 0..K-1."""
    _require_gpu()
    n, F = gXK.shape
    assert n == g.n and gXK.stride(1) == 1
    if out is None:
        out = torch.empty((n, F), dtype=gXK.dtype, device=gXK.device)
    if ws is None:
        ws = propagate_workspace(g, gXK.dtype, F, K)
    stride = 0
    if g_layers is not None:
        assert g_layers.shape == (K - 1, n, F) and g_layers.is_contiguous() and gXK.stride(0) == F
        stride = n * F
    if g_shared is not None:
        assert g_layers is None and g_shared.shape == (n, F) and g_shared.is_contiguous() and gXK.stride(0) == F
        g_layers = g_shared
    fn = B.e2eg_propagate_bwd if g.val is None else B.e2eg_propagate_weighted_bwd
    fn(g.n, g.nnz, g.row_ptr, g.col_idx, g.dinv_sqrt, g.sched, _dtype_code(gXK), F, K,
       gXK, gXK.stride(0), g_layers, stride, out, F, ws, None, _stream())
    return out


def layer_transform_fwd(P: torch.Tensor, W: torch.Tensor, relu: bool = True) -> torch.Tensor:
    _require_gpu()
    n, Fin = P.shape
    Fout = W.shape[1]
    assert W.shape[0] == Fin and P.is_contiguous() and W.is_contiguous()
    H = torch.empty((n, Fout), dtype=P.dtype, device=P.device)
    code = _dtype_code(P)
    ws = _bytes(B.e2eg_layer_transform_workspace_bytes(B.E2EG_TRANSFORM_FWD, n, Fin, Fout, code), P.device)
    B.e2eg_layer_transform(B.E2EG_TRANSFORM_FWD, n, Fin, Fout, code, int(relu), P, W, H, None, None, None, ws, None,
                           _stream())
    return H


def layer_transform_bwd(P: torch.Tensor, W: torch.Tensor, H: torch.Tensor, gH: torch.Tensor, relu: bool = True):
    """-> (dP [n, Fin] in the storage dtype, dW [Fin, Fout] float32)."""
    _require_gpu()
    n, Fin = P.shape
    Fout = W.shape[1]
    assert P.is_contiguous() and W.is_contiguous() and H.is_contiguous() and gH.is_contiguous()
    gP = torch.empty((n, Fin), dtype=P.dtype, device=P.device)
    gW = torch.empty((Fin, Fout), dtype=torch.float32, device=P.device)
    code = _dtype_code(P)
    ws = _bytes(B.e2eg_layer_transform_workspace_bytes(B.E2EG_TRANSFORM_BWD, n, Fin, Fout, code), P.device)
    B.e2eg_layer_transform(B.E2EG_TRANSFORM_BWD, n, Fin, Fout, code, int(relu), P, W, H, gH, gP, gW, ws, None,
                           _stream())
    return gP, gW


def readout_mean(X0: torch.Tensor, layers: torch.Tensor) -> torch.Tensor:
    """Y = (X0 + layers[0] + ... + layers[K-1]) / (K + 1); layers is [K, n, F] as propagate_fwd stores it."""
    _require_gpu()
    n, F = X0.shape
    K = layers.shape[0]
    assert layers.shape == (K, n, F) and layers.is_contiguous() and X0.stride(1) == 1 and layers.dtype == X0.dtype
    Y = torch.empty((n, F), dtype=X0.dtype, device=X0.device)
    B.e2eg_readout_mean(n, _dtype_code(X0), F, K, X0, X0.stride(0), layers, F, n * F, Y, F, _stream())
    return Y


def gfae_loss(X: torch.Tensor, Y: torch.Tensor, grad_scale: float = 1.0, want_grad: bool = True):
    """-> (loss as a 1-element float64 device tensor, grad_scale * 2 (Y - X) or None)."""
    _require_gpu()
    n, F = X.shape
    assert Y.shape == (n, F) and X.stride(1) == 1 and Y.stride(1) == 1 and X.dtype == Y.dtype
    loss = torch.empty(1, dtype=torch.float64, device=X.device)
    gY = torch.empty((n, F), dtype=X.dtype, device=X.device) if want_grad else None
    ws = _bytes(B.e2eg_gfae_loss_workspace_bytes(n, F), X.device)
    B.e2eg_gfae_loss(n, _dtype_code(X), F, X, X.stride(0), Y, Y.stride(0), loss, gY, F, float(grad_scale), ws, None,
                     _stream())
    return loss, gY


def aggregate(g: Graph, X: torch.Tensor, mode: int, addend: torch.Tensor | None = None,
              out: torch.Tensor | None = None) -> torch.Tensor:
    """Y = S_out M S_in X (+ addend) over the graph's stored structure; X, addend and out may be
    column slices of wider row-major arrays (stride(1) == 1)."""
    _require_gpu()
    n, F = X.shape
    assert n == g.n and X.stride(1) == 1
    if out is None:
        out = torch.empty((n, F), dtype=X.dtype, device=X.device)
    assert out.shape == (n, F) and out.stride(1) == 1 and out.dtype == X.dtype
    code = _dtype_code(X)
    ws = _bytes(B.e2eg_aggregate_workspace_bytes(g.n, g.nnz, code, F), X.device)
    B.e2eg_aggregate(mode, g.n, g.nnz, g.row_ptr, g.col_idx, g.sched, code, F, X, X.stride(0),
                     addend, addend.stride(0) if addend is not None else 0, out, out.stride(0), ws, None, _stream())
    return out


def block_norms(G: torch.Tensor, T: int) -> torch.Tensor:
    """2-norms of the T column blocks of G [n, T*F] as a float64 device tensor of length T."""
    _require_gpu()
    n, TF = G.shape
    assert TF % T == 0 and G.stride(1) == 1
    norms = torch.empty(T, dtype=torch.float64, device=G.device)
    ws = _bytes(B.e2eg_block_norms_workspace_bytes(n, TF // T, T), G.device)
    B.e2eg_block_norms(n, _dtype_code(G), TF // T, T, G, G.stride(0), norms, ws, None, _stream())
    return norms
