"""GPU parity: libe2eg.so (through its C ABI) against the CPU oracle, same seeded inputs.

Integer results (CSR structure, degrees) must be bit-exact.  Features: max error relative to
the abs-sum scale <= 1e-5 (fp32) / 2e-2 (bf16 storage, fp32 accumulate).
"""
import numpy as np
import pytest
import torch

from parity import TOL, assert_close, errors, to_device, to_f64
from workloads import f32_to_bf16_bits, make_config, make_features, uniform_bipartite

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2511_20564_amd.device as d
    d.B.load_library()
    return d


def gpu_graph(dev, nu, ni, users, items, self_loops=True):
    u = torch.from_numpy(np.ascontiguousarray(users, dtype=np.int32)).cuda()
    i = torch.from_numpy(np.ascontiguousarray(items, dtype=np.int32)).cuda()
    g = dev.build_graph(nu, ni, u, i, add_self_loops=self_loops)
    torch.cuda.synchronize()
    return g


def check_structure(oracle, g, nu, ni, users, items, self_loops=True):
    row_ptr, col = oracle.build_csr(nu, ni, users, items, add_self_loops=self_loops)
    assert g.nnz == col.size
    assert np.array_equal(g.row_ptr.cpu().numpy().astype(np.int64), row_ptr)
    assert np.array_equal(g.col_idx.cpu().numpy(), col)
    deg, dinv = oracle.normalize(row_ptr)
    assert np.array_equal(g.deg.cpu().numpy().astype(np.int64), deg)
    ref = dinv.astype(np.float32)                     # (float)(1/sqrt((double)d))
    got = g.dinv_sqrt.cpu().numpy()
    ulp = np.abs(got.view(np.int32).astype(np.int64) - ref.view(np.int32).astype(np.int64))
    assert ulp.max(initial=0) <= 1
    return row_ptr, col


# ------------------------------------------------------------------ structure
@pytest.mark.parametrize("cfg,scale", [(1, 1.0), (2, 1.0), (3, 0.02)])
def test_build_csr_configs(dev, oracle, cfg, scale):
    c = make_config(cfg, scale=scale, features=False)
    g = gpu_graph(dev, c["n_users"], c["n_items"], c["users"], c["items"])
    check_structure(oracle, g, c["n_users"], c["n_items"], c["users"], c["items"])


@pytest.mark.parametrize("nu,ni,ne", [(1, 1, 1), (1, 1, 0), (5, 3, 0), (7, 300, 2047), (300, 7, 2049),
                                      (1000, 1, 1000), (1, 1000, 1000), (70000, 66000, 300001)])
@pytest.mark.parametrize("self_loops", [True, False])
def test_build_csr_shapes(dev, oracle, nu, ni, ne, self_loops):
    users, items = uniform_bipartite(nu, ni, ne, seed=nu * 7 + ni)
    if ne > 10:  # repeated pairs collapse
        users = np.concatenate([users, users[: ne // 3]])
        items = np.concatenate([items, items[: ne // 3]])
    g = gpu_graph(dev, nu, ni, users, items, self_loops)
    check_structure(oracle, g, nu, ni, users, items, self_loops)


def test_build_csr_rejects_bad_ids(dev):
    u = torch.tensor([0, 5], dtype=torch.int32).cuda()
    i = torch.tensor([0, 1], dtype=torch.int32).cuda()
    with pytest.raises(dev.B.E2egError) as e:
        dev.build_graph(5, 2, u, i)
    assert e.value.status == dev.B.E2EG_ERR_BAD_INDEX


# ------------------------------------------------------------------ propagation
def run_case(dev, oracle, c, K=None, self_loops=True):
    K = c["K"] if K is None else K
    dt = c["dtype"]
    g = gpu_graph(dev, c["n_users"], c["n_items"], c["users"], c["items"], self_loops)
    row_ptr, col = check_structure(oracle, g, c["n_users"], c["n_items"], c["users"], c["items"], self_loops)
    X0 = to_device(c["X0"], dt)
    gY = to_device(c["gY"], dt)
    # forward, all layers
    H = dev.propagate_fwd(g, X0, K, all_layers=True)
    HK = dev.propagate_fwd(g, X0, K)
    torch.cuda.synchronize()
    ref = oracle.propagate_fwd(row_ptr, col, c["X0"], K)
    scale = oracle.propagate_fwd(row_ptr, col, np.abs(oracle.as_f64(c["X0"])), K)
    worst = 0.0
    for k in range(K):
        comp, _ = assert_close(to_f64(H[k]), ref[k], scale[k], dt, f"fwd layer {k + 1}")
        worst = max(worst, comp)
    assert_close(to_f64(HK), ref[K - 1], scale[K - 1], dt, "fwd last layer only")
    # backward
    gX0 = dev.propagate_bwd(g, gY, K)
    torch.cuda.synchronize()
    refb = oracle.propagate_bwd(row_ptr, col, c["gY"], K)
    scaleb = oracle.propagate_bwd(row_ptr, col, np.abs(oracle.as_f64(c["gY"])), K)
    comp, _ = assert_close(to_f64(gX0), refb, scaleb, dt, "bwd")
    return g, max(worst, comp)


@pytest.mark.parametrize("cfg,scale", [(1, 1.0), (2, 1.0), (3, 0.02), (5, 0.002)])
def test_propagate_configs(dev, oracle, cfg, scale):
    c = make_config(cfg, scale=scale)
    _, worst = run_case(dev, oracle, c)
    print(f"config {cfg} x{scale}: worst componentwise error {worst:.3e} (tol {TOL[c['dtype']]})")


@pytest.mark.parametrize("dtype,F", [("f32", 4), ("f32", 24), ("f32", 64), ("f32", 320), ("bf16", 8), ("bf16", 64),
                                     ("bf16", 200), ("bf16", 1024)])
@pytest.mark.parametrize("K", [1, 4])
def test_propagate_feature_widths(dev, oracle, dtype, F, K):
    nu, ni, ne = 700, 90, 6000        # item rows long enough to be split into segments
    users, items = uniform_bipartite(nu, ni, ne, seed=F + K)
    n = nu + ni
    c = dict(n_users=nu, n_items=ni, users=users, items=items, dtype=dtype, K=K,
             X0=make_features(n, F, 0.1, 1, dtype), gY=make_features(n, F, 1.0, 2, dtype))
    run_case(dev, oracle, c)


@pytest.mark.parametrize("dtype,F,K", [("f32", 8, 3), ("bf16", 16, 2), ("bf16", 8, 1)])
def test_propagate_narrow_rows_on_a_dense_graph(dev, oracle, dtype, F, K):
    """More than 2^20 stored entries and many entries per byte of feature row: the case in which the
    first layer reads pre-scaled rows made by a streaming pass instead of the caller's rows directly
    (the library takes the direct form when 4 nnz < 2 n row-bytes or the graph is small; both forms
    must give the oracle's result)."""
    nu, ni, ne = 40_000, 20_000, 1_200_000
    users, items = uniform_bipartite(nu, ni, ne, seed=17)
    n = nu + ni
    esz = 4 if dtype == "f32" else 2
    assert 2 * ne + n > 1 << 20 and 2 * (2 * ne + n) >= n * F * esz
    c = dict(n_users=nu, n_items=ni, users=users, items=items, dtype=dtype, K=K,
             X0=make_features(n, F, 0.1, 1, dtype), gY=make_features(n, F, 1.0, 2, dtype))
    run_case(dev, oracle, c)


@pytest.mark.parametrize("dtype,F", [("f32", 8), ("f32", 64), ("f32", 320), ("bf16", 16), ("bf16", 128), ("bf16", 1024)])
def test_propagate_long_rows_feature_widths(dev, oracle, dtype, F):
    """Rows of every class at each lane layout: a few items with thousands of neighbours (cut at
    window boundaries and by length), items and users with 129..512 (one wavefront per row) and
    short rows, on more nodes than one window holds."""
    rng = np.random.default_rng(F)
    nu, ni = 12000, 300
    deg = np.concatenate([np.full(4, 9000), np.full(40, 700), np.full(60, 300), np.full(ni - 104, 12)])
    items = np.repeat(np.arange(ni), deg)
    users = np.concatenate([rng.choice(nu, size=d, replace=False) for d in deg])
    heavy = rng.choice(nu, size=8, replace=False)             # a few users with 129..300 items
    hu = np.repeat(heavy, ni)
    hi = np.tile(np.arange(ni), 8)
    users = np.concatenate([users, hu]).astype(np.int32)
    items = np.concatenate([items, hi]).astype(np.int32)
    n = nu + ni
    c = dict(n_users=nu, n_items=ni, users=users, items=items, dtype=dtype, K=2,
             X0=make_features(n, F, 0.1, 1, dtype), gY=make_features(n, F, 1.0, 2, dtype))
    run_case(dev, oracle, c)


def test_identical_addends_in_long_wide_fp32_rows(dev, oracle):
    """The worst case of the fp32 sums: one item joined to thousands of users with one item each and no
    self-loops, so that from the second layer on the item's row adds thousands of IDENTICAL values, and rows
    of 528 bytes, which one lane group sums 512 entries at a time.  Adding a constant to a growing partial
    sum rounds the same way every time: the error grows with the number of terms, not with its root.  Each
    fp32 add loses at most 2^-24 of the partial sum, so a run of 512 loses at most 512 * 2^-24 = 3.1e-5 of
    the abs-sum, runs are added in double, and every layer can add as much again: asserted K * 512 * 2^-24
    (measured 7.2e-6 per layer of such sums, 1.2e-5 after K = 4)."""
    nu, K, F = 9000, 4, 132
    rng = np.random.default_rng(140)
    users = np.unique(rng.integers(0, nu, 15000)).astype(np.int32)
    items = np.zeros(users.size, dtype=np.int32)
    g = dev.build_graph(nu, 1, torch.from_numpy(users).cuda(), torch.from_numpy(items).cuda(), add_self_loops=False)
    row_ptr, col = oracle.build_csr(nu, 1, users, items, add_self_loops=False)
    assert np.array_equal(g.col_idx.cpu().numpy(), col)
    Xh, gh = make_features(nu + 1, F, 0.1, 140, "f32"), make_features(nu + 1, F, 1.0, 141, "f32")
    H = dev.propagate_fwd(g, to_device(Xh, "f32"), K)
    G0 = dev.propagate_bwd(g, to_device(gh, "f32"), K)
    torch.cuda.synchronize()
    bound = K * 512 * 2.0 ** -24
    for got, ref, scale, what in (
            (H, oracle.propagate_fwd(row_ptr, col, Xh, K)[K - 1],
             oracle.propagate_fwd(row_ptr, col, np.abs(oracle.as_f64(Xh)), K)[K - 1], "fwd"),
            (G0, oracle.propagate_bwd(row_ptr, col, gh, K),
             oracle.propagate_bwd(row_ptr, col, np.abs(oracle.as_f64(gh)), K), "bwd")):
        comp, norm = errors(to_f64(got), ref, scale)
        assert comp <= bound and norm <= bound, (what, comp, norm, bound)


def test_propagate_many_tiny_segments(dev, oracle):
    """A thousand popular items that each have one neighbour in every window of the node range and
    a dense run in one: the segment list is mostly one-entry segments, all dealt to one XCD, many
    more than the launch provides workgroups for, so those workgroups go round the list again."""
    rng = np.random.default_rng(11)
    nu, ni = 300_000, 1024
    dense = rng.choice(nu, size=3000, replace=False)
    wins = nu // 8192
    u_parts, i_parts = [], []
    for it in range(ni):
        spread = (np.arange(1, wins) * 8192 + rng.integers(0, 8192, size=wins - 1)).astype(np.int64)
        u = np.unique(np.concatenate([dense, spread[spread < nu]]))
        u_parts.append(u)
        i_parts.append(np.full(u.size, it))
    users = np.concatenate(u_parts).astype(np.int32)
    items = np.concatenate(i_parts).astype(np.int32)
    n, F = nu + ni, 16
    c = dict(n_users=nu, n_items=ni, users=users, items=items, dtype="f32", K=2,
             X0=make_features(n, F, 0.1, 1, "f32"), gY=make_features(n, F, 1.0, 2, "f32"))
    run_case(dev, oracle, c)


@pytest.mark.parametrize("nu,item_degs", [
    (600, [128, 129, 127, 1, 0, 512, 513, 511, 600]),               # the cut-off lengths of the row classes
    (8190, [2, 3, 8190, 5000]),                                     # n just below / at the renumbered block
    (8191, [1, 8191]),
    (8200, [8200, 4096, 513, 513, 513]),                            # two windows, rows crossing the boundary
    (16383, [16383, 9000, 1]),
    (16390, [16390, 700] + [130] * 40),
    (40000, [40000, 20000, 3000, 1025] + [64] * 50),                # five windows, rows of every class
])
def test_propagate_boundary_sizes(dev, oracle, nu, item_degs):
    """Graphs built so that row lengths and node counts sit on the limits the schedule branches
    on: 128/129 and 512/513 entries, node counts around the size of the renumbered block and of
    the column windows."""
    rng = np.random.default_rng(nu)
    ni = len(item_degs)
    users = np.concatenate([rng.choice(nu, size=d, replace=False) for d in item_degs] + [np.zeros(0, np.int64)])
    items = np.repeat(np.arange(ni), item_degs)
    n, F = nu + ni, 16
    c = dict(n_users=nu, n_items=ni, users=users.astype(np.int32), items=items.astype(np.int32), dtype="f32", K=2,
             X0=make_features(n, F, 0.1, 1, "f32"), gY=make_features(n, F, 1.0, 2, "f32"))
    run_case(dev, oracle, c)
    run_case(dev, oracle, c, self_loops=False)


def test_propagate_without_self_loops(dev, oracle):
    nu, ni, ne = 50, 400, 900         # leaves many items without neighbours
    users, items = uniform_bipartite(nu, ni, ne, seed=5)
    n = nu + ni
    c = dict(n_users=nu, n_items=ni, users=users, items=items, dtype="f32", K=2,
             X0=make_features(n, 16, 0.1, 1, "f32"), gY=make_features(n, 16, 1.0, 2, "f32"))
    run_case(dev, oracle, c, self_loops=False)


def test_propagate_no_edges_is_identity(dev):
    n = 37
    g = gpu_graph(dev, 30, 7, np.zeros(0, np.int32), np.zeros(0, np.int32))
    X = torch.randn(n, 16, device="cuda")
    out = dev.propagate_fwd(g, X, 3)
    torch.cuda.synchronize()
    assert torch.allclose(out, X, rtol=1e-6, atol=0)


def test_propagate_strided_input_and_direct_terms(dev, oracle):
    c = make_config(1)
    K = 3
    g = gpu_graph(dev, c["n_users"], c["n_items"], c["users"], c["items"])
    row_ptr, col = oracle.build_csr(c["n_users"], c["n_items"], c["users"], c["items"])
    n, F = c["n"], c["F"]
    wide = torch.zeros(n, F + 32, device="cuda")
    wide[:, :F] = torch.from_numpy(c["X0"]).cuda()
    out = dev.propagate_fwd(g, wide[:, :F], K)           # leading dimension F + 32
    ref = oracle.propagate_fwd(row_ptr, col, c["X0"], K)[-1]
    scale = oracle.propagate_fwd(row_ptr, col, np.abs(c["X0"]).astype(np.float64), K)[-1]
    assert_close(to_f64(out), ref, scale, "f32", "strided fwd")
    direct = [make_features(n, F, 1.0, 70 + k, "f32") for k in range(K - 1)]
    gl = torch.from_numpy(np.stack(direct)).cuda()
    gY = torch.from_numpy(c["gY"]).cuda()
    got = dev.propagate_bwd(g, gY, K, g_layers=gl)
    torch.cuda.synchronize()
    refb = oracle.propagate_bwd(row_ptr, col, c["gY"], K, g_layers=direct)
    scaleb = oracle.propagate_bwd(row_ptr, col, np.abs(c["gY"]), K, g_layers=[np.abs(d) for d in direct])
    assert_close(to_f64(got), refb, scaleb, "f32", "bwd with direct terms")


def test_sqrt_degree_is_a_fixed_point_on_gpu(dev):
    """A^ D~^1/2 1 = D~^1/2 1 at every layer (checked on the GPU's own output)."""
    c = make_config(2, features=False)
    g = gpu_graph(dev, c["n_users"], c["n_items"], c["users"], c["items"])
    v = g.deg.to(torch.float32).sqrt()
    X = v[:, None].repeat(1, 4).contiguous()
    out = dev.propagate_fwd(g, X, 3, all_layers=True)
    torch.cuda.synchronize()
    for k in range(3):
        assert torch.allclose(out[k], X, rtol=2e-5, atol=0)


def test_results_are_reproducible(dev):
    c = make_config(2)
    g = gpu_graph(dev, c["n_users"], c["n_items"], c["users"], c["items"])
    X0 = to_device(c["X0"], "f32")
    a = dev.propagate_fwd(g, X0, 3).clone()
    b = dev.propagate_fwd(g, X0, 3)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
