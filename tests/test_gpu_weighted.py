"""GPU parity of the weighted graph path (Section 3, "Notation": A_ij > 0 carries the strength of
edge (i,j); D~ and A^ are built from those values): entry values, weighted degrees, and the
K-layer propagation forward and backward, each against the oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from parity import assert_close, to_device, to_f64
from workloads import make_config, make_edge_weights, make_features, uniform_bipartite

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2511_20564_amd.device as d
    d.B.load_library()
    return d


def ulps(got, ref):
    return np.abs(got.view(np.int32).astype(np.int64) - ref.view(np.int32).astype(np.int64)).max(initial=0)


def weighted_graph(dev, nu, ni, users, items, weights):
    u = torch.from_numpy(np.ascontiguousarray(users, dtype=np.int32)).cuda()
    i = torch.from_numpy(np.ascontiguousarray(items, dtype=np.int32)).cuda()
    w = torch.from_numpy(np.ascontiguousarray(weights, dtype=np.float32)).cuda()
    g = dev.build_weighted_graph(nu, ni, u, i, w)
    torch.cuda.synchronize()
    return g


def check_values(oracle, g, nu, ni, users, items, weights):
    """Values bit-exact (they are copies of the inputs), d~ and d~^-1/2 to one unit in the last place
    (double sums in another order, then one rounding to float)."""
    row_ptr, col = oracle.build_csr(nu, ni, users, items)
    assert g.nnz == col.size and np.array_equal(g.col_idx.cpu().numpy(), col)
    val = oracle.edge_values(nu, users, items, weights.astype(np.float64), row_ptr, col)
    assert np.array_equal(g.val.cpu().numpy(), val.astype(np.float32))
    assert np.array_equal(val.astype(np.float32).astype(np.float64), val)
    deg = oracle.weighted_degrees(row_ptr, val)
    assert ulps(g.deg_w.cpu().numpy(), deg.astype(np.float32)) <= 1
    assert ulps(g.dinv_sqrt.cpu().numpy(), (1.0 / np.sqrt(deg)).astype(np.float32)) <= 1
    return row_ptr, col, val


def run_weighted(dev, oracle, nu, ni, users, items, weights, dtype, F, K, seed=1):
    n = nu + ni
    g = weighted_graph(dev, nu, ni, users, items, weights)
    row_ptr, col, val = check_values(oracle, g, nu, ni, users, items, weights)
    X0h = make_features(n, F, 0.1, seed, dtype)
    gYh = make_features(n, F, 1.0, seed + 1, dtype)
    H = dev.propagate_fwd(g, to_device(X0h, dtype), K, all_layers=True)
    HK = dev.propagate_fwd(g, to_device(X0h, dtype), K)
    gX0 = dev.propagate_bwd(g, to_device(gYh, dtype), K)
    torch.cuda.synchronize()
    ref, scale = oracle.as_f64(X0h), np.abs(oracle.as_f64(X0h))     # the values are >= 0: |A^| = A^
    worst = 0.0
    for k in range(K):
        ref = oracle.propagate_layer_weighted(row_ptr, col, val, ref)
        scale = oracle.propagate_layer_weighted(row_ptr, col, val, scale)
        comp, _ = assert_close(to_f64(H[k]), ref, scale, dtype, f"weighted fwd layer {k + 1}")
        worst = max(worst, comp)
    assert_close(to_f64(HK), ref, scale, dtype, "weighted fwd, last layer only")
    refb = oracle.propagate_weighted(row_ptr, col, val, gYh, K, transposed=True)
    scaleb = oracle.propagate_weighted(row_ptr, col, val, np.abs(oracle.as_f64(gYh)), K, transposed=True)
    comp, _ = assert_close(to_f64(gX0), refb, scaleb, dtype, "weighted bwd")
    return g, max(worst, comp)


@pytest.mark.parametrize("cfg,scale", [(1, 1.0), (2, 0.2), (3, 0.02)])
def test_weighted_configs(dev, oracle, cfg, scale):
    c = make_config(cfg, scale=scale, features=False)
    w = make_edge_weights(c["users"].size, seed=cfg)
    _, worst = run_weighted(dev, oracle, c["n_users"], c["n_items"], c["users"], c["items"], w, c["dtype"], c["F"], c["K"])
    print(f"weighted config {cfg} x{scale}: worst componentwise error {worst:.3e}")


def test_repeated_pairs_and_unusable_weights(dev, oracle):
    """A pair listed several times keeps its largest weight whatever the order; weights that are
    zero, negative or NaN leave the entry at 0 (the edge stays in the structure)."""
    nu, ni, ne = 500, 200, 6000
    users, items = uniform_bipartite(nu, ni, ne, seed=5)
    w = make_edge_weights(ne, seed=6)
    w[::7] = 0.0
    w[1::11] = -2.0
    w[2::13] = np.nan
    rep = np.arange(0, ne, 3)
    users = np.concatenate([users, users[rep], users[rep[::2]]])
    items = np.concatenate([items, items[rep], items[rep[::2]]])
    w = np.concatenate([w, make_edge_weights(rep.size, seed=7), make_edge_weights(rep[::2].size, seed=8)]).astype(np.float32)
    g = weighted_graph(dev, nu, ni, users, items, w)
    check_values(oracle, g, nu, ni, users, items, w)
    order = np.random.default_rng(9).permutation(users.size)
    g2 = weighted_graph(dev, nu, ni, users[order], items[order], w[order])
    assert torch.equal(g.val, g2.val) and torch.equal(g.deg_w, g2.deg_w)


@pytest.mark.parametrize("dtype,F", [("f32", 24), ("bf16", 64), ("bf16", 1024)])
def test_weighted_long_rows(dev, oracle, dtype, F):
    """Rows of every class of the schedule (thousands of entries cut by column window and by length,
    129..512 in one piece, short ones) so that each gather loop runs with values."""
    rng = np.random.default_rng(F)
    nu, ni = 12000, 300
    deg = np.concatenate([np.full(4, 9000), np.full(40, 700), np.full(60, 300), np.full(ni - 104, 12)])
    items = np.repeat(np.arange(ni), deg)
    users = np.concatenate([rng.choice(nu, size=d, replace=False) for d in deg])
    heavy = rng.choice(nu, size=8, replace=False)
    users = np.concatenate([users, np.repeat(heavy, ni)]).astype(np.int32)
    items = np.concatenate([items, np.tile(np.arange(ni), 8)]).astype(np.int32)
    w = make_edge_weights(users.size, seed=F)
    run_weighted(dev, oracle, nu, ni, users, items, w, dtype, F, K=2)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_unit_weights_equal_the_unweighted_path(dev, dtype):
    """With every weight 1 the weighted operator is the unweighted one, and since 1*x + acc rounds
    like x + acc the two GPU paths agree bit for bit."""
    c = make_config(2, scale=0.1, features=False)
    nu, ni, n, F, K = c["n_users"], c["n_items"], c["n"], 64, 3
    u = torch.from_numpy(c["users"]).cuda()
    i = torch.from_numpy(c["items"]).cuda()
    g0 = dev.build_graph(nu, ni, u, i)
    g1 = dev.build_weighted_graph(nu, ni, u, i, torch.ones(u.numel(), dtype=torch.float32, device="cuda"))
    assert torch.equal(g0.dinv_sqrt, g1.dinv_sqrt)
    assert torch.equal(g0.deg.to(torch.float32), g1.deg_w)
    X0 = to_device(make_features(n, F, 0.1, 1, dtype), dtype)
    gY = to_device(make_features(n, F, 1.0, 2, dtype), dtype)
    assert torch.equal(dev.propagate_fwd(g0, X0, K, all_layers=True), dev.propagate_fwd(g1, X0, K, all_layers=True))
    assert torch.equal(dev.propagate_bwd(g0, gY, K), dev.propagate_bwd(g1, gY, K))


def test_weighted_graph_without_edges(dev):
    """Only the diagonal is stored: d~ = 1 and A^ is the identity."""
    e = torch.zeros(0, dtype=torch.int32, device="cuda")
    g = dev.build_weighted_graph(40, 9, e, e, torch.zeros(0, dtype=torch.float32, device="cuda"))
    assert g.nnz == 49 and torch.equal(g.val, torch.ones(49, device="cuda")) and torch.equal(g.deg_w, torch.ones(49, device="cuda"))
    X0 = to_device(make_features(49, 8, 1.0, 3, "f32"), "f32")
    assert torch.equal(dev.propagate_fwd(g, X0, 2), X0)
