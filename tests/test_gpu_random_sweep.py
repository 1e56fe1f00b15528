"""GPU parity on a seeded sweep of small random graphs: sizes, degree shapes, feature widths,
storage types, depths, with and without self-loops, with and without edge weights, chosen by a
generator so that combinations nobody thought of by hand are run as well.  Each case is checked
element by element against the oracle like the hand-made ones."""
import numpy as np
import pytest
import torch

from parity import assert_close, to_device, to_f64
from workloads import make_edge_weights, make_features

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2511_20564_amd.device as d
    d.B.load_library()
    return d


def random_case(seed):
    rng = np.random.default_rng(1000 + seed)
    nu = int(rng.choice([1, 2, 7, 63, 64, 65, 500, 4095, 4097, 9000, 20000]))
    ni = int(rng.choice([1, 3, 31, 33, 200, 1500]))
    shape = rng.choice(["uniform", "hubs", "sparse", "dense"])
    if shape == "uniform":
        ne = int(rng.integers(0, 6 * (nu + ni)))
        users, items = rng.integers(0, nu, ne), rng.integers(0, ni, ne)
    elif shape == "hubs":       # a few items joined to a large part of the users, the rest sparse
        hubs = int(min(ni, rng.integers(1, 6)))
        parts_u, parts_i = [], []
        for h in range(hubs):
            d = int(rng.integers(1, nu + 1))
            parts_u.append(rng.choice(nu, size=d, replace=False))
            parts_i.append(np.full(d, h))
        ne = int(rng.integers(0, 2 * (nu + ni)))
        parts_u.append(rng.integers(0, nu, ne))
        parts_i.append(rng.integers(0, ni, ne))
        users, items = np.concatenate(parts_u), np.concatenate(parts_i)
    elif shape == "sparse":
        ne = int(rng.integers(0, max(1, (nu + ni) // 3)))
        users, items = rng.integers(0, nu, ne), rng.integers(0, ni, ne)
    else:                       # every pair present (capped)
        uu, ii = np.meshgrid(np.arange(min(nu, 600)), np.arange(min(ni, 200)), indexing="ij")
        users, items = uu.ravel(), ii.ravel()
    dtype = str(rng.choice(["f32", "bf16"]))
    vec = 4 if dtype == "f32" else 8
    F = int(vec * rng.choice([1, 2, 3, 8, 16, 33]))
    return dict(nu=nu, ni=ni, users=users.astype(np.int32), items=items.astype(np.int32), dtype=dtype, F=F,
                K=int(rng.integers(1, 5)), self_loops=bool(rng.integers(0, 4) > 0), weighted=bool(rng.integers(0, 2)),
                shape=str(shape))


@pytest.mark.parametrize("seed", range(40))
def test_random_graph(dev, oracle, seed):
    c = random_case(seed)
    nu, ni, dt, F, K = c["nu"], c["ni"], c["dtype"], c["F"], c["K"]
    n = nu + ni
    u = torch.from_numpy(c["users"]).cuda()
    i = torch.from_numpy(c["items"]).cuda()
    Xh, gh = make_features(n, F, 0.1, seed, dt), make_features(n, F, 1.0, seed + 1, dt)
    X, gY = to_device(Xh, dt), to_device(gh, dt)
    what = f"seed {seed}: {c['shape']} {nu}+{ni} nodes, {c['users'].size} pairs, {dt} F={F} K={K} " \
           f"self_loops={c['self_loops']} weighted={c['weighted']}"
    print(what, flush=True)
    if c["weighted"]:           # the weighted path always carries the self-loop
        w = make_edge_weights(c["users"].size, seed=seed)
        g = dev.build_weighted_graph(nu, ni, u, i, torch.from_numpy(w).cuda())
        row_ptr, col = oracle.build_csr(nu, ni, c["users"], c["items"])
        val = oracle.edge_values(nu, c["users"], c["items"], w.astype(np.float64), row_ptr, col)
        assert np.array_equal(g.col_idx.cpu().numpy(), col) and np.array_equal(g.val.cpu().numpy(), val.astype(np.float32))
        ref = oracle.propagate_weighted(row_ptr, col, val, Xh, K)
        scale = oracle.propagate_weighted(row_ptr, col, val, np.abs(oracle.as_f64(Xh)), K)
        refb = oracle.propagate_weighted(row_ptr, col, val, gh, K, transposed=True)
        scaleb = oracle.propagate_weighted(row_ptr, col, val, np.abs(oracle.as_f64(gh)), K, transposed=True)
    else:
        g = dev.build_graph(nu, ni, u, i, add_self_loops=c["self_loops"])
        row_ptr, col = oracle.build_csr(nu, ni, c["users"], c["items"], add_self_loops=c["self_loops"])
        assert np.array_equal(g.row_ptr.cpu().numpy().astype(np.int64), row_ptr) and np.array_equal(g.col_idx.cpu().numpy(), col)
        ref = oracle.propagate_fwd(row_ptr, col, Xh, K)[K - 1]
        scale = oracle.propagate_fwd(row_ptr, col, np.abs(oracle.as_f64(Xh)), K)[K - 1]
        refb = oracle.propagate_bwd(row_ptr, col, gh, K)
        scaleb = oracle.propagate_bwd(row_ptr, col, np.abs(oracle.as_f64(gh)), K)
    H = dev.propagate_fwd(g, X, K)
    G0 = dev.propagate_bwd(g, gY, K)
    torch.cuda.synchronize()
    assert_close(to_f64(H), ref, scale, dt, what + " fwd")
    assert_close(to_f64(G0), refb, scaleb, dt, what + " bwd")
