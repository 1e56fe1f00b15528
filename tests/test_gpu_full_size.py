"""GPU parity at the stated sizes, in the launch configuration bench.py times.

 * 50 M-edge graph: CSR bit-exact against the oracle's, all K layers forward and the backward
   against the full fp64 oracle.
 * the sampled mini-batch drawn from that graph: staged pipeline checks.
 * 500 M-edge graph: degrees / row_ptr bit-exact in full; column lists bit-exact and every layer
   (teacher-forced from the GPU's previous layer) within tolerance on sampled rows computed one
   by one; plus properties that hold at any size: the D~^1/2 1 fixed point and the adjoint
   identity <A^ x, g> = <x, A^T g> evaluated on the GPU's outputs.
"""
import time

import numpy as np
import pytest
import torch

from conftest import progress
from parity import TOL, assert_close, to_device, to_f64
from test_gpu_transform import run_minibatch
from workloads import make_config

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2511_20564_amd.device as d
    d.B.load_library()
    return d


def test_config3_full(dev, oracle):
    t0 = time.time()
    c = make_config(3)
    progress(f"config 3 generated ({time.time() - t0:.0f}s)")
    K, dt = c["K"], c["dtype"]
    u = torch.from_numpy(c["users"]).cuda()
    i = torch.from_numpy(c["items"]).cuda()
    g = dev.build_graph(c["n_users"], c["n_items"], u, i)
    del u, i
    row_ptr, col = oracle.build_csr(c["n_users"], c["n_items"], c["users"], c["items"])
    progress(f"oracle CSR built ({time.time() - t0:.0f}s)")
    assert g.nnz == col.size == 2 * c["n_edges"] + c["n"]
    assert np.array_equal(g.row_ptr.cpu().numpy().astype(np.int64), row_ptr)
    assert np.array_equal(g.col_idx.cpu().numpy(), col)
    deg, dinv = oracle.normalize(row_ptr)
    assert np.array_equal(g.deg.cpu().numpy().astype(np.int64), deg)
    X0, gY = to_device(c["X0"], dt), to_device(c["gY"], dt)
    H = dev.propagate_fwd(g, X0, K, all_layers=True)
    HK = dev.propagate_fwd(g, X0, K)                      # the call bench.py times
    gX0 = dev.propagate_bwd(g, gY, K)
    torch.cuda.synchronize()
    assert torch.equal(H[K - 1], HK)
    ref = oracle.propagate_fwd(row_ptr, col, c["X0"], K)
    progress(f"oracle forward done ({time.time() - t0:.0f}s)")
    scale = oracle.propagate_fwd(row_ptr, col, np.abs(oracle.as_f64(c["X0"])), K)
    for k in range(K):
        comp, norm = assert_close(to_f64(H[k]), ref[k], scale[k], dt, f"layer {k + 1}")
        progress(f"config 3 fwd layer {k + 1}: componentwise {comp:.2e} normwise {norm:.2e} (tol {TOL[dt]})")
    del ref, scale, H
    refb = oracle.propagate_bwd(row_ptr, col, c["gY"], K)
    progress(f"oracle backward done ({time.time() - t0:.0f}s)")
    scaleb = oracle.propagate_bwd(row_ptr, col, np.abs(oracle.as_f64(c["gY"])), K)
    comp, norm = assert_close(to_f64(gX0), refb, scaleb, dt, "bwd")
    progress(f"config 3 bwd: componentwise {comp:.2e} normwise {norm:.2e} ({time.time() - t0:.0f}s)")


def test_config4_full(dev, oracle):
    t0 = time.time()
    c = make_config(4)
    progress(f"config 4 sampled: {c['n_users']} users + {c['n_items']} items, {c['n_edges']} edges "
             f"({time.time() - t0:.0f}s)")
    run_minibatch(dev, oracle, c)
    progress(f"config 4 pipeline ok ({time.time() - t0:.0f}s)")


def test_config5_sampled(dev, oracle):
    t0 = time.time()
    c = make_config(5, features=False)
    nu, ni, n, E = c["n_users"], c["n_items"], c["n"], c["n_edges"]
    F, K = c["F"], c["K"]
    progress(f"config 5 generated: E={E} ({time.time() - t0:.0f}s)")
    users, items = c["users"], c["items"]
    u = torch.from_numpy(users).cuda()
    i = torch.from_numpy(items).cuda()
    g = dev.build_graph(nu, ni, u, i)
    torch.cuda.synchronize()
    del u, i
    progress(f"GPU CSR built: nnz={g.nnz} ({time.time() - t0:.0f}s)")
    # --- structure, in full: degrees and row_ptr from plain counting of the distinct pairs
    deg = np.concatenate([np.bincount(users, minlength=nu), np.bincount(items, minlength=ni)]).astype(np.int64) + 1
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(deg, out=row_ptr[1:])
    assert g.nnz == 2 * E + n == row_ptr[-1]
    assert np.array_equal(g.deg.cpu().numpy().astype(np.int64), deg)
    assert np.array_equal(g.row_ptr.cpu().numpy().astype(np.int64), row_ptr)
    ref_dinv = (1.0 / np.sqrt(deg.astype(np.float64))).astype(np.float32)
    got_dinv = g.dinv_sqrt.cpu().numpy()
    assert np.abs(got_dinv.view(np.int32).astype(np.int64) - ref_dinv.view(np.int32).astype(np.int64)).max() <= 1
    # --- structure, sampled rows: neighbour lists straight from the edge list
    rng = np.random.default_rng(5)
    top_items = np.argsort(deg[nu:])[-4:] + nu
    rows = np.unique(np.concatenate([rng.integers(0, nu, 150), nu + rng.integers(0, ni, 150), top_items,
                                     [0, nu - 1, nu, n - 1]])).astype(np.int64)
    um = np.isin(users, rows[rows < nu])
    im = np.isin(items, rows[rows >= nu] - nu)
    progress(f"sampled rows located ({time.time() - t0:.0f}s)")
    su, si = users[um].astype(np.int64), items[um].astype(np.int64)
    tu, ti = users[im].astype(np.int64), items[im].astype(np.int64)
    col_host = np.zeros(g.nnz, dtype=np.int32)      # only the sampled rows' ranges are filled
    col_gpu = g.col_idx
    for r in rows:
        if r < nu:
            want = np.concatenate([[r], np.sort(si[su == r]) + nu])
        else:
            want = np.concatenate([np.sort(tu[ti == r - nu]), [r]])
        assert want.size == deg[r]
        got = col_gpu[row_ptr[r]:row_ptr[r + 1]].cpu().numpy()
        assert np.array_equal(got, want.astype(np.int32)), f"row {r}"
        col_host[row_ptr[r]:row_ptr[r + 1]] = want
    # columns strictly ascending inside every row (checked on the device, any size)
    d = (col_gpu[1:] > col_gpu[:-1])
    d[g.row_ptr[1:-1].long() - 1] = True
    assert bool(d.all())
    del d, um, im
    progress(f"structure ok on {rows.size} sampled rows ({time.time() - t0:.0f}s)")
    # --- propagation: synthetic features made on the device from a seed (same values both sides)
    gen = torch.Generator(device="cuda").manual_seed(c["seed"] + 1000)
    X0 = (torch.randn(n, F, device="cuda", generator=gen) * 0.1).to(torch.bfloat16)
    gY = torch.randn(n, F, device="cuda", generator=gen).to(torch.bfloat16)
    H = dev.propagate_fwd(g, X0, K, all_layers=True)
    torch.cuda.synchronize()
    progress(f"GPU forward done ({time.time() - t0:.0f}s)")
    layers = [X0] + [H[k] for k in range(K)]
    for k in range(K):   # teacher forcing: oracle rows from the GPU's previous layer
        Xin = to_f64(layers[k])
        ref = oracle.propagate_rows(row_ptr, col_host, Xin, rows)
        sc = oracle.propagate_rows(row_ptr, col_host, np.abs(Xin), rows)
        got = to_f64(layers[k + 1][torch.from_numpy(rows).cuda()])
        comp, norm = assert_close(got, ref, sc, "bf16", f"config 5 layer {k + 1}")
        progress(f"config 5 layer {k + 1} sampled rows: componentwise {comp:.2e} ({time.time() - t0:.0f}s)")
        del Xin
    # --- properties at full size
    gX0 = dev.propagate_bwd(g, gY, K)
    HK = dev.propagate_fwd(g, X0, K)
    torch.cuda.synchronize()
    lhs = (HK.double() * gY.double()).sum().item()
    rhs = (X0.double() * gX0.double()).sum().item()
    denom = (HK.double().abs() * gY.double().abs()).sum().item()
    assert abs(lhs - rhs) <= 2e-2 * denom, (lhs, rhs, denom)      # adjoint identity
    v = g.deg.to(torch.float32).sqrt()[:, None].repeat(1, 8).contiguous()
    out = dev.propagate_fwd(g, v, K, all_layers=True)
    torch.cuda.synchronize()
    for k in range(K):
        assert torch.allclose(out[k], v, rtol=2e-5, atol=0)         # D~^1/2 1 is a fixed point
    progress(f"config 5 adjoint {abs(lhs - rhs) / denom:.2e}, fixed point ok ({time.time() - t0:.0f}s)")
