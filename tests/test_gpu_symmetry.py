"""The transposed entry points apply the stored operator itself, which is the transpose the
backward pass needs (Appendix A, the "GNN backprop" factor: multiplication by A^T) only on a
symmetric structure with symmetric values.  e2eg_normalize finds out while it builds the schedule;
these tests check the verdict, the refusal on the device, and that the forward pass still serves
any structure."""
import numpy as np
import pytest
import torch

from parity import assert_close, to_f64
from workloads import make_config, make_edge_weights

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2511_20564_amd.device as d
    d.B.load_library()
    return d


def graph_from_csr(dev, row_ptr, col, val=None):
    n, nnz = row_ptr.size - 1, col.size
    rp = torch.from_numpy(row_ptr.astype(np.int32)).cuda()
    ci = torch.from_numpy(col.astype(np.int32)).cuda()
    if val is None:
        deg, dinv, sched = dev.normalize(n, nnz, rp, ci)
        return dev.Graph(n, 0, n, nnz, rp, ci, deg, dinv, sched)
    v = torch.from_numpy(val.astype(np.float32)).cuda()
    deg, deg_w, dinv, sched = dev.normalize_weighted(n, nnz, rp, ci, v)
    return dev.Graph(n, 0, n, nnz, rp, ci, deg, dinv, sched, v, deg_w)


def test_nonsymmetric_structure_is_refused_by_the_transposed_calls(dev, oracle):
    # row 0 holds column 1 but row 1 does not hold column 0, and so on
    row_ptr = np.array([0, 2, 3, 4, 7], dtype=np.int64)
    col = np.array([1, 3, 0, 3, 0, 1, 2], dtype=np.int32)
    g = graph_from_csr(dev, row_ptr, col)
    with pytest.raises(dev.B.E2egError) as e:
        dev.check_symmetric(g.sched)
    assert e.value.status == dev.B.E2EG_ERR_INVALID_ARG and "(i, j) without (j, i)" in str(e.value)
    rng = np.random.default_rng(7)
    X = rng.standard_normal((4, 8)).astype(np.float32)
    # the forward pass is defined on any structure
    H = dev.propagate_fwd(g, torch.from_numpy(X).cuda(), 2, all_layers=True)
    ref = oracle.propagate_fwd(row_ptr, col, X, 2)
    scale = oracle.propagate_fwd(row_ptr, col, np.abs(X).astype(np.float64), 2)
    for k in range(2):
        assert_close(to_f64(H[k]), ref[k], scale[k], "f32", f"layer {k + 1}")
    # the transposed calls refuse it on the device: nothing but NaN comes back
    for K in (1, 3):
        G = dev.propagate_bwd(g, torch.from_numpy(X).cuda(), K)
        assert bool(torch.isnan(G).all())
    Y = dev.aggregate(g, torch.from_numpy(X).cuda(), dev.B.E2EG_AGG_MEAN_T)
    assert bool(torch.isnan(Y).all())
    Y = dev.aggregate(g, torch.from_numpy(X).cuda(), dev.B.E2EG_AGG_MEAN)
    assert not bool(torch.isnan(Y).any())


def test_one_missing_mirror_entry_in_a_large_structure(dev, oracle):
    c = make_config(2, scale=0.05, features=False)
    row_ptr, col = oracle.build_csr(c["n_users"], c["n_items"], c["users"], c["items"])
    g = graph_from_csr(dev, row_ptr, col)
    dev.check_symmetric(g.sched)                      # as built: symmetric
    # drop one off-diagonal entry of a long row
    r = int(np.argmax(np.diff(row_ptr)))
    e = int(row_ptr[r]) + 3
    assert col[e] != r
    col2 = np.delete(col, e)
    rp2 = row_ptr.copy()
    rp2[r + 1:] -= 1
    g2 = graph_from_csr(dev, rp2, col2)
    with pytest.raises(dev.B.E2egError):
        dev.check_symmetric(g2.sched)
    x = torch.ones(g2.n, 8, device="cuda")
    assert bool(torch.isnan(dev.propagate_bwd(g2, x, 1)).all())
    assert not bool(torch.isnan(dev.propagate_fwd(g2, x, 1)).any())


def test_every_built_graph_is_symmetric(dev):
    for cfg, scale in ((1, 1.0), (2, 0.1), (3, 0.01)):
        c = make_config(cfg, scale=scale, features=False)
        u, i = torch.from_numpy(c["users"]).cuda(), torch.from_numpy(c["items"]).cuda()
        for loops in (True, False):
            g = dev.build_graph(c["n_users"], c["n_items"], u, i, add_self_loops=loops)
            dev.check_symmetric(g.sched)
        w = torch.from_numpy(make_edge_weights(c["users"].size, seed=cfg)).cuda()
        gw = dev.build_weighted_graph(c["n_users"], c["n_items"], u, i, w)
        dev.check_symmetric(gw.sched)
        assert torch.equal(gw.deg, (gw.row_ptr[1:] - gw.row_ptr[:-1]))    # row lengths come from the library


def test_unsymmetric_values_are_refused(dev, oracle):
    c = make_config(1, features=False)
    nu, ni = c["n_users"], c["n_items"]
    row_ptr, col = oracle.build_csr(nu, ni, c["users"], c["items"])
    w = make_edge_weights(c["users"].size, seed=3)
    val = oracle.edge_values(nu, c["users"], c["items"], w.astype(np.float64), row_ptr, col).astype(np.float32)
    g = graph_from_csr(dev, row_ptr, col, val)
    dev.check_symmetric(g.sched)
    bad = val.copy()
    e = int(row_ptr[5]) + 1                            # an off-diagonal entry of user 5
    assert col[e] != 5
    bad[e] = np.nextafter(bad[e], np.float32(np.inf))
    g2 = graph_from_csr(dev, row_ptr, col, bad)
    with pytest.raises(dev.B.E2egError) as err:
        dev.check_symmetric(g2.sched)
    assert "values" in str(err.value)
    x = torch.ones(g2.n, 8, device="cuda")
    assert bool(torch.isnan(dev.propagate_bwd(g2, x, 2)).all())
    assert not bool(torch.isnan(dev.propagate_fwd(g2, x, 2)).any())
