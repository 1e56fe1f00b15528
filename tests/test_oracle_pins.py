"""Pins for the CPU oracle: it is checked against things that are not itself.

 * a dense A^ assembled literally from the definitions of Section 3 ("Notation"):
   A from the edge set, A~ = A + I, D = diag(A 1), D~ = D + I, A^ = D~^-1/2 A~ D~^-1/2;
 * closed forms that follow from that definition on graphs solvable by hand
   (values in tests/golden/);
 * invariants: symmetry, spectrum in (-1, 1] (L^ = I - A^ is a normalized Laplacian),
   D~^1/2 1 a fixed point;
 * the backward being the transpose (dense A^T G, adjoint identity, finite differences),
   also on a deliberately non-symmetric structure;
 * an independent library evaluation (scipy.sparse);
 * the per-node LightGCN update of Section 3.1 written as python loops (no self-loop variant);
 * GraphSAGE: dense D^-1 A written from the layer's definition, the star's centre, finite differences;
 * layer-mean readout and GFAE loss: a hand-worked single-edge case (tests/golden/), the dense
   mean of powers of A^, numpy's Frobenius norm, finite differences of the whole chain.
"""
import os

import numpy as np
import pytest

from workloads import make_config, uniform_bipartite

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- dense definition
def dense_ahat(n_users, n_items, users, items, self_loops=True):
    """A^ from Section 3 "Notation", dense and literal."""
    n = n_users + n_items
    A = np.zeros((n, n))
    for u, i in zip(users, items):          # A_ij > 0 iff (i,j) in E, undirected
        A[u, n_users + i] = 1.0
        A[n_users + i, u] = 1.0
    I = np.eye(n)
    D = np.diag(A @ np.ones(n))
    if self_loops:
        At, Dt = A + I, D + I
        assert np.array_equal(np.diag(Dt), At @ np.ones(n))   # D + I == diag(A~ 1)
    else:
        At, Dt = A, D
    d = np.diag(Dt)
    s = np.where(d > 0, 1.0 / np.sqrt(np.where(d > 0, d, 1.0)), 0.0)
    return np.diag(s) @ At @ np.diag(s), At


def small_graph(seed, nu=13, ni=9, ne=40, dup=True):
    rng = np.random.default_rng(seed)
    u, i = uniform_bipartite(nu, ni, ne, seed)
    if dup:  # repeated pairs must collapse to one edge
        k = rng.integers(0, ne, size=7)
        u = np.concatenate([u, u[k]])
        i = np.concatenate([i, i[k]])
    return nu, ni, u, i


def relerr(a, b):
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-300)


# ---------------------------------------------------------------- structure
@pytest.mark.parametrize("seed", [1, 2, 3])
@pytest.mark.parametrize("self_loops", [True, False])
def test_csr_matches_dense_pattern(oracle, seed, self_loops):
    nu, ni, u, i = small_graph(seed)
    row_ptr, col = oracle.build_csr(nu, ni, u, i, add_self_loops=self_loops)
    _, At = dense_ahat(nu, ni, u, i, self_loops)
    n = nu + ni
    assert row_ptr[0] == 0 and row_ptr[-1] == col.size == int((At > 0).sum())
    for r in range(n):
        cols = col[row_ptr[r]:row_ptr[r + 1]]
        assert np.array_equal(cols, np.flatnonzero(At[r] > 0))   # ascending, no repeats


def test_csr_structure_config1(oracle):
    c = make_config(1, features=False)
    nu, ni = c["n_users"], c["n_items"]
    n, E = c["n"], c["n_edges"]
    row_ptr, col = oracle.build_csr(nu, ni, c["users"], c["items"])
    assert col.size == 2 * E + n == 43_000
    deg = np.diff(row_ptr)
    assert (deg >= 1).all()
    assert deg[:nu].sum() - nu == E and deg[nu:].sum() - ni == E
    for r in range(n):
        cols = col[row_ptr[r]:row_ptr[r + 1]]
        assert (np.diff(cols) > 0).all()
        if r < nu:   # user row: itself first, then items
            assert cols[0] == r and (cols[1:] >= nu).all()
        else:        # item row: users, itself last
            assert cols[-1] == r and (cols[:-1] < nu).all()
    # structural symmetry
    rows = np.repeat(np.arange(n), deg)
    fwd = set(zip(rows.tolist(), col.tolist()))
    assert all((c_, r_) in fwd for r_, c_ in fwd)


@pytest.mark.parametrize("self_loops", [True, False])
def test_csr_by_row_ranges_is_the_csr(oracle, self_loops):
    """Building the structure range by range gives the rows of the whole structure (and of the dense
    pattern), for ranges inside the users, inside the items, across both, empty and whole."""
    nu, ni, u, i = small_graph(9, nu=17, ni=11, ne=60)
    n = nu + ni
    row_ptr, col = oracle.build_csr(nu, ni, u, i, add_self_loops=self_loops)
    _, At = dense_ahat(nu, ni, u, i, self_loops)
    for lo, hi in [(0, n), (0, 5), (5, nu), (nu - 3, nu + 4), (nu, n), (n - 1, n), (7, 7)]:
        rp, cl = oracle.build_csr_rows(nu, ni, u, i, lo, hi, add_self_loops=self_loops)
        assert rp[0] == 0 and np.array_equal(rp, row_ptr[lo:hi + 1] - row_ptr[lo])
        assert np.array_equal(cl, col[row_ptr[lo]:row_ptr[hi]])
        for r in range(lo, hi):
            assert np.array_equal(cl[rp[r - lo]:rp[r - lo + 1]], np.flatnonzero(At[r] > 0))
    with pytest.raises(ValueError):
        oracle.build_csr_rows(nu, ni, u, i, 3, n + 1)


def test_transposed_rows_to_targets_is_the_dense_transpose(oracle):
    """The backward restricted to target nodes, built up over row ranges, equals rows of A^T G of the
    dense operator -- on a symmetric structure and on one that is not."""
    nu, ni, u, i = small_graph(31, nu=12, ni=10, ne=50)
    n = nu + ni
    Ahat, _ = dense_ahat(nu, ni, u, i)
    row_ptr, col = oracle.build_csr(nu, ni, u, i)
    rng = np.random.default_rng(2)
    G = rng.standard_normal((n, 4))
    targets = np.array([0, 3, nu - 1, nu, nu + 4, n - 1])
    out = np.zeros((targets.size, 4))
    for lo, hi in [(0, 7), (7, nu + 2), (nu + 2, n)]:
        rp, cl = oracle.build_csr_rows(nu, ni, u, i, lo, hi)
        oracle.transposed_to_targets(lo, rp, cl, np.diff(row_ptr), G, targets, out)
    assert relerr(out, (Ahat.T @ G)[targets]) < 1e-13
    # a structure that is not symmetric: the rows of M^T G, not of M G
    row_ptr = np.array([0, 2, 3, 4, 7], dtype=np.int64)
    col = np.array([1, 3, 0, 3, 0, 1, 2], dtype=np.int32)
    length = np.diff(row_ptr)
    M = np.zeros((4, 4))
    for r in range(4):
        for p in range(row_ptr[r], row_ptr[r + 1]):
            M[r, col[p]] = 1.0 / np.sqrt(length[r] * length[col[p]])
    G = rng.standard_normal((4, 3))
    out = np.zeros((3, 3))
    oracle.transposed_to_targets(0, row_ptr[:3], col[:row_ptr[2]], length, G, np.array([0, 1, 3]), out)
    oracle.transposed_to_targets(2, row_ptr[2:] - row_ptr[2], col[row_ptr[2]:], length, G, np.array([0, 1, 3]), out)
    assert relerr(out, (M.T @ G)[[0, 1, 3]]) < 1e-13 and relerr(out, (M @ G)[[0, 1, 3]]) > 1e-2


def test_build_csr_rejects_bad_ids(oracle):
    with pytest.raises(ValueError):
        oracle.build_csr(3, 2, np.array([0, 3]), np.array([0, 1]))
    with pytest.raises(ValueError):
        oracle.build_csr(3, 2, np.array([0, 1]), np.array([0, -1]))


def test_normalize_degrees(oracle):
    nu, ni, u, i = small_graph(5)
    row_ptr, _ = oracle.build_csr(nu, ni, u, i)
    deg, dinv = oracle.normalize(row_ptr)
    _, At = dense_ahat(nu, ni, u, i)
    assert np.array_equal(deg, (At @ np.ones(nu + ni)).astype(np.int64))
    assert np.allclose(dinv * dinv * deg, 1.0, rtol=1e-15)


# ---------------------------------------------------------------- forward vs dense
@pytest.mark.parametrize("seed", [11, 12, 13, 14])
@pytest.mark.parametrize("K", [1, 2, 4])
def test_forward_matches_dense_small(oracle, seed, K):
    nu, ni, u, i = small_graph(seed)
    Ahat, _ = dense_ahat(nu, ni, u, i)
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((nu + ni, 5))
    row_ptr, col = oracle.build_csr(nu, ni, u, i)
    layers = oracle.propagate_fwd(row_ptr, col, X, K)
    ref = X
    for k in range(K):
        ref = Ahat @ ref
        assert relerr(layers[k], ref) < 1e-12


def test_forward_matches_dense_config1(oracle):
    c = make_config(1)
    Ahat, _ = dense_ahat(c["n_users"], c["n_items"], c["users"], c["items"])
    row_ptr, col = oracle.build_csr(c["n_users"], c["n_items"], c["users"], c["items"])
    layers = oracle.propagate_fwd(row_ptr, col, c["X0"], c["K"])
    X = c["X0"].astype(np.float64)
    assert relerr(layers[0], Ahat @ X) < 1e-12
    assert relerr(layers[1], Ahat @ (Ahat @ X)) < 1e-12


def test_forward_matches_dense_hypothesis(oracle):
    hyp = pytest.importorskip("hypothesis")
    st = hyp.strategies

    @hyp.settings(max_examples=60, deadline=None)
    @hyp.given(nu=st.integers(1, 7), ni=st.integers(1, 6), data=st.data())
    def run(nu, ni, data):
        ne = data.draw(st.integers(0, 25))
        u = np.array(data.draw(st.lists(st.integers(0, nu - 1), min_size=ne, max_size=ne)), dtype=np.int32)
        i = np.array(data.draw(st.lists(st.integers(0, ni - 1), min_size=ne, max_size=ne)), dtype=np.int32)
        Ahat, _ = dense_ahat(nu, ni, u, i)
        X = np.arange((nu + ni) * 3, dtype=np.float64).reshape(nu + ni, 3) - 4.0
        row_ptr, col = oracle.build_csr(nu, ni, u, i)
        out = oracle.propagate_fwd(row_ptr, col, X, 2)[-1]
        assert relerr(out, Ahat @ Ahat @ X) < 1e-12

    run()


def test_planted_mistakes_are_caught(oracle):
    """The dense pin has teeth: operators that differ from A^ by one plausible slip
    (D for D~, no self-loop, row normalisation, one-sided scaling) do not match."""
    nu, ni, u, i = small_graph(21)
    n = nu + ni
    Ahat, At = dense_ahat(nu, ni, u, i)
    A = At - np.eye(n)
    d = A.sum(1)
    dt = d + 1
    wrong = [
        np.diag(dt ** -0.5) @ A @ np.diag(dt ** -0.5),                 # forgot + I in A~
        np.diag(np.maximum(d, 1) ** -0.5) @ At @ np.diag(np.maximum(d, 1) ** -0.5),  # D, not D~
        np.diag(1.0 / dt) @ At,                                        # row normalisation
        np.diag(dt ** -0.5) @ At,                                      # one-sided
    ]
    X = np.random.default_rng(0).standard_normal((n, 4))
    row_ptr, col = oracle.build_csr(nu, ni, u, i)
    out = oracle.propagate_layer(row_ptr, col, X)
    assert relerr(out, Ahat @ X) < 1e-12
    for M in wrong:
        assert relerr(out, M @ X) > 1e-3


# ---------------------------------------------------------------- closed forms
def _ahat_from_oracle(oracle, nu, ni, u, i, self_loops=True):
    """A^ column by column: propagate the identity."""
    row_ptr, col = oracle.build_csr(nu, ni, np.asarray(u, np.int32), np.asarray(i, np.int32),
                                    add_self_loops=self_loops)
    return oracle.propagate_layer(row_ptr, col, np.eye(nu + ni))


def _golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                vals[k.strip()] = float(v)
    return vals


def test_closed_form_no_edges(oracle):
    M = _ahat_from_oracle(oracle, 3, 2, [], [])
    assert np.array_equal(M, np.eye(5))          # A^ = I: every layer returns its input


def test_closed_form_single_edge(oracle):
    M = _ahat_from_oracle(oracle, 1, 1, [0], [0])
    assert np.allclose(M, 0.5, rtol=0, atol=1e-16)   # pair average, idempotent
    assert np.allclose(M @ M, M)


def test_closed_form_star_golden(oracle):
    g = _golden("star_m5.txt")
    m = 5
    M = _ahat_from_oracle(oracle, m, 1, list(range(m)), [0] * m)
    item = m
    assert abs(M[item, item] - g["item_item"]) < 1e-12
    for u in range(m):
        assert abs(M[item, u] - g["item_user"]) < 1e-12
        assert abs(M[u, item] - g["item_user"]) < 1e-12
        assert abs(M[u, u] - g["user_user"]) < 1e-12
    ev = np.linalg.eigvalsh(M)
    assert abs(ev.min() - g["lambda_min"]) < 1e-12 and abs(ev.max() - g["lambda_max"]) < 1e-12


@pytest.mark.parametrize("m", [1, 2, 7, 30])
def test_closed_form_star(oracle, m):
    M = _ahat_from_oracle(oracle, m, 1, list(range(m)), [0] * m)
    assert np.isclose(M[m, m], 1.0 / (m + 1), rtol=1e-14)
    assert np.allclose(M[m, :m], 1.0 / np.sqrt(2.0 * (m + 1)), rtol=1e-14)
    assert np.allclose(np.diag(M)[:m], 0.5, rtol=1e-14)
    off = M[:m, :m] - np.diag(np.diag(M)[:m])
    assert np.array_equal(off, np.zeros_like(off))


@pytest.mark.parametrize("a,b", [(2, 3), (4, 4), (1, 6)])
def test_closed_form_complete_bipartite(oracle, a, b):
    u, i = np.meshgrid(np.arange(a), np.arange(b), indexing="ij")
    M = _ahat_from_oracle(oracle, a, b, u.ravel(), i.ravel())
    assert np.allclose(np.diag(M)[:a], 1.0 / (b + 1), rtol=1e-14)
    assert np.allclose(np.diag(M)[a:], 1.0 / (a + 1), rtol=1e-14)
    assert np.allclose(M[:a, a:], 1.0 / np.sqrt((a + 1.0) * (b + 1.0)), rtol=1e-14)
    assert np.array_equal(M[:a, :a] - np.diag(np.diag(M)[:a]), np.zeros((a, a)))


@pytest.mark.parametrize("d", [1, 2, 3])
def test_closed_form_regular(oracle, d):
    """d-regular bipartite (circulant): A^ = (A + I) / (d + 1)."""
    m = 6
    u = np.repeat(np.arange(m), d)
    i = (u + np.tile(np.arange(d), m)) % m
    M = _ahat_from_oracle(oracle, m, m, u, i)
    _, At = dense_ahat(m, m, u, i)
    assert np.allclose(M, At / (d + 1.0), rtol=1e-14, atol=0)


# ---------------------------------------------------------------- invariants
@pytest.mark.parametrize("seed", [31, 32])
def test_invariants_small(oracle, seed):
    nu, ni, u, i = small_graph(seed, nu=40, ni=25, ne=300)
    M = _ahat_from_oracle(oracle, nu, ni, u, i)
    row_ptr, col = oracle.build_csr(nu, ni, u, i)
    deg, dinv = oracle.normalize(row_ptr)
    assert np.allclose(M, M.T, rtol=1e-15, atol=0)               # symmetric
    nz = M[M != 0]
    assert (nz > 0).all() and (nz <= 1).all()
    assert np.allclose(np.diag(M), 1.0 / deg, rtol=1e-14)        # A^_ii = 1 / d~_i
    ev = np.linalg.eigvalsh(M)
    assert ev.max() <= 1 + 1e-12 and ev.min() > -1               # spectrum in (-1, 1]
    assert abs(ev.max() - 1.0) < 1e-12
    v = np.sqrt(deg.astype(np.float64))[:, None]                 # D~^1/2 1
    for out in oracle.propagate_fwd(row_ptr, col, v, 5):
        assert np.allclose(out, v, rtol=1e-13)


def test_invariants_config2(oracle):
    """Fixed point and contraction on the 2 M-edge power-law graph (O(nnz) checks)."""
    c = make_config(2, features=False)
    row_ptr, col = oracle.build_csr(c["n_users"], c["n_items"], c["users"], c["items"])
    assert col.size == 2 * c["n_edges"] + c["n"]
    deg, _ = oracle.normalize(row_ptr)
    v = np.sqrt(deg.astype(np.float64))
    x = np.random.default_rng(3).standard_normal(c["n"])
    X = np.stack([v, x], axis=1)
    out = oracle.propagate_fwd(row_ptr, col, X, 3)
    for k in range(3):
        assert np.allclose(out[k][:, 0], v, rtol=1e-12)
    norms = [np.linalg.norm(x)] + [np.linalg.norm(o[:, 1]) for o in out]
    assert all(b <= a * (1 + 1e-12) for a, b in zip(norms, norms[1:]))   # ||A^ x|| <= ||x||


def test_scipy_cross_check_config2(oracle):
    sp = pytest.importorskip("scipy.sparse")
    c = make_config(2)
    nu, ni, n = c["n_users"], c["n_items"], c["n"]
    u = c["users"].astype(np.int64)
    i = c["items"].astype(np.int64) + nu
    A = sp.coo_matrix((np.ones(2 * u.size), (np.concatenate([u, i]), np.concatenate([i, u]))), shape=(n, n)).tocsr()
    A.data[:] = 1.0
    At = A + sp.identity(n, format="csr")
    s = 1.0 / np.sqrt(np.asarray(At.sum(1)).ravel())
    Ahat = sp.diags(s) @ At @ sp.diags(s)
    X = c["X0"][:, :8].astype(np.float64)
    row_ptr, col = oracle.build_csr(nu, ni, c["users"], c["items"])
    got = oracle.propagate_fwd(row_ptr, col, X, 3)[-1]
    ref = Ahat @ (Ahat @ (Ahat @ X))
    scale = abs(Ahat) @ (abs(Ahat) @ (abs(Ahat) @ np.abs(X)))
    assert (np.abs(got - ref) / (scale + 1e-300)).max() < 1e-12
    G = c["gY"][:, :8].astype(np.float64)
    gb = oracle.propagate_bwd(row_ptr, col, G, 2)
    refb = Ahat.T @ (Ahat.T @ G)
    assert relerr(gb, refb) < 1e-12


# ---------------------------------------------------------------- backward
@pytest.mark.parametrize("seed", [41, 42])
@pytest.mark.parametrize("K", [1, 3])
def test_backward_is_dense_transpose(oracle, seed, K):
    nu, ni, u, i = small_graph(seed)
    Ahat, _ = dense_ahat(nu, ni, u, i)
    rng = np.random.default_rng(seed)
    G = rng.standard_normal((nu + ni, 6))
    direct = [rng.standard_normal((nu + ni, 6)) for _ in range(K - 1)]
    row_ptr, col = oracle.build_csr(nu, ni, u, i)
    got = oracle.propagate_bwd(row_ptr, col, G, K, g_layers=direct if K > 1 else None)
    ref = G
    for l in range(K - 1, -1, -1):
        ref = Ahat.T @ ref
        if l >= 1:
            ref = ref + direct[l - 1]
    assert relerr(got, ref) < 1e-12


def test_backward_transposes_a_nonsymmetric_structure(oracle):
    """The scatter form is A^T on any CSR, not only on symmetric ones (every referenced
    column has a non-empty row, so all weights 1/sqrt(len_i len_j) are finite)."""
    n = 4
    rng = np.random.default_rng(7)
    X = rng.standard_normal((n, 3))
    G = rng.standard_normal((n, 3))
    row_ptr = np.array([0, 2, 3, 4, 7], dtype=np.int64)
    col = np.array([1, 3, 0, 3, 0, 1, 2], dtype=np.int32)
    length = np.diff(row_ptr).astype(np.float64)
    M = np.zeros((n, n))
    for r in range(n):
        for p in range(row_ptr[r], row_ptr[r + 1]):
            M[r, col[p]] = 1.0 / np.sqrt(length[r] * length[col[p]])
    assert not np.allclose(M, M.T)
    assert relerr(oracle.propagate_layer(row_ptr, col, X), M @ X) < 1e-13
    assert relerr(oracle.propagate_layer_transposed(row_ptr, col, G), M.T @ G) < 1e-13


@pytest.mark.parametrize("K", [1, 2, 3])
def test_adjoint_identity(oracle, K):
    c = make_config(1)
    row_ptr, col = oracle.build_csr(c["n_users"], c["n_items"], c["users"], c["items"])
    X = c["X0"].astype(np.float64)
    G = c["gY"].astype(np.float64)
    lhs = (oracle.propagate_fwd(row_ptr, col, X, K)[-1] * G).sum()
    rhs = (X * oracle.propagate_bwd(row_ptr, col, G, K)).sum()
    assert abs(lhs - rhs) <= 1e-12 * max(abs(lhs), 1e-300) + 1e-15 * np.abs(X).sum()


def test_backward_finite_differences(oracle):
    """d/dX of L = 1/2 ||A^^K X||^2 is (A^T)^K (A^^K X)."""
    nu, ni, u, i = small_graph(51, nu=6, ni=5, ne=14)
    row_ptr, col = oracle.build_csr(nu, ni, u, i)
    rng = np.random.default_rng(51)
    X = rng.standard_normal((nu + ni, 2))
    K = 2

    def loss(Xv):
        return 0.5 * (oracle.propagate_fwd(row_ptr, col, Xv, K)[-1] ** 2).sum()

    Y = oracle.propagate_fwd(row_ptr, col, X, K)[-1]
    grad = oracle.propagate_bwd(row_ptr, col, Y, K)
    h = 1e-6
    for idx in [(0, 0), (3, 1), (7, 0), (10, 1)]:
        Xp, Xm = X.copy(), X.copy()
        Xp[idx] += h
        Xm[idx] -= h
        fd = (loss(Xp) - loss(Xm)) / (2 * h)
        assert abs(fd - grad[idx]) < 1e-7 * max(1.0, abs(grad[idx]))


# ---------------------------------------------------------------- per-node LightGCN update
def test_no_self_loop_variant_matches_per_node_sums(oracle):
    """Section 3.1, per-node form: h_u = sum_{i in N(u)} h_i / (sqrt|N(u)| sqrt|N(i)|), and
    the same with the roles swapped; nodes without neighbours get zero."""
    nu, ni, u, i = small_graph(61, nu=9, ni=7, ne=20, dup=False)
    rng = np.random.default_rng(61)
    H = rng.standard_normal((nu + ni, 3))
    Nu = {a: sorted(set(int(x) for x in i[u == a])) for a in range(nu)}
    Ni = {b: sorted(set(int(x) for x in u[i == b])) for b in range(ni)}
    ref = np.zeros_like(H)
    for a in range(nu):
        for b in Nu[a]:
            ref[a] += H[nu + b] / (np.sqrt(len(Nu[a])) * np.sqrt(len(Ni[b])))
    for b in range(ni):
        for a in Ni[b]:
            ref[nu + b] += H[a] / (np.sqrt(len(Ni[b])) * np.sqrt(len(Nu[a])))
    row_ptr, col = oracle.build_csr(nu, ni, u, i, add_self_loops=False)
    assert relerr(oracle.propagate_layer(row_ptr, col, H), ref) < 1e-13
    Ad, _ = dense_ahat(nu, ni, u, i, self_loops=False)
    assert relerr(oracle.propagate_layer(row_ptr, col, H), Ad @ H) < 1e-13


# ---------------------------------------------------------------- plumbing
def test_rows_mode_equals_full(oracle):
    c = make_config(1)
    row_ptr, col = oracle.build_csr(c["n_users"], c["n_items"], c["users"], c["items"])
    X = c["X0"].astype(np.float64)
    full = oracle.propagate_layer(row_ptr, col, X)
    rows = np.array([0, 5, 1999, 2000, 2999, 17])
    assert np.array_equal(oracle.propagate_rows(row_ptr, col, X, rows), full[rows])


def test_thread_count_does_not_change_bits(oracle):
    c = make_config(1)
    row_ptr, col = oracle.build_csr(c["n_users"], c["n_items"], c["users"], c["items"])
    X = c["X0"].astype(np.float64)
    nt = oracle.max_threads()
    oracle.set_threads(1)
    a = oracle.propagate_layer(row_ptr, col, X)
    b = oracle.propagate_layer_transposed(row_ptr, col, X)
    oracle.set_threads(nt)
    assert np.array_equal(a, oracle.propagate_layer(row_ptr, col, X))
    assert np.array_equal(b, oracle.propagate_layer_transposed(row_ptr, col, X))


def test_bf16_bits_are_read_exactly(oracle):
    torch = pytest.importorskip("torch")
    bits = np.arange(0, 65536, 7, dtype=np.uint16)
    bits = bits[((bits >> 7) & 0xFF) != 0xFF]          # finite values only
    ref = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).double().numpy()
    assert np.array_equal(oracle.bf16_bits_to_f64(bits), ref)


# ---------------------------------------------------------------- dense update
@pytest.mark.parametrize("relu", [True, False])
def test_transform_matches_numpy(oracle, relu):
    rng = np.random.default_rng(71)
    P = rng.standard_normal((37, 12))
    W = rng.standard_normal((12, 9))
    gH = rng.standard_normal((37, 9))
    Z, H = oracle.transform_fwd(P, W, relu)
    assert relerr(Z, P @ W) < 1e-13
    assert np.array_equal(H, np.maximum(Z, 0) if relu else Z)
    dP, dW = oracle.transform_bwd(P, W, Z, gH, relu)
    dZ = gH * (P @ W > 0) if relu else gH
    assert relerr(dP, dZ @ W.T) < 1e-13
    assert relerr(dW, P.T @ dZ) < 1e-13
    dP2, dW2 = oracle.transform_bwd(P, W, H, gH, relu)      # mask from H is the same mask
    assert np.array_equal(dP, dP2) and np.array_equal(dW, dW2)


def test_transform_finite_differences(oracle):
    rng = np.random.default_rng(72)
    P = rng.standard_normal((8, 5))
    W = rng.standard_normal((5, 4))
    T = rng.standard_normal((8, 4))

    def loss(Pv, Wv):
        return (oracle.transform_fwd(Pv, Wv, True)[1] * T).sum()

    Z, _ = oracle.transform_fwd(P, W, True)
    dP, dW = oracle.transform_bwd(P, W, Z, T, True)
    h = 1e-6
    for idx in [(0, 0), (3, 2), (7, 4)]:
        Pp, Pm = P.copy(), P.copy()
        Pp[idx] += h
        Pm[idx] -= h
        assert abs((loss(Pp, W) - loss(Pm, W)) / (2 * h) - dP[idx]) < 1e-6
    for idx in [(0, 0), (2, 3), (4, 1)]:
        Wp, Wm = W.copy(), W.copy()
        Wp[idx] += h
        Wm[idx] -= h
        assert abs((loss(P, Wp) - loss(P, Wm)) / (2 * h) - dW[idx]) < 1e-6


# ---------------------------------------------------------------- readout + GFAE loss
def test_readout_and_gfae_single_edge_golden(oracle):
    g = _golden("gfae_single_edge.txt")
    row_ptr, col = oracle.build_csr(1, 1, np.array([0], np.int32), np.array([0], np.int32))
    X = np.array([[3.0, -1.0], [1.0, 5.0]])
    loss, Y, gX = oracle.gfae_step(row_ptr, col, X, 2)
    assert np.allclose(Y, [[g["y_u0"], g["y_u1"]], [g["y_i0"], g["y_i1"]]], rtol=1e-14)
    assert abs(loss - g["loss"]) < 1e-13
    _, gY = oracle.gfae_loss(X, Y)
    assert np.allclose(gY[0], [g["gy_u0"], g["gy_u1"]], rtol=1e-14)
    assert np.allclose(gX, [[g["gx_u0"], g["gx_u1"]], [g["gx_i0"], g["gx_i1"]]], rtol=1e-13)


def test_readout_no_edges_reproduces_input(oracle):
    row_ptr, col = oracle.build_csr(4, 3, np.zeros(0, np.int32), np.zeros(0, np.int32))
    X = np.random.default_rng(3).standard_normal((7, 5))
    loss, Y, gX = oracle.gfae_step(row_ptr, col, X, 3)
    assert np.array_equal(Y, X) and loss == 0.0 and not gX.any()


@pytest.mark.parametrize("seed,K", [(1, 1), (2, 2), (3, 4)])
def test_readout_and_loss_match_dense(oracle, seed, K):
    nu, ni, u, i = small_graph(seed)
    n = nu + ni
    Ahat, _ = dense_ahat(nu, ni, u, i)
    X = np.random.default_rng(seed).standard_normal((n, 6))
    M = sum(np.linalg.matrix_power(Ahat, l) for l in range(K + 1)) / (K + 1)
    row_ptr, col = oracle.build_csr(nu, ni, u, i)
    loss, Y, gX = oracle.gfae_step(row_ptr, col, X, K)
    assert relerr(Y, M @ X) < 1e-12
    assert abs(loss - np.linalg.norm(X - M @ X, "fro") ** 2) <= 1e-12 * loss
    R = np.eye(n) - M
    assert relerr(gX, 2.0 * R.T @ (R @ X)) < 1e-11
    # plausible slips are not within reach of these pins: mean over K instead of K+1, layer 0
    # left out of the mean, the sign of the gradient, the direct dependence on X forgotten
    layers = oracle.propagate_fwd(row_ptr, col, X, K)
    assert relerr(sum(layers) / K, M @ X) > 1e-3
    assert relerr((X + sum(layers)) / K, M @ X) > 1e-3
    g = 2.0 * (Y - X) / (K + 1)
    G0 = oracle.propagate_bwd(row_ptr, col, g, K, g_shared=g)
    assert relerr(G0, 2.0 * R.T @ (R @ X)) > 1e-3            # without the - gY term
    assert relerr(-gX, 2.0 * R.T @ (R @ X)) > 1e-3


def test_gfae_gradient_finite_differences(oracle):
    nu, ni, u, i = small_graph(8, nu=6, ni=4, ne=14)
    row_ptr, col = oracle.build_csr(nu, ni, u, i)
    K = 3
    rng = np.random.default_rng(0)
    X = rng.standard_normal((nu + ni, 3))
    _, _, gX = oracle.gfae_step(row_ptr, col, X, K)
    h = 1e-6
    for _ in range(12):
        r, c = rng.integers(0, nu + ni), rng.integers(0, 3)
        Xp, Xm = X.copy(), X.copy()
        Xp[r, c] += h
        Xm[r, c] -= h
        fd = (oracle.gfae_step(row_ptr, col, Xp, K)[0] - oracle.gfae_step(row_ptr, col, Xm, K)[0]) / (2 * h)
        assert abs(fd - gX[r, c]) <= 1e-6 * max(1.0, abs(gX[r, c]))


def test_shared_direct_terms_equal_explicit_ones(oracle):
    """propagate_bwd with one shared direct term equals the general form fed K-1 copies, plus
    the term of layer 0."""
    nu, ni, u, i = small_graph(4)
    row_ptr, col = oracle.build_csr(nu, ni, u, i)
    rng = np.random.default_rng(1)
    g = rng.standard_normal((nu + ni, 4))
    gK = rng.standard_normal((nu + ni, 4))
    K = 3
    a = oracle.propagate_bwd(row_ptr, col, gK, K, g_shared=g)
    b = oracle.propagate_bwd(row_ptr, col, gK, K, g_layers=[g] * (K - 1)) + g
    assert relerr(a, b) < 1e-14


# ---------------------------------------------------------------- GraphSAGE layer
def test_mean_aggregator_matches_dense(oracle):
    nu, ni, u, i = small_graph(6)
    n = nu + ni
    _, At = dense_ahat(nu, ni, u, i)
    A = At - np.eye(n)                                   # neighbour sets, no self-loop
    d = A.sum(1)
    Dinv = np.diag(np.where(d > 0, 1.0 / np.where(d > 0, d, 1.0), 0.0))
    row_ptr, col = oracle.build_csr(nu, ni, u, i, add_self_loops=False)
    X = np.random.default_rng(6).standard_normal((n, 5))
    assert relerr(oracle.mean_neighbours(row_ptr, col, X), Dinv @ A @ X) < 1e-13
    G = np.random.default_rng(7).standard_normal((n, 5))
    assert relerr(oracle.mean_neighbours_transposed(row_ptr, col, G), (Dinv @ A).T @ G) < 1e-13
    # one-slip variants are out of reach: sum instead of mean, symmetric normalisation, self included
    assert relerr(oracle.mean_neighbours(row_ptr, col, X), A @ X) > 1e-3
    s = np.where(d > 0, np.where(d > 0, d, 1.0) ** -0.5, 0.0)
    assert relerr(oracle.mean_neighbours(row_ptr, col, X), np.diag(s) @ A @ np.diag(s) @ X) > 1e-3
    assert relerr(oracle.mean_neighbours(row_ptr, col, X), np.diag(1.0 / (d + 1)) @ At @ X) > 1e-3


def test_mean_aggregator_star_and_isolated(oracle):
    # one item joined to 4 users, plus an item nobody touched
    row_ptr, col = oracle.build_csr(4, 2, np.arange(4, dtype=np.int32), np.zeros(4, np.int32), add_self_loops=False)
    X = np.arange(12, dtype=np.float64).reshape(6, 2)
    M = oracle.mean_neighbours(row_ptr, col, X)
    assert np.array_equal(M[4], X[:4].mean(0))           # the centre: average of its four users
    assert np.array_equal(M[:4], np.tile(X[4], (4, 1)))  # each user: its only neighbour
    assert not M[5].any()                                # empty neighbourhood: zero


def test_sage_layer_matches_numpy_and_finite_differences(oracle):
    nu, ni, u, i = small_graph(9, nu=7, ni=5, ne=18)
    n, F, Fo = nu + ni, 3, 4
    row_ptr, col = oracle.build_csr(nu, ni, u, i, add_self_loops=False)
    rng = np.random.default_rng(2)
    H = rng.standard_normal((n, F))
    W = rng.standard_normal((2 * F, Fo))
    _, At = dense_ahat(nu, ni, u, i)
    A = At - np.eye(n)
    d = A.sum(1)
    Mdense = np.diag(np.where(d > 0, 1.0 / np.where(d > 0, d, 1.0), 0.0)) @ A
    C, Z, Hn = oracle.sage_layer_fwd(row_ptr, col, H, W)
    assert relerr(Z, np.concatenate([H, Mdense @ H], axis=1) @ W) < 1e-13
    assert np.array_equal(Hn, np.maximum(Z, 0))
    R = rng.standard_normal((n, Fo))                     # L = <relu(Z), R>
    gH, dW = oracle.sage_layer_bwd(row_ptr, col, C, W, Z, R)

    def loss(Hv, Wv):
        return float((oracle.sage_layer_fwd(row_ptr, col, Hv, Wv)[2] * R).sum())

    h = 1e-6
    for _ in range(10):
        r, c = rng.integers(0, n), rng.integers(0, F)
        Hp, Hm = H.copy(), H.copy()
        Hp[r, c] += h
        Hm[r, c] -= h
        assert abs((loss(Hp, W) - loss(Hm, W)) / (2 * h) - gH[r, c]) < 1e-6
        r, c = rng.integers(0, 2 * F), rng.integers(0, Fo)
        Wp, Wm = W.copy(), W.copy()
        Wp[r, c] += h
        Wm[r, c] -= h
        assert abs((loss(H, Wp) - loss(H, Wm)) / (2 * h) - dW[r, c]) < 1e-6


# ---------------------------------------------------------------- GradNorm
def test_gradnorm_step_golden(oracle):
    g = _golden("gradnorm_two_tasks.txt")
    meta, w = oracle.gradnorm_step([2.0, 3.0], [4.0, 4.0], [3.0, 1.0], [1.0, 1.0], gamma=1.0, lr=0.1)
    assert abs(meta - g["meta"]) < 1e-14
    assert np.allclose(w, [g["w1"], g["w2"]], rtol=1e-15)


def test_gradnorm_invariants(oracle):
    rng = np.random.default_rng(0)
    for T in (2, 3, 5):
        loss, loss0, gn = rng.uniform(0.5, 2, T), rng.uniform(0.5, 2, T), rng.uniform(0.1, 3, T)
        w0 = rng.uniform(0.5, 1.5, T)
        w0 *= T / w0.sum()
        meta, w = oracle.gradnorm_step(loss, loss0, gn, w0, gamma=1.5, lr=0.01)
        assert abs(w.sum() - T) < 1e-12 and (w > 0).all()
        # the meta-loss the function reports is the formula of Section 4.3.1 written with numpy
        G = w0 * gn
        r = (loss / loss0) / (loss / loss0).mean()
        assert abs(meta - np.abs(G - G.mean() * r ** 1.5).sum()) < 1e-12
        # the step goes against the derivative of the meta-loss with the targets held constant
        target = G.mean() * r ** 1.5
        h = 1e-7
        for i in range(T):
            wp, wm = w0.copy(), w0.copy()
            wp[i] += h
            wm[i] -= h
            fd = (np.abs(wp * gn - target).sum() - np.abs(wm * gn - target).sum()) / (2 * h)
            assert abs(fd - np.sign(G[i] - target[i]) * gn[i]) < 1e-6
        raw = w0 - 0.01 * np.sign(G - target) * gn
        assert np.allclose(w, raw * T / raw.sum(), rtol=1e-12)
    # balanced gradients and equal progress: nothing to correct, the weights stay
    meta, w = oracle.gradnorm_step([1.0, 1.0], [2.0, 2.0], [2.0, 2.0], [1.0, 1.0])
    assert meta == 0.0 and np.array_equal(w, [1.0, 1.0])


def test_block_norms_match_numpy(oracle):
    G = np.random.default_rng(5).standard_normal((37, 12))
    got = oracle.block_norms(G, 3)
    assert np.allclose(got, [np.linalg.norm(G[:, 4 * t:4 * t + 4]) for t in range(3)], rtol=1e-14)


# ---------------------------------------------------------------- weighted graphs
def dense_weighted_ahat(nu, ni, u, i, w):
    """A^ from Section 3 "Notation" with real weights: A_ij = weight, A~ = A + I, D~ = D + I."""
    n = nu + ni
    A = np.zeros((n, n))
    for a, b, x in zip(u, i, w):
        A[a, nu + b] = max(A[a, nu + b], x)          # a repeated pair keeps its largest weight
        A[nu + b, a] = A[a, nu + b]
    At = A + np.eye(n)
    d = A.sum(1) + 1.0
    return np.diag(d ** -0.5) @ At @ np.diag(d ** -0.5), d


def test_weighted_operator_matches_dense(oracle):
    nu, ni, u, i = small_graph(12)
    w = np.random.default_rng(12).uniform(0.1, 3.0, size=u.size)
    Ahat, d = dense_weighted_ahat(nu, ni, u, i, w)
    row_ptr, col = oracle.build_csr(nu, ni, u, i)
    val = oracle.edge_values(nu, u, i, w, row_ptr, col)
    assert np.allclose(oracle.weighted_degrees(row_ptr, val), d, rtol=1e-14)
    X = np.random.default_rng(1).standard_normal((nu + ni, 4))
    assert relerr(oracle.propagate_layer_weighted(row_ptr, col, val, X), Ahat @ X) < 1e-13
    assert relerr(oracle.propagate_layer_weighted(row_ptr, col, val, X, transposed=True), Ahat.T @ X) < 1e-13
    assert relerr(oracle.propagate_weighted(row_ptr, col, val, X, 3), np.linalg.matrix_power(Ahat, 3) @ X) < 1e-12
    # invariants of the weighted operator: symmetric, D~^1/2 1 a fixed point, spectrum in (-1, 1]
    assert np.allclose(Ahat, Ahat.T)
    r = np.sqrt(d)[:, None]
    assert relerr(oracle.propagate_layer_weighted(row_ptr, col, val, r), r) < 1e-13
    ev = np.linalg.eigvalsh(Ahat)
    assert ev.max() <= 1 + 1e-12 and ev.min() > -1
    # slips: weights ignored, degrees counted instead of summed, self-loop weighted like an edge
    Au, _ = dense_ahat(nu, ni, u, i)
    assert relerr(oracle.propagate_layer_weighted(row_ptr, col, val, X), Au @ X) > 1e-3


def test_weighted_single_edge_closed_form_and_unit_weights(oracle):
    # one edge of weight w: d~ = 1 + w on both ends, A^ = [[1, w], [w, 1]] / (1 + w)
    row_ptr, col = oracle.build_csr(1, 1, np.array([0], np.int32), np.array([0], np.int32))
    val = oracle.edge_values(1, [0], [0], [3.0], row_ptr, col)
    M = oracle.propagate_layer_weighted(row_ptr, col, val, np.eye(2))
    assert np.allclose(M, np.array([[1.0, 3.0], [3.0, 1.0]]) / 4.0, rtol=1e-15)
    # all weights 1: the unweighted operator
    nu, ni, u, i = small_graph(5)
    row_ptr, col = oracle.build_csr(nu, ni, u, i)
    val = oracle.edge_values(nu, u, i, np.ones(u.size), row_ptr, col)
    X = np.random.default_rng(2).standard_normal((nu + ni, 3))
    assert relerr(oracle.propagate_layer_weighted(row_ptr, col, val, X), oracle.propagate_layer(row_ptr, col, X)) < 1e-14


# ---------------------------------------------------------------- importance sampling (Section 4.1)
def test_philox_known_answers(oracle):
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        rows = [[int(w, 16) for w in line.split()] for line in f if line.strip() and not line.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        assert list(oracle.philox4x32_10(r[0:4], r[4:6])) == r[6:10]


def one_user_graph(oracle, weights):
    """User 0 joined to items 0..m-1 with the given weights; -> (row_ptr, col, val)."""
    m = len(weights)
    u, i = np.zeros(m, np.int32), np.arange(m, dtype=np.int32)
    row_ptr, col = oracle.build_csr(1, m, u, i)
    return row_ptr, col, oracle.edge_values(1, u, i, np.asarray(weights, np.float64), row_ptr, col)


def test_sampling_weights_are_powers(oracle):
    w = np.array([0.5, 2.0, 0.0, 3.0, -1.0, 7.25])
    assert np.array_equal(oracle.sampling_weights(w, 1.0), np.where(w > 0, w, 0.0))
    assert np.array_equal(oracle.sampling_weights(w, 0.0), (w > 0).astype(np.float64))    # beta = 0: uniform
    assert np.allclose(oracle.sampling_weights(w, 2.5), np.where(w > 0, np.abs(w) ** 2.5, 0.0), rtol=1e-15)


def test_sampling_table_is_the_distribution_in_integers(oracle):
    rng = np.random.default_rng(4)
    nu, ni, u, i = small_graph(21, nu=30, ni=20, ne=300)
    row_ptr, col = oracle.build_csr(nu, ni, u, i)
    p = rng.uniform(0.01, 5.0, size=col.size).astype(np.float32)
    bad = rng.choice(col.size, size=40, replace=False)
    p[bad[:10]], p[bad[10:20]], p[bad[20:30]], p[bad[30:]] = 0.0, -1.0, np.nan, np.inf
    q = oracle.sampling_table(row_ptr, col, p)
    for r in range(nu + ni):
        sl = slice(row_ptr[r], row_ptr[r + 1])
        ok = (col[sl] != r) & (p[sl] > 0) & np.isfinite(p[sl])
        assert np.array_equal(q[sl] > 0, ok)                 # the diagonal and unusable entries cannot be drawn
        if ok.any():
            assert q[sl].max() == 1 << 24                    # the largest weight of the row maps to 2^24
            pr = p[sl][ok].astype(np.float64)
            assert np.allclose(q[sl][ok] / q[sl][ok].sum(), pr / pr.sum(), rtol=2e-5)
    # a weight far below the row maximum keeps the smallest positive chance instead of none
    row_ptr, col, _ = one_user_graph(oracle, [1.0, 1.0])
    q = oracle.sampling_table(row_ptr, col, np.array([0.0, 1.0, 1e-12, 1.0, 1.0, 1.0, 1.0], np.float32))
    assert sorted(q[row_ptr[0]:row_ptr[1]].tolist()) == [0, 1, 1 << 24]


def test_sampler_pick_follows_from_the_random_bits(oracle):
    """Three neighbours with integer weights 2^24, 2^23, 2^23 (total 2^25): the pick of draw t is
    decided by r = floor(bits * total / 2^64), worked out here with Python integers from the
    generator's output for counter (t, node, hop, 0) and the seed's halves as key."""
    row_ptr, col, val = one_user_graph(oracle, [2.0, 1.0, 1.0])
    q = oracle.sampling_table(row_ptr, col, val.astype(np.float32))
    assert q[row_ptr[0]:row_ptr[1]].tolist() == [0, 1 << 24, 1 << 23, 1 << 23]
    seed = 0x1234567890ABCDEF
    hop_of, src, dst, entry = oracle.sample_picks(row_ptr, col, q, [0], [2], seed)
    assert src.tolist() == [0, 0] and hop_of[0] == 1
    for t in range(2):
        out = oracle.philox4x32_10([t, 0, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
        r = ((int(out[0]) | (int(out[1]) << 32)) * (1 << 25)) >> 64
        want = 1 if r < (1 << 24) else 2 if r < (1 << 24) + (1 << 23) else 3
        assert dst[t] == want and entry[t] == row_ptr[0] + want
    # second hop, from item node 2 (a row of two entries: user 0 and itself) with fan-out 1 < 2 entries
    hop_of, src, dst, entry = oracle.sample_picks(row_ptr, col, q, [2], [1, 2], seed)
    assert src.tolist()[0] == 2 and dst.tolist()[0] == 0 and hop_of[0] == 2   # its only neighbour, whatever the bits
    for t in range(2):                                                         # hop 1 from node 0: counter (t, 0, 1, 0)
        out = oracle.philox4x32_10([t, 0, 1, 0], [seed & 0xFFFFFFFF, seed >> 32])
        r = ((int(out[0]) | (int(out[1]) << 32)) * (1 << 25)) >> 64
        want = 1 if r < (1 << 24) else 2 if r < (1 << 24) + (1 << 23) else 3
        assert src[1 + t] == 0 and dst[1 + t] == want


@pytest.mark.parametrize("beta", [0.0, 1.0, 1.7])
def test_sampler_frequencies_follow_the_sampling_probability(oracle, beta):
    """Draws of one node over many seeds are independent samples of p(u->v) = w^beta / sum w^beta:
    a chi-square test of the counts against that distribution (39 degrees of freedom)."""
    rng = np.random.default_rng(8)
    w = rng.uniform(0.2, 4.0, size=40)
    row_ptr, col, val = one_user_graph(oracle, w)
    q = oracle.sampling_table(row_ptr, col, oracle.sampling_weights(val, beta).astype(np.float32))
    counts = np.zeros(41)
    reps, k = 3000, 8
    for s in range(reps):
        _, src, dst, _ = oracle.sample_picks(row_ptr, col, q, [0], [k], 1000 + s)
        assert src.size == k
        counts += np.bincount(dst, minlength=41)
    assert counts[0] == 0                                   # never the node itself
    prob = w ** beta / (w ** beta).sum()
    chi2 = (((counts[1:] - reps * k * prob) ** 2) / (reps * k * prob)).sum()
    assert chi2 < 39 + 5 * np.sqrt(2 * 39), chi2
    # and a planted mistake (the neighbour after the drawn one) is far outside
    shifted = np.roll(counts[1:], 1)
    assert (((shifted - reps * k * prob) ** 2) / (reps * k * prob)).sum() > 10 * 39 or beta == 0.0


def test_sampler_large_beta_keeps_the_strongest_neighbour(oracle):
    w = np.array([1.0, 1.5, 0.7, 3.0, 2.9, 0.1, 1.1, 2.0]) / 3.0
    row_ptr, col, val = one_user_graph(oracle, w)
    q = oracle.sampling_table(row_ptr, col, oracle.sampling_weights(val, 2000.0).astype(np.float32))
    assert q[row_ptr[0]:row_ptr[1]].max() == 1 << 24 and np.sort(q[row_ptr[0]:row_ptr[1]])[-2] <= 1
    _, _, dst, _ = oracle.sample_picks(row_ptr, col, q, [0], [4], 5)
    assert dst.tolist() == [4, 4, 4, 4]                     # item 3 = node 4; (2.9/3)^2000 is below 2^-24


def test_sampler_keeps_all_of_exactly_k_neighbours(oracle):
    """Section 4.1 caps a node at k neighbours: a node that has exactly k keeps every one of them (no
    draws with replacement, which would lose some), whichever end of the row its own diagonal entry
    sits at; with k + 1 neighbours k draws are made."""
    for k in (1, 3, 7):
        w = np.linspace(0.5, 2.0, k)
        row_ptr, col, val = one_user_graph(oracle, w)                  # user 0: diagonal first, then k items
        q = oracle.sampling_table(row_ptr, col, val.astype(np.float32))
        _, src, dst, _ = oracle.sample_picks(row_ptr, col, q, [0], [k], 11)
        assert src.tolist() == [0] * k and dst.tolist() == list(range(1, k + 1))
        # an item with exactly k users: its diagonal entry is the LAST of its row
        u, i = np.arange(k, dtype=np.int32), np.zeros(k, np.int32)
        rp, cl = oracle.build_csr(k, 1, u, i)
        vv = oracle.edge_values(k, u, i, w, rp, cl)
        qq = oracle.sampling_table(rp, cl, vv.astype(np.float32))
        _, src, dst, _ = oracle.sample_picks(rp, cl, qq, [k], [k], 11)
        assert src.tolist() == [k] * k and dst.tolist() == list(range(k))
        # one more neighbour than k: k draws (with replacement, so possibly fewer distinct ones)
        row_ptr, col, val = one_user_graph(oracle, np.linspace(0.5, 2.0, k + 1))
        q = oracle.sampling_table(row_ptr, col, val.astype(np.float32))
        _, src, dst, _ = oracle.sample_picks(row_ptr, col, q, [0], [k], 11)
        assert dst.size == k and set(dst.tolist()) <= set(range(1, k + 2))
    # a weight that cannot be drawn stays out even when every neighbour is kept
    row_ptr, col, val = one_user_graph(oracle, [1.0, 0.0, 2.0])
    q = oracle.sampling_table(row_ptr, col, val.astype(np.float32))
    _, _, dst, _ = oracle.sample_picks(row_ptr, col, q, [0], [3], 11)
    assert dst.tolist() == [1, 3]


def test_sampler_structure(oracle):
    """Two hops on a power-law graph: what must hold for any random bits."""
    c = make_config(2, scale=0.02, features=False)
    nu, ni = c["n_users"], c["n_items"]
    n = nu + ni
    row_ptr, col = oracle.build_csr(nu, ni, c["users"], c["items"])
    rng = np.random.default_rng(3)
    w = rng.uniform(0.1, 3.0, size=c["users"].size)
    w[::9] = 0.0                                            # edges that are stored but cannot be drawn
    val = oracle.edge_values(nu, c["users"], c["items"], w, row_ptr, col)
    q = oracle.sampling_table(row_ptr, col, oracle.sampling_weights(val, 1.0).astype(np.float32))
    seeds = rng.choice(nu, size=50, replace=False).astype(np.int32)
    seeds = np.concatenate([seeds, seeds[:5]])              # a seed given twice is one seed
    fan = [6, 4]
    hop_of, src, dst, entry = oracle.sample_picks(row_ptr, col, q, seeds, fan, 77)
    row_of_entry = np.searchsorted(row_ptr, entry, side="right") - 1
    assert np.array_equal(row_of_entry, src) and np.array_equal(col[entry], dst)      # picks are stored entries
    assert (q[entry] > 0).all() and (src != dst).all()
    assert set(np.nonzero(hop_of == 1)[0]) == set(seeds.tolist())
    assert (hop_of[dst] >= 1).all() and (hop_of[dst] <= hop_of[src] + 1).all()
    deg = np.diff(row_ptr)
    for h, k in enumerate(fan):
        frontier = np.nonzero(hop_of == h + 1)[0]
        sel = hop_of[src] == h + 1
        per_node = np.bincount(src[sel], minlength=n)
        assert per_node[np.setdiff1d(np.arange(n), frontier)].sum() == 0              # only the frontier is expanded
        for u in frontier:
            mine = np.sort(entry[sel & (src == u)])
            usable = np.arange(row_ptr[u], row_ptr[u + 1])[q[row_ptr[u]:row_ptr[u + 1]] > 0]
            if deg[u] - 1 <= k:                                                       # the row also holds the node itself
                assert np.array_equal(mine, usable)                                    # at most k neighbours: all of them
            else:
                assert mine.size == (k if usable.size else 0)                          # else exactly k draws
        reached = np.nonzero(hop_of == h + 2)[0]                                       # first reached at this hop
        assert set(reached.tolist()) <= set(dst[sel].tolist())
    assert (hop_of[src] <= len(fan)).all()                                             # the last hop's nodes are leaves
    # local numbering
    s = oracle.sample_subgraph(nu, row_ptr, col, q, seeds, fan, 77)
    assert np.array_equal(s["nodes"], np.nonzero(hop_of)[0]) and s["n_users"] == (s["nodes"] < nu).sum()
    gu, gi = s["nodes"][s["users"]], s["nodes"][s["n_users"] + s["items"]]
    assert np.array_equal(np.minimum(src, dst), gu) and np.array_equal(np.maximum(src, dst), gi)
    # another seed gives other picks; the same seed the same
    again = oracle.sample_picks(row_ptr, col, q, seeds, fan, 77)
    other = oracle.sample_picks(row_ptr, col, q, seeds, fan, 78)
    assert np.array_equal(again[3], entry) and not np.array_equal(other[3][:entry.size], entry[:other[3].size])
