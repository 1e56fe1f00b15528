"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function
the header declares, the binding covers them all, and argument errors are caught before any
device work is enqueued."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "e2eg.h")


@pytest.fixture(scope="module")
def B():
    from paper_2511_20564_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2511_20564_amd import build
        build.build(verbose=False)
    binding.load_library()
    return binding


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(e2eg_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_five_entry_points():
    names = declared_functions()
    for required in ("e2eg_build_csr", "e2eg_normalize", "e2eg_propagate_fwd", "e2eg_propagate_bwd",
                     "e2eg_layer_transform"):
        assert required in names


def test_library_exports_every_declared_symbol(B):
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in e2eg.h but not exported"


def test_binding_mirrors_the_header(B):
    assert sorted(B.SIGNATURES) == declared_functions()
    for name in declared_functions():
        assert hasattr(B, name), f"binding has no wrapper named {name}"


def test_status_strings(B):
    assert B.e2eg_status_string(0) == "ok"
    for code in range(-8, 0):
        assert B.e2eg_status_string(code) not in ("ok", "unknown status")
    assert B.e2eg_status_string(-99) == "unknown status"
    assert B.e2eg_version() >= 100


def test_workspace_queries_are_pure_host_functions(B):
    assert B.e2eg_build_csr_workspace_bytes(1000, 500, 20000) >= 2 * 8 * 20000
    assert B.e2eg_build_csr_workspace_bytes(-1, 5, 5) == 0
    assert B.e2eg_sched_bytes(3000, 43000) > 16 * 3000
    assert B.e2eg_normalize_workspace_bytes(3000, 43000) > 12 * 3000
    one = B.e2eg_propagate_workspace_bytes(3000, 43000, B.E2EG_F32, 64, 1)
    two = B.e2eg_propagate_workspace_bytes(3000, 43000, B.E2EG_F32, 64, 2)
    assert two >= one + 3000 * 64 * 4 > 0
    assert B.e2eg_propagate_workspace_bytes(3000, 43000, 7, 64, 2) == 0
    assert B.e2eg_layer_transform_workspace_bytes(B.E2EG_TRANSFORM_BWD, 1000, 128, 128, B.E2EG_BF16) >= 128 * 128 * 4
    for q in (B.e2eg_sched_bytes(10, 10), one, two):
        assert q % 256 == 0


def test_workspace_queries_at_the_largest_sizes_the_abi_accepts(B):
    """nnz up to INT32_MAX: the sizes are computed in 64 bits (a wrapped product would fall below these
    lower bounds, which count only the largest arrays each call needs)."""
    n, nnz = 60_000_000, 2 ** 31 - 1
    assert B.e2eg_sched_bytes(n, nnz) >= 12 * nnz                  # columns, node ids, scales per entry
    assert B.e2eg_sched_weighted_bytes(n, nnz) >= 16 * nnz         # and values
    assert B.e2eg_normalize_workspace_bytes(n, nnz) >= 16 * nnz    # two arrays of 8-byte sort keys
    assert B.e2eg_propagate_workspace_bytes(n, nnz, B.E2EG_BF16, 128, 3) >= 2 * (n + 1) * 128 * 2   # two Z buffers
    assert B.e2eg_propagate_workspace_bytes(n, nnz, B.E2EG_F32, 256, 3) >= 2 * (n + 1) * 256 * 4
    n_users, n_items = 40_000_000, 20_000_000
    E = (nnz - n) // 2                                             # 2 E + n stored entries
    assert B.e2eg_build_csr_workspace_bytes(n_users, n_items, E) >= 16 * E
    big = B.e2eg_layer_transform_workspace_bytes(B.E2EG_TRANSFORM_BWD, 2 ** 31 - 1, 256, 256, B.E2EG_BF16)
    assert 256 * 256 * 4 * 250 <= big <= 256 * 256 * 4 * 260       # about 256 partial matrices whatever n
    for k in (1, 2, 3):                                            # monotone in K
        assert B.e2eg_propagate_workspace_bytes(n, nnz, B.E2EG_BF16, 128, k) <= \
            B.e2eg_propagate_workspace_bytes(n, nnz, B.E2EG_BF16, 128, k + 1)


FAKE = 0x1000  # non-null, 256-byte aligned; never dereferenced because validation fails first


def status_of(B, fn, *args):
    with pytest.raises(B.E2egError) as e:
        fn(*args)
    assert B.e2eg_last_error() != ""
    return e.value.status


def test_build_csr_argument_errors(B):
    f = B.e2eg_build_csr
    assert status_of(B, f, -1, 5, 3, FAKE, FAKE, 1, FAKE, FAKE, 100, FAKE, 1 << 20) == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, f, 5, 5, 3, FAKE, FAKE, 2, FAKE, FAKE, 100, FAKE, 1 << 20) == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, f, 5, 5, 3, None, FAKE, 1, FAKE, FAKE, 100, FAKE, 1 << 20) == B.E2EG_ERR_NULL_PTR
    assert status_of(B, f, 5, 5, 3, FAKE, FAKE, 1, None, FAKE, 100, FAKE, 1 << 20) == B.E2EG_ERR_NULL_PTR
    assert status_of(B, f, 5, 5, 3, FAKE, FAKE, 1, FAKE, FAKE, 15, FAKE, 1 << 20) == B.E2EG_ERR_CAPACITY
    assert status_of(B, f, 5, 5, 3, FAKE, FAKE, 1, FAKE, FAKE, 16, None, 0) == B.E2EG_ERR_WORKSPACE
    assert status_of(B, f, 5, 5, 3, FAKE, FAKE, 1, FAKE, FAKE, 16, FAKE + 8, 1 << 20) == B.E2EG_ERR_WORKSPACE
    assert status_of(B, f, 5, 5, 3, FAKE, FAKE, 1, FAKE, FAKE, 16, FAKE, 64) == B.E2EG_ERR_WORKSPACE
    # nnz bound 2*E + n beyond int32
    big = 1_100_000_000
    assert status_of(B, f, 5, 5, big, FAKE, FAKE, 1, FAKE, FAKE, 3 * big, FAKE, 1 << 40) == B.E2EG_ERR_OVERFLOW
    assert status_of(B, f, 0, 5, 3, FAKE, FAKE, 1, FAKE, FAKE, 100, FAKE, 1 << 20) == B.E2EG_ERR_INVALID_ARG


def test_normalize_argument_errors(B):
    f = B.e2eg_normalize
    assert status_of(B, f, -1, 10, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 20, FAKE, 1 << 20) == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, f, 10, 1 << 31, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 40, FAKE, 1 << 40) == B.E2EG_ERR_OVERFLOW
    assert status_of(B, f, 10, 20, None, FAKE, FAKE, FAKE, FAKE, 1 << 20, FAKE, 1 << 20) == B.E2EG_ERR_NULL_PTR
    assert status_of(B, f, 10, 20, FAKE, None, FAKE, FAKE, FAKE, 1 << 20, FAKE, 1 << 20) == B.E2EG_ERR_NULL_PTR
    assert status_of(B, f, 10, 20, FAKE, FAKE, FAKE, FAKE, FAKE, 16, FAKE, 1 << 20) == B.E2EG_ERR_CAPACITY
    assert status_of(B, f, 10, 20, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 20, FAKE, 16) == B.E2EG_ERR_WORKSPACE


def test_propagate_argument_errors(B):
    f = B.e2eg_propagate_fwd
    ok = dict(n=10, nnz=20, rp=FAKE, ci=FAKE, di=FAKE, sc=FAKE, dt=B.E2EG_F32, F=64, K=2, x=FAKE, ldx=64, o=FAKE,
              ldo=64, ls=0, ws=FAKE, wsb=1 << 30)

    def call(**kw):
        a = dict(ok, **kw)
        return status_of(B, f, a["n"], a["nnz"], a["rp"], a["ci"], a["di"], a["sc"], a["dt"], a["F"], a["K"],
                         a["x"], a["ldx"], a["o"], a["ldo"], a["ls"], a["ws"], a["wsb"])

    assert call(n=-1) == B.E2EG_ERR_INVALID_ARG
    assert call(nnz=1 << 31) == B.E2EG_ERR_OVERFLOW
    assert call(dt=5) == B.E2EG_ERR_BAD_DTYPE
    assert call(F=66) == B.E2EG_ERR_INVALID_ARG            # fp32 rows are read 16 bytes at a time
    assert call(dt=B.E2EG_BF16, F=68) == B.E2EG_ERR_INVALID_ARG
    assert call(K=0) == B.E2EG_ERR_INVALID_ARG
    assert call(rp=None) == B.E2EG_ERR_NULL_PTR
    assert call(x=None) == B.E2EG_ERR_NULL_PTR
    assert call(x=FAKE + 4) == B.E2EG_ERR_INVALID_ARG       # misaligned
    assert call(ldx=60) == B.E2EG_ERR_INVALID_ARG           # ld < F
    assert call(ldo=66) == B.E2EG_ERR_INVALID_ARG
    assert call(ls=100) == B.E2EG_ERR_INVALID_ARG           # 0 < layer_stride < n*ldo
    assert call(ws=None) == B.E2EG_ERR_WORKSPACE
    assert call(wsb=128) == B.E2EG_ERR_WORKSPACE
    g = B.e2eg_propagate_bwd
    assert status_of(B, g, 10, 20, FAKE, FAKE, FAKE, FAKE, B.E2EG_F32, 64, 2, None, 64, None, 0, FAKE, 64, FAKE,
                     1 << 30) == B.E2EG_ERR_NULL_PTR
    assert status_of(B, g, 10, 20, FAKE, FAKE, FAKE, FAKE, B.E2EG_F32, 64, 3, FAKE, 64, FAKE, 8, FAKE, 64, FAKE,
                     1 << 30) == B.E2EG_ERR_INVALID_ARG      # direct-term stride too small


def test_layer_transform_argument_errors(B):
    f = B.e2eg_layer_transform
    assert status_of(B, f, 9, 10, 128, 128, B.E2EG_BF16, 1, FAKE, FAKE, FAKE, None, None, None, FAKE, 1 << 20) \
        == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, f, 0, 10, 128, 128, B.E2EG_F32, 1, FAKE, FAKE, FAKE, None, None, None, FAKE, 1 << 20) \
        == B.E2EG_ERR_BAD_DTYPE
    assert status_of(B, f, 0, 10, 100, 128, B.E2EG_BF16, 1, FAKE, FAKE, FAKE, None, None, None, FAKE, 1 << 20) \
        == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, f, 0, 10, 128, 512, B.E2EG_BF16, 1, FAKE, FAKE, FAKE, None, None, None, FAKE, 1 << 20) \
        == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, f, 0, 10, 128, 128, B.E2EG_BF16, 1, None, FAKE, FAKE, None, None, None, FAKE, 1 << 20) \
        == B.E2EG_ERR_NULL_PTR
    assert status_of(B, f, 1, 10, 128, 128, B.E2EG_BF16, 1, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, 1 << 20) \
        == B.E2EG_ERR_NULL_PTR                                # backward without d_gH
    assert status_of(B, f, 1, 10, 128, 128, B.E2EG_BF16, 1, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 16) \
        == B.E2EG_ERR_WORKSPACE


def test_aggregate_argument_errors(B):
    f = B.e2eg_aggregate
    ok = dict(mode=B.E2EG_AGG_MEAN, n=10, nnz=30, rp=FAKE, col=FAKE, sched=FAKE, dtype=B.E2EG_F32, F=8, X=FAKE, ldx=8,
              add=None, lda=0, Y=FAKE, ldy=8, ws=FAKE, wsb=1 << 30)

    def call(**kw):
        a = dict(ok, **kw)
        return status_of(B, f, a["mode"], a["n"], a["nnz"], a["rp"], a["col"], a["sched"], a["dtype"], a["F"], a["X"],
                         a["ldx"], a["add"], a["lda"], a["Y"], a["ldy"], a["ws"], a["wsb"])

    assert call(mode=9) == B.E2EG_ERR_INVALID_ARG
    assert call(dtype=5) == B.E2EG_ERR_BAD_DTYPE
    assert call(F=6) == B.E2EG_ERR_INVALID_ARG
    assert call(sched=None) == B.E2EG_ERR_NULL_PTR
    assert call(X=None) == B.E2EG_ERR_NULL_PTR
    assert call(ldy=4) == B.E2EG_ERR_INVALID_ARG
    assert call(add=FAKE, lda=4) == B.E2EG_ERR_INVALID_ARG
    assert call(wsb=16) == B.E2EG_ERR_WORKSPACE
    assert call(nnz=1 << 31) == B.E2EG_ERR_OVERFLOW
    assert B.e2eg_aggregate_workspace_bytes(10, 30, B.E2EG_F32, 8) > 0


def test_readout_and_gfae_argument_errors(B):
    r = B.e2eg_readout_mean
    assert status_of(B, r, 10, B.E2EG_F32, 6, 2, FAKE, 6, FAKE, 6, 60, FAKE, 6) == B.E2EG_ERR_INVALID_ARG   # F % 4
    assert status_of(B, r, 10, 7, 8, 2, FAKE, 8, FAKE, 8, 80, FAKE, 8) == B.E2EG_ERR_BAD_DTYPE
    assert status_of(B, r, 10, B.E2EG_F32, 8, 2, None, 8, FAKE, 8, 80, FAKE, 8) == B.E2EG_ERR_NULL_PTR
    assert status_of(B, r, 10, B.E2EG_F32, 8, 2, FAKE, 8, None, 8, 80, FAKE, 8) == B.E2EG_ERR_NULL_PTR
    assert status_of(B, r, 10, B.E2EG_F32, 8, 2, FAKE, 8, FAKE, 8, 40, FAKE, 8) == B.E2EG_ERR_INVALID_ARG  # stride < n*ld
    assert status_of(B, r, 10, B.E2EG_F32, 8, -1, FAKE, 8, FAKE, 8, 80, FAKE, 8) == B.E2EG_ERR_INVALID_ARG
    r(0, B.E2EG_F32, 8, 0, FAKE, 8, None, 8, 0, FAKE, 8)       # n = 0: nothing to do, nothing launched
    g = B.e2eg_gfae_loss
    assert B.e2eg_gfae_loss_workspace_bytes(10, 8) > 0
    assert status_of(B, g, 10, B.E2EG_BF16, 12, FAKE, 16, FAKE, 16, FAKE, None, 16, 1.0, FAKE, 1 << 20) \
        == B.E2EG_ERR_INVALID_ARG                             # F % 8
    assert status_of(B, g, 10, B.E2EG_BF16, 16, FAKE, 16, FAKE, 16, None, None, 16, 1.0, FAKE, 1 << 20) \
        == B.E2EG_ERR_NULL_PTR                                # no place for the loss
    assert status_of(B, g, 10, B.E2EG_BF16, 16, FAKE, 16, FAKE, 8, FAKE, None, 16, 1.0, FAKE, 1 << 20) \
        == B.E2EG_ERR_INVALID_ARG                             # ldy < F
    assert status_of(B, g, 10, B.E2EG_BF16, 16, FAKE, 16, FAKE, 16, FAKE, None, 16, 1.0, FAKE, 8) \
        == B.E2EG_ERR_WORKSPACE


def test_gradnorm_step_is_host_arithmetic(B, oracle):
    """e2eg_gradnorm_step needs no GPU: compared with the oracle here, on the CPU."""
    rng = np.random.default_rng(3)
    for T in (1, 2, 4):
        loss, loss0, gn = rng.uniform(0.5, 2, T), rng.uniform(0.5, 2, T), rng.uniform(0.1, 3, T)
        w0 = rng.uniform(0.5, 1.5, T)
        meta, w = B.e2eg_gradnorm_step(list(loss), list(loss0), list(gn), list(w0), gamma=1.0, lr=0.05)
        meta_r, w_r = oracle.gradnorm_step(loss, loss0, gn, w0, gamma=1.0, lr=0.05)
        assert abs(meta - meta_r) <= 1e-12 * max(1.0, meta_r)
        assert np.allclose(w, w_r, rtol=1e-12)
    assert status_of(B, B.e2eg_gradnorm_step, [1.0], [0.0], [1.0], [1.0]) == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, B.e2eg_block_norms, 10, B.E2EG_F32, 8, 9, FAKE, 72, FAKE, FAKE, 1 << 20) == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, B.e2eg_block_norms, 10, B.E2EG_F32, 8, 2, FAKE, 8, FAKE, FAKE, 1 << 20) == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, B.e2eg_block_norms, 10, B.E2EG_F32, 8, 2, FAKE, 16, None, FAKE, 1 << 20) == B.E2EG_ERR_NULL_PTR
    assert B.e2eg_block_norms_workspace_bytes(10, 8, 2) > 0 and B.e2eg_block_norms_workspace_bytes(10, 8, 9) == 0


def test_weighted_graph_argument_errors(B):
    w = B.e2eg_edge_weights
    assert status_of(B, w, 5, 5, -1, FAKE, FAKE, FAKE, 10, FAKE, FAKE, FAKE) == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, w, 5, 5, 3, FAKE, FAKE, None, 10, FAKE, FAKE, FAKE) == B.E2EG_ERR_NULL_PTR
    assert status_of(B, w, 5, 5, 3, FAKE, FAKE, FAKE, 10, FAKE, FAKE, None) == B.E2EG_ERR_NULL_PTR
    assert status_of(B, w, 5, 5, 3, FAKE, FAKE, FAKE, 1 << 31, FAKE, FAKE, FAKE) == B.E2EG_ERR_OVERFLOW
    assert status_of(B, w, 0, 0, 0, None, None, None, 4, FAKE, FAKE, FAKE) == B.E2EG_ERR_INVALID_ARG
    w(5, 5, 0, None, None, None, 0, FAKE, None, None)            # nothing stored: nothing to do
    # the weighted schedule is the unweighted one plus the values
    assert B.e2eg_sched_weighted_bytes(100, 1000) >= B.e2eg_sched_bytes(100, 1000) + 4 * 1000
    assert B.e2eg_sched_weighted_bytes(-1, 0) == 0
    nw = B.e2eg_normalize_weighted
    big = 1 << 30
    assert status_of(B, nw, 10, 30, FAKE, FAKE, None, None, None, FAKE, FAKE, big, FAKE, big) == B.E2EG_ERR_NULL_PTR
    assert status_of(B, nw, 10, 30, FAKE, FAKE, FAKE, None, None, None, FAKE, big, FAKE, big) == B.E2EG_ERR_NULL_PTR
    assert status_of(B, nw, 10, 30, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, B.e2eg_sched_bytes(10, 30), FAKE, big) == B.E2EG_ERR_CAPACITY
    assert status_of(B, nw, 10, 30, FAKE, FAKE, FAKE, None, None, FAKE, FAKE, big, FAKE, 16) == B.E2EG_ERR_WORKSPACE
    assert status_of(B, B.e2eg_sched_check_symmetric, None) == B.E2EG_ERR_NULL_PTR
    f = B.e2eg_propagate_weighted_fwd
    assert status_of(B, f, 10, 30, FAKE, FAKE, FAKE, FAKE, B.E2EG_F32, 6, 2, FAKE, 8, FAKE, 8, 0, FAKE, big) == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, f, 10, 30, FAKE, FAKE, FAKE, None, B.E2EG_F32, 8, 2, FAKE, 8, FAKE, 8, 0, FAKE, big) == B.E2EG_ERR_NULL_PTR
    assert status_of(B, f, 10, 30, FAKE, FAKE, FAKE, FAKE, B.E2EG_F32, 8, 2, FAKE, 8, FAKE, 8, 0, FAKE, 16) == B.E2EG_ERR_WORKSPACE
    f = B.e2eg_propagate_weighted_bwd
    assert status_of(B, f, 10, 30, FAKE, FAKE, FAKE, FAKE, B.E2EG_F32, 6, 2, FAKE, 8, None, 0, FAKE, 8, FAKE, big) == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, f, 10, 30, FAKE, FAKE, FAKE, FAKE, B.E2EG_F32, 8, 2, None, 8, None, 0, FAKE, 8, FAKE, big) == B.E2EG_ERR_NULL_PTR
    assert "propagate_weighted_bwd" in B.e2eg_last_error()


def test_sampler_argument_errors(B):
    big = 1 << 30
    assert status_of(B, B.e2eg_sampling_weights, 10, FAKE, -1.0, FAKE) == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, B.e2eg_sampling_weights, 10, FAKE, float("nan"), FAKE) == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, B.e2eg_sampling_weights, 10, None, 1.0, FAKE) == B.E2EG_ERR_NULL_PTR
    B.e2eg_sampling_weights(0, None, 1.0, None)
    assert B.e2eg_sampler_table_bytes(1000) >= 8 * 1001 and B.e2eg_sampler_table_bytes(-1) == 0
    pr = B.e2eg_sampler_prepare
    assert status_of(B, pr, 10, 30, FAKE, FAKE, None, FAKE, big, FAKE, big) == B.E2EG_ERR_NULL_PTR
    assert status_of(B, pr, 10, 30, FAKE, FAKE, FAKE, FAKE, 64, FAKE, big) == B.E2EG_ERR_CAPACITY
    assert status_of(B, pr, 10, 30, FAKE, FAKE, FAKE, FAKE, big, FAKE, 0) == B.E2EG_ERR_WORKSPACE
    assert status_of(B, pr, 10, 1 << 31, FAKE, FAKE, FAKE, FAKE, big, FAKE, big) == B.E2EG_ERR_OVERFLOW
    # the plan: seeds x fan-outs, a frontier never larger than the graph
    assert B.e2eg_sample_capacity(1000, 10, [5, 3]) == 10 * 5 + 50 * 3
    assert B.e2eg_sample_capacity(20, 10, [5, 3]) == 10 * 5 + 20 * 3
    assert B.e2eg_sample_capacity(20, 50, [5]) == 20 * 5
    for bad in ([], [0], [5, 1 << 17], [2] * 9):
        with pytest.raises(B.E2egError):
            B.e2eg_sample_capacity(1000, 10, bad)
    with pytest.raises(B.E2egError):
        B.e2eg_sample_capacity(1 << 30, 1 << 30, [1 << 16])        # more draws than int32 holds
    assert B.e2eg_sample_subgraph_workspace_bytes(1000, 10, [5, 3]) > 0
    f = B.e2eg_sample_subgraph

    def call(n_users=600, n=1000, nnz=5000, table=FAKE, val=None, n_seeds=10, seeds=FAKE, fanout=(5, 3), nodes=FAKE,
             node_cap=1000, eu=FAKE, ei=FAKE, ew=None, edge_cap=200, ws=FAKE, wsb=big):
        return status_of(B, f, n_users, n, nnz, FAKE, FAKE, table, val, n_seeds, seeds, list(fanout), 7, nodes, node_cap,
                         eu, ei, ew, edge_cap, ws, wsb)

    assert call(n_users=2000) == B.E2EG_ERR_INVALID_ARG
    assert call(fanout=(5, 0)) == B.E2EG_ERR_INVALID_ARG
    assert call(table=None) == B.E2EG_ERR_NULL_PTR
    assert call(seeds=None) == B.E2EG_ERR_NULL_PTR
    assert call(ew=FAKE) == B.E2EG_ERR_NULL_PTR                   # weights asked for, no values given
    assert call(edge_cap=199) == B.E2EG_ERR_CAPACITY
    assert call(node_cap=209) == B.E2EG_ERR_CAPACITY
    assert call(wsb=64) == B.E2EG_ERR_WORKSPACE
    assert f(600, 1000, 5000, FAKE, FAKE, FAKE, None, 0, None, [5, 3], 7, FAKE, 1000, FAKE, FAKE, None, 200, FAKE, big) == (0, 0, 0)


def test_profile_aid_rejects_bad_arguments(B):
    assert status_of(B, B.e2eg_profile_begin, -1) == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, B.e2eg_profile_copy, None, None, 16) == B.E2EG_ERR_NULL_PTR
    assert status_of(B, B.e2eg_profile_copy, 4096, 8192, 24) == B.E2EG_ERR_INVALID_ARG


def test_device_helpers_refuse_to_run_without_gpu():
    torch = pytest.importorskip("torch")
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    import paper_2511_20564_amd.device as dev
    with pytest.raises(RuntimeError):
        dev.propagate_fwd(None, torch.zeros(4, 4), 1)


def test_noalloc_transform_checks_arguments_before_it_touches_the_device(B):
    f = B.e2eg_layer_transform_noalloc
    fwd, bwd = B.E2EG_TRANSFORM_FWD, B.E2EG_TRANSFORM_BWD
    assert status_of(B, f, 7, 10, 128, 128, B.E2EG_BF16, 1, FAKE, FAKE, FAKE, None, None, None) == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, f, fwd, 10, 128, 128, B.E2EG_F32, 1, FAKE, FAKE, FAKE, None, None, None) == B.E2EG_ERR_BAD_DTYPE
    assert status_of(B, f, fwd, 10, 100, 128, B.E2EG_BF16, 1, FAKE, FAKE, FAKE, None, None, None) == B.E2EG_ERR_INVALID_ARG
    assert status_of(B, f, fwd, 10, 128, 128, B.E2EG_BF16, 1, None, FAKE, FAKE, None, None, None) == B.E2EG_ERR_NULL_PTR
    assert status_of(B, f, bwd, 10, 128, 128, B.E2EG_BF16, 1, FAKE, FAKE, FAKE, None, FAKE, FAKE) == B.E2EG_ERR_NULL_PTR
    # more partial matrices than the static array holds: refused on the host, nothing enqueued
    assert B.e2eg_layer_transform_workspace_bytes(bwd, 100_000, 256, 256, B.E2EG_BF16) > 16 << 20
    assert status_of(B, f, bwd, 100_000, 256, 256, B.E2EG_BF16, 1, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE) == B.E2EG_ERR_CAPACITY
    assert "static array" in B.e2eg_last_error()
    # any n fits with 128 x 128 weights
    assert B.e2eg_layer_transform_workspace_bytes(bwd, 2_000_000_000, 128, 128, B.E2EG_BF16) <= 16 << 20
