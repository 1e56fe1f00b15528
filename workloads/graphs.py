"""Seeded generators for user-item interaction graphs and node features.

The paper's graphs are production interaction logs that are not public, so
synthetic bipartite graphs stand in for them: a uniform tiny one, power-law
ones (Zipf item popularity, log-normal user activity) and a two-hop sampled
mini-batch subgraph with the fan-outs of the paper's experiment section
(Section 5, "Subgraph Sampling").  Everything here is input generation; no
normalisation, propagation or transform arithmetic lives in this module.
"""
from __future__ import annotations

import hashlib
import os

import numpy as np

BASE_SEED = 20251120

# The five workloads.  `n_edges` counts distinct (user, item) pairs.
CONFIGS = {
    1: dict(name="tiny", kind="uniform", n_users=2_000, n_items=1_000, n_edges=20_000,
            F=64, dtype="f32", K=2),
    2: dict(name="medium", kind="powerlaw", n_users=100_000, n_items=50_000, n_edges=2_000_000,
            zipf_s=1.0, dmax=2000, item_cap=None, F=64, dtype="f32", K=3),
    3: dict(name="large", kind="powerlaw", n_users=1_000_000, n_items=500_000, n_edges=50_000_000,
            zipf_s=1.1, dmax=2000, item_cap=None, F=128, dtype="bf16", K=3),
    4: dict(name="minibatch", kind="sampled", parent=3, n_seeds=4096, fanout=(25, 10),
            F=128, dtype="bf16", K=2, transform=True),
    5: dict(name="xlarge", kind="powerlaw", n_users=10_000_000, n_items=2_000_000,
            n_edges=500_000_000, zipf_s=1.1, dmax=2000, item_cap=100_000, F=64, dtype="bf16", K=3),
}


# --------------------------------------------------------------------------
# bf16 encoding of inputs (round-to-nearest-even on the upper 16 bits of fp32)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 array of bf16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> the fp32 values they denote (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_features(n: int, F: int, std: float, seed: int, dtype: str) -> np.ndarray:
    """[n, F] array ~ N(0, std^2).  dtype 'f32' -> float32 values; 'bf16' -> uint16
    bit patterns of the RNE-rounded values (that array *is* the input)."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, F), dtype=np.float32)
    x *= np.float32(std)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def make_edge_weights(n_edges: int, seed: int) -> np.ndarray:
    """Interaction strengths for a weighted graph: float32, log-normal around 1 (a few repeat
    visits are common, heavy engagement is rare), clipped to [0.05, 50]."""
    rng = np.random.default_rng(seed)
    w = np.exp(rng.standard_normal(n_edges, dtype=np.float32) * np.float32(0.8))
    return np.clip(w, np.float32(0.05), np.float32(50.0)).astype(np.float32)


# --------------------------------------------------------------------------
# edge lists
# --------------------------------------------------------------------------
def uniform_bipartite(n_users: int, n_items: int, n_edges: int, seed: int):
    """`n_edges` distinct (user, item) pairs, uniform over the n_users x n_items grid,
    returned in shuffled order as two int32 arrays."""
    if n_edges > n_users * n_items:
        raise ValueError("more edges than user-item pairs")
    rng = np.random.default_rng(seed)
    if 2 * n_edges > n_users * n_items:   # dense: draw the pairs directly
        keys = rng.choice(n_users * n_items, size=n_edges, replace=False).astype(np.int64)
        return (keys // n_items).astype(np.int32), (keys % n_items).astype(np.int32)
    keys = np.empty(0, dtype=np.int64)
    while keys.size < n_edges:
        extra = rng.integers(0, n_users * n_items, size=n_edges - keys.size, dtype=np.int64)
        keys = np.unique(np.concatenate([keys, extra]))
    keys = rng.permutation(keys)
    return (keys // n_items).astype(np.int32), (keys % n_items).astype(np.int32)


def _user_degrees(rng, n_users, n_items, n_edges, dmin, dmax):
    """Log-normal(2.5, 1.0) activity, rescaled so that it sums to n_edges, rounded,
    clipped to [dmin, dmax], then nudged by +-1 on random users until the sum is exact."""
    hi = min(dmax, n_items)
    if not (n_users * dmin <= n_edges <= n_users * hi):
        raise ValueError("edge count not reachable with these degree bounds")
    raw = rng.lognormal(2.5, 1.0, n_users)
    deg = np.clip(np.rint(raw * (n_edges / raw.sum())).astype(np.int64), dmin, hi)
    diff = int(n_edges - deg.sum())
    while diff != 0:
        step = 1 if diff > 0 else -1
        elig = np.flatnonzero(deg < hi) if step > 0 else np.flatnonzero(deg > dmin)
        take = min(abs(diff), elig.size)
        pick = rng.choice(elig, size=take, replace=False)
        deg[pick] += step
        diff -= step * take
    return deg


def _item_cdf(n_items, zipf_s, n_edges, item_cap):
    """Cumulative popularity over ranks 1..n_items: p_r ~ r^-s, optionally flattened
    at the head (p_r ~ min(r^-s, c)) so the most popular item expects ~item_cap edges."""
    w = np.arange(1, n_items + 1, dtype=np.float64) ** (-zipf_s)
    if item_cap is not None and n_edges * w[0] / w.sum() > item_cap:
        lo, hi = w[-1], w[0]
        for _ in range(80):  # bisection on the plateau height c
            c = 0.5 * (lo + hi)
            if n_edges * c / np.minimum(w, c).sum() > item_cap:
                hi = c
            else:
                lo = c
        w = np.minimum(w, 0.5 * (lo + hi))
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    return cdf


def _in_sorted(sorted_keys, q):
    if sorted_keys.size == 0:
        return np.zeros(q.shape, dtype=bool)
    pos = np.searchsorted(sorted_keys, q)
    pos[pos == sorted_keys.size] = sorted_keys.size - 1
    return sorted_keys[pos] == q


def powerlaw_bipartite(n_users, n_items, n_edges, zipf_s, seed, dmin=1, dmax=2000,
                       item_cap=None, max_rounds=96, verbose=False):
    """Power-law bipartite graph: each user draws its items *without replacement* from a
    Zipf(s) popularity over item ranks (ranks mapped to ids by a seeded permutation, so
    popular items are not id-contiguous).  Drawing with replacement and dropping repeats,
    round after round until every user holds its target count, is that same successive
    sampling.  Returns shuffled int32 arrays (users, items); the realised number of
    pairs can fall short of n_edges by the few draws still missing after `max_rounds`.
    """
    rng = np.random.default_rng(seed)
    deg = _user_degrees(rng, n_users, n_items, n_edges, dmin, dmax)
    cdf = _item_cdf(n_items, zipf_s, n_edges, item_cap)
    perm = rng.permutation(n_items).astype(np.int64)
    uid = np.arange(n_users, dtype=np.int64)

    main = np.empty(0, dtype=np.int64)   # sorted keys user*n_items+item
    side = np.empty(0, dtype=np.int64)   # sorted, small; folded into main now and then
    need = deg.copy()
    for rnd in range(max_rounds):
        total = int(need.sum())
        if total == 0:
            break
        u = np.repeat(uid, need)
        r = np.searchsorted(cdf, rng.random(total), side="right")
        np.minimum(r, n_items - 1, out=r)
        cand = np.unique(u * n_items + perm[r])
        del u, r
        if main.size:
            cand = cand[~_in_sorted(main, cand)]
        if side.size:
            cand = cand[~_in_sorted(side, cand)]
        need -= np.bincount(cand // n_items, minlength=n_users)
        if main.size == 0:
            main = cand
        else:
            side = np.sort(np.concatenate([side, cand]), kind="stable")
            if side.size > main.size // 8:
                main = np.sort(np.concatenate([main, side]), kind="stable")
                side = np.empty(0, dtype=np.int64)
        if verbose:
            print(f"  [powerlaw] round {rnd}: missing {int(need.sum())}", flush=True)
    keys = np.concatenate([main, side]) if side.size else main
    keys = rng.permutation(keys)
    return (keys // n_items).astype(np.int32), (keys % n_items).astype(np.int32)


# --------------------------------------------------------------------------
# mini-batch: uniform two-hop neighbour sampling, relabelled to local ids
# --------------------------------------------------------------------------
def _adjacency(rows, cols, n_rows):
    order = np.argsort(rows, kind="stable")
    ptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=n_rows), out=ptr[1:])
    return ptr, cols[order]


def _sample_neighbours(rng, ptr, nbr, nodes, fanout):
    """For each node: all its neighbours if it has <= fanout, else `fanout` of them
    uniformly without replacement.  Returns (node_of_each_pick, picked_neighbour)."""
    deg = ptr[nodes + 1] - ptr[nodes]
    src_out, nbr_out = [], []
    # (a) short lists: take everything
    small = deg <= fanout
    if small.any():
        nn, dd = nodes[small], deg[small]
        src = np.repeat(nn, dd)
        off = np.arange(dd.sum()) - np.repeat(np.cumsum(dd) - dd, dd)
        src_out.append(src)
        nbr_out.append(nbr[ptr[src] + off])
    # (b) moderately long lists: random key per neighbour, keep the `fanout` smallest
    mid = (~small) & (deg <= 8 * fanout)
    if mid.any():
        nn, dd = nodes[mid], deg[mid]
        src = np.repeat(nn, dd)
        seg = np.repeat(np.arange(nn.size), dd)
        off = np.arange(dd.sum()) - np.repeat(np.cumsum(dd) - dd, dd)
        key = rng.random(src.size)
        order = np.lexsort((key, seg))
        rank = np.arange(src.size) - np.repeat(np.cumsum(dd) - dd, dd)  # rank within segment after sort
        keep = order[rank < fanout]
        src_out.append(src[keep])
        nbr_out.append(nbr[ptr[src[keep]] + off[keep]])
    # (c) long lists: draw positions, redraw the repeats
    big = deg > 8 * fanout
    if big.any():
        nn, dd = nodes[big], deg[big]
        seg = np.repeat(np.arange(nn.size), fanout)
        pos = (rng.random(seg.size) * dd[seg]).astype(np.int64)
        while True:
            key = seg * (int(dd.max()) + 1) + pos
            _, first = np.unique(key, return_index=True)
            dup = np.ones(key.size, dtype=bool)
            dup[first] = False
            if not dup.any():
                break
            pos[dup] = (rng.random(int(dup.sum())) * dd[seg[dup]]).astype(np.int64)
        src_out.append(nn[seg])
        nbr_out.append(nbr[ptr[nn[seg]] + pos])
    return np.concatenate(src_out), np.concatenate(nbr_out)


def sample_subgraph(users, items, n_users, n_items, n_seeds, fanout, seed):
    """Two-hop uniform neighbour sampling from a bipartite graph, relabelled to local ids.

    hop 1: up to fanout[0] items of every seed user; hop 2: up to fanout[1] users of every
    distinct hop-1 item.  Local users = seeds (ascending global id) followed by the new
    hop-2 users (ascending); local items = hop-1 items (ascending).  Returns a dict with
    local int32 edge arrays (distinct pairs) and the global ids of the local nodes.
    """
    rng = np.random.default_rng(seed)
    users = users.astype(np.int64)
    items = items.astype(np.int64)
    uptr, unbr = _adjacency(users, items, n_users)
    iptr, inbr = _adjacency(items, users, n_items)
    seeds = np.sort(rng.choice(n_users, size=n_seeds, replace=False)).astype(np.int64)
    s1, i1 = _sample_neighbours(rng, uptr, unbr, seeds, fanout[0])
    hop1_items = np.unique(i1)
    i2, u2 = _sample_neighbours(rng, iptr, inbr, hop1_items, fanout[1])
    new_users = np.setdiff1d(np.unique(u2), seeds)
    g_users = np.concatenate([seeds, new_users])
    g_items = hop1_items
    # local ids
    order = np.argsort(g_users, kind="stable")
    su = g_users[order]

    def local_user(g):
        return order[np.searchsorted(su, g)]

    eu = np.concatenate([local_user(s1), local_user(u2)])
    ei = np.concatenate([np.searchsorted(g_items, i1), np.searchsorted(g_items, i2)])
    keys = np.unique(eu * g_items.size + ei)
    keys = rng.permutation(keys)
    return dict(
        n_users=int(g_users.size), n_items=int(g_items.size),
        users=(keys // g_items.size).astype(np.int32), items=(keys % g_items.size).astype(np.int32),
        global_users=g_users, global_items=g_items, n_seeds=int(n_seeds),
    )


# --------------------------------------------------------------------------
# whole configurations
# --------------------------------------------------------------------------
def _cache_path(tag: str):
    root = os.environ.get("E2EG_WORKLOAD_CACHE", "")
    if not root:
        return None
    if tag.startswith("xlarge|"):      # too large to be worth writing to disk
        return None
    os.makedirs(root, exist_ok=True)
    return os.path.join(root, hashlib.sha1(tag.encode()).hexdigest()[:16] + ".npz")


def _edges(cfg: dict, seed: int, scale: float, verbose: bool):
    nu = max(8, int(round(cfg["n_users"] * scale)))
    ni = max(8, int(round(cfg["n_items"] * scale)))
    ne = max(8, int(round(cfg["n_edges"] * scale)))
    tag = f"{cfg['name']}|{seed}|{nu}|{ni}|{ne}|v1"
    path = _cache_path(tag)
    if path and os.path.exists(path):
        z = np.load(path)
        return nu, ni, z["users"], z["items"]
    if cfg["kind"] == "uniform":
        users, items = uniform_bipartite(nu, ni, ne, seed)
    else:
        cap = cfg["item_cap"]
        if cap is not None:
            cap = max(4, int(round(cap * scale)))
        users, items = powerlaw_bipartite(nu, ni, ne, cfg["zipf_s"], seed, dmin=1,
                                          dmax=cfg["dmax"], item_cap=cap, verbose=verbose)
    if path:
        tmp = path + f".{os.getpid()}.tmp.npz"
        np.savez(tmp, users=users, items=items)
        os.replace(tmp, path)
    return nu, ni, users, items


def make_config(idx: int, seed: int | None = None, scale: float = 1.0, features: bool = True,
                verbose: bool = False) -> dict:
    """Build workload `idx` (1..5).  `scale` shrinks node and edge counts together (tests
    use it for cases the oracle finishes quickly); 1.0 is the stated size.

    Returns a dict: n_users, n_items, users, items (int32 edge arrays, distinct pairs,
    shuffled), F, dtype ('f32' | 'bf16'), K, and if `features`: X0 and gY as [n, F] arrays
    (float32 values, or uint16 bf16 bit patterns), plus W (list of K [F, F] arrays) for
    the mini-batch workload.
    """
    cfg = CONFIGS[idx]
    seed = BASE_SEED + idx if seed is None else seed
    out = dict(index=idx, name=cfg["name"], F=cfg["F"], dtype=cfg["dtype"], K=cfg["K"], seed=seed,
               transform=bool(cfg.get("transform", False)))
    if cfg["kind"] == "sampled":
        parent = CONFIGS[cfg["parent"]]
        pseed = BASE_SEED + cfg["parent"]
        pnu, pni, pusers, pitems = _edges(parent, pseed, scale, verbose)
        n_seeds = max(4, int(round(cfg["n_seeds"] * scale)))
        sub = sample_subgraph(pusers, pitems, pnu, pni, n_seeds, cfg["fanout"], seed)
        out.update(sub)
        if features:
            # rows of the parent's feature table (users first, then items)
            px = make_features(pnu + pni, parent["F"], 0.1, pseed + 1000, parent["dtype"])
            rows = np.concatenate([sub["global_users"], pnu + sub["global_items"]])
            out["X0"] = np.ascontiguousarray(px[rows])
            del px
    else:
        nu, ni, users, items = _edges(cfg, seed, scale, verbose)
        out.update(n_users=nu, n_items=ni, users=users, items=items)
        if features:
            out["X0"] = make_features(nu + ni, cfg["F"], 0.1, seed + 1000, cfg["dtype"])
    n = out["n_users"] + out["n_items"]
    out["n"] = n
    out["n_edges"] = int(out["users"].size)
    if features:
        out["gY"] = make_features(n, cfg["F"], 1.0, seed + 2000, cfg["dtype"])
        if out["transform"]:
            F = cfg["F"]
            out["W"] = [make_features(F, F, (1.0 / F) ** 0.5, seed + 3000 + k, cfg["dtype"])
                        for k in range(cfg["K"])]
    return out
