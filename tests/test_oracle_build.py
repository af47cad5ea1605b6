"""Pins for robustPrune and batch insertion (no GPU)."""
import os

import numpy as np
import pytest

import oracle
from paper_2601_07048_amd import datagen


def _read(golden_dir, name):
    return [l for l in open(os.path.join(golden_dir, name)) if l.strip() and not l.startswith("#")]


def test_prune_1d_golden(golden_dir):
    for line in _read(golden_dir, "prune_1d.txt"):
        head, cand, kept = [s.split() for s in line.split("|")]
        alpha, R = float(head[0]), int(head[1])
        coords = [0.0] + [float(c) for c in cand]
        base = np.zeros((len(coords), 4), np.float32)
        base[:, 0] = coords
        ids = np.arange(1, len(coords), dtype=np.uint32)
        dist = np.array([c * c for c in coords[1:]], np.float64)
        out = oracle.robust_prune(0, ids, dist, base, R, alpha)
        assert [coords[i] for i in out] == [float(k) for k in kept], line
        # candidate order must not matter
        perm = np.random.default_rng(0).permutation(len(ids))
        out2 = oracle.robust_prune(0, ids[perm], dist[perm], base, R, alpha)
        assert out2.tolist() == out.tolist()


def test_prune_orthogonal_axes_is_top_R():
    """Candidates s_i*e_i on distinct axes from p = 0: alpha*(s_i^2+s_j^2) <=
    s_j^2 never holds for alpha >= 1, so nothing is discarded and the result
    is the plain top-R by (distance, id)."""
    d = 32
    rng = np.random.default_rng(5)
    s = rng.integers(1, 20, d).astype(np.float32)
    base = np.zeros((d + 1, d), np.float32)
    for i in range(d):
        base[i + 1, i] = s[i]
    ids = np.arange(1, d + 1, dtype=np.uint32)
    dist = (s.astype(np.float64)) ** 2
    for R in (5, 32, 64):
        out = oracle.robust_prune(0, ids, dist, base, R, 1.2)
        expect = [int(ids[i]) for i in np.lexsort((ids, dist))[:R]]
        assert out.tolist() == expect


def test_prune_removes_self_and_duplicates():
    base = np.zeros((4, 4), np.float32)
    base[:, 0] = [0, 1, -2, 40]
    ids = np.array([0, 1, 1, 2, 3, 3, 0xFFFFFFFF], np.uint32)
    dist = np.array([0, 1, 1, 4, 1600, 1600, 0], np.float64)
    out = oracle.robust_prune(0, ids, dist, base, 8, 1.0)
    # 1 kept; -2: d(1,-2)=9<=4 no -> kept; 40: d(1,40)=1521<=1600 -> dropped
    assert out.tolist() == [1, 2]


def _check_alpha_rule(p, cand_ids, cand_dist, base, R, alpha, out):
    """Brute-force validation of the output against the definition: walk the
    candidates in (distance,id) order; a candidate is kept iff no earlier kept
    candidate p* has alpha*d(p*,c) <= d(p,c); stop at R."""
    order = sorted(set(zip(cand_dist.tolist(), cand_ids.tolist())))
    kept = []
    a32 = np.float32(alpha)
    for dpc, c in order:
        if c == p or len(kept) == R:
            continue
        dead = False
        for s in kept:
            dsc = np.float32(oracle.l2sq(base[s], base[c]))
            if a32 * dsc <= np.float32(dpc):
                dead = True
                break
        if not dead:
            kept.append(c)
    assert out.tolist() == kept


@pytest.mark.parametrize("dtype", [np.uint8, np.float32])
def test_prune_alpha_rule_invariant(dtype):
    rng = np.random.default_rng(6)
    n, d = 400, 16
    base = (rng.integers(0, 256, (n, d), dtype=np.uint8) if dtype == np.uint8
            else rng.standard_normal((n, d)).astype(np.float32))
    for trial in range(5):
        p = int(rng.integers(0, n))
        cand = rng.choice(n, 120, replace=False).astype(np.uint32)
        dist = np.array([oracle.l2sq(base[p], base[c]) for c in cand], np.float64)
        for R, alpha in ((8, 1.0), (32, 1.2), (200, 1.2)):
            out = oracle.robust_prune(p, cand, dist, base, R, alpha)
            assert len(out) <= R and p not in out and len(set(out.tolist())) == len(out)
            _check_alpha_rule(p, cand, dist, base, R, alpha, out)


def test_insert_1d_golden(golden_dir):
    lines = _read(golden_dir, "insert_1d.txt")
    entry = int(lines[0].split()[1])
    rows = {int(l.split("|")[0]): [int(t) for t in l.split("|")[1].split()] for l in lines[1:]}
    base = np.zeros((5, 4), np.float32)
    base[:, 0] = [0, 10, 4, 5, 20]
    for nt in (1, 3):
        ix = oracle.Index(4, np.float32, 2, 4, 1.2, 8, batch_growth=1.0)
        ix.insert(base, nthreads=nt)
        adj, deg = ix.graph()
        assert ix.entry == entry and ix.n == 5
        for i in range(5):
            assert adj[i, : deg[i]].tolist() == rows[i], (i, adj[i])
            assert (adj[i, deg[i]:] == oracle.NONE).all()


def _graph_invariants(adj, deg, n, R):
    assert adj.shape == (n, R)
    for i in range(n):
        row = adj[i, : deg[i]]
        assert (adj[i, deg[i]:] == oracle.NONE).all()
        assert (row < n).all() and i not in row
        assert len(set(row.tolist())) == len(row)


@pytest.mark.parametrize("workload,n,R,L", [(1, 1500, 12, 24), (2, 1500, 16, 32)])
def test_insert_invariants_and_incremental(workload, n, R, L):
    x = datagen.base(workload, n)
    a = oracle.Index(x.shape[1], x.dtype, R, L, 1.2, n)
    a.insert(x[:1000])
    adj0, deg0 = a.graph()
    _graph_invariants(adj0, deg0, 1000, R)
    a.insert(x[1000:])
    adj, deg = a.graph()
    _graph_invariants(adj, deg, n, R)
    assert (deg >= 1).all()
    # thread count must not change the graph (disjoint rows, total orders)
    b = oracle.Index(x.shape[1], x.dtype, R, L, 1.2, n)
    b.insert(x[:1000], nthreads=1)
    b.insert(x[1000:], nthreads=1)
    adjb, _ = b.graph()
    assert np.array_equal(adj, adjb) and a.entry == b.entry
    # entry: nearest point of the first call to that call's mean
    m = x[:1000].astype(np.float64).mean(0).astype(np.float32).astype(np.float64)
    dm = ((x[:1000].astype(np.float64) - m) ** 2).sum(1)
    assert a.entry == int(np.argmin(dm))
    # almost every vertex reachable from the entry (robustPrune may drop the
    # last in-edge of a vertex, so reachability is not guaranteed by the method)
    seen = np.zeros(n, bool)
    stack = [a.entry]
    seen[a.entry] = True
    while stack:
        u = stack.pop()
        for v in adj[u, : deg[u]]:
            if not seen[v]:
                seen[v] = True
                stack.append(int(v))
    assert seen.mean() > 0.9


def test_cand_mode_visited_superset_quality():
    """Frontier candidates (Alg. 2's output) vs expansion-list candidates
    (Alg. 4 as printed): both must give a navigable graph."""
    x = datagen.base(1, 2000)
    q = datagen.queries(1, 200)
    gt, _ = oracle.bruteforce(x, q, 10)
    rec = []
    for mode in (oracle.CAND_FRONTIER, oracle.CAND_VISITED):
        ix = oracle.Index(128, np.float32, 16, 32, 1.2, 2000, cand_mode=mode)
        ix.insert(x)
        rec.append(oracle.recall_at_k(ix.search(q, 10, 32)["ids"], gt))
    assert min(rec) > 0.9 and abs(rec[0] - rec[1]) < 0.05


def test_workload1_recall_target():
    """Workload 1 of the benchmark definition: N=10,000, R=32, L_build=64,
    alpha=1.2, seeded random insertion order; search L=64, k=10 must reach
    recall@10 >= 0.95 against brute force."""
    n = 10000
    x = datagen.base(1, n)[datagen.insertion_order(1, n)]
    q = datagen.queries(1, 1000)
    ix = oracle.Index(128, np.float32, 32, 64, 1.2, n)
    ix.insert(x)
    adj, deg = ix.graph()
    _graph_invariants(adj, deg, n, 32)
    gt, _ = oracle.bruteforce(x, q, 10)
    rec = oracle.recall_at_k(ix.search(q, 10, 64)["ids"], gt)
    assert rec >= 0.95, rec


# ---------------------------------------------------------------------------------------------------------------
# The batch schedule (Sec. 3.2 / 3.4, Alg. 4; batch-size sweep of Sec. 6.2).  The schedule cuts a call into
# internal batches of min(remaining, max(1, floor(batch_growth * linked))) points; these pins fix what the
# batching may and may not change.

def _sequential_vamana(x, R, L, alpha, entry, v_cap=0):
    """One-at-a-time insertion written out from Sec. 3.1 / Alg. 3-4 with batches of one, from the separately pinned
    primitives (beamSearch, robustPrune, distance): search from the entry point on the graph as it stands, prune the
    frontier into the new row, then add the reverse edge to every kept neighbour -- appended while the row has room,
    else the row becomes robustPrune(row + new point)."""
    n = len(x)
    adj = np.full((n, R), oracle.NONE, np.uint32)
    deg = np.zeros(n, np.int64)
    for p in range(n):
        if p == entry:
            continue
        res = oracle.beam_search(adj, x, x[p], L, entry, V_cap=v_cap)
        if v_cap:   # Alg. 4 step 2 as printed: prune the expansion list V (its first v_cap entries)
            row = oracle.robust_prune(p, res["V_ids"], res["V_dist"], x, R, alpha)
        else:       # Alg. 2's output: the final frontier
            row = oracle.robust_prune(p, res["F_ids"], res["F_dist"], x, R, alpha)
        adj[p, : len(row)] = row
        deg[p] = len(row)
        for v in row.tolist():
            if p in adj[v, : deg[v]]:
                continue
            if deg[v] < R:
                adj[v, deg[v]] = p
                deg[v] += 1
            else:
                cand = np.append(adj[v, : deg[v]], np.uint32(p)).astype(np.uint32)
                dist = np.array([oracle.l2sq(x[v], x[c]) for c in cand], np.float64)
                new = oracle.robust_prune(v, cand, dist, x, R, alpha)
                adj[v] = oracle.NONE
                adj[v, : len(new)] = new
                deg[v] = len(new)
    return adj


@pytest.mark.parametrize("dtype", [np.uint8, np.float32])
def test_all_ones_schedule_is_sequential_insertion(dtype):
    """batch_growth -> 0 gives internal batches of one point each; the batch machinery (snapshot search, edge
    sort, per-target merge) must then reproduce plain sequential insertion, row for row.  R is small so that most
    reverse edges overflow their row and take the prune branch."""
    rng = np.random.default_rng(21)
    n, d, R, L = 260, 16, 5, 12
    if dtype == np.uint8:
        x = rng.integers(0, 256, (n, d), dtype=np.uint8)
    else:
        x = rng.standard_normal((n, d)).astype(np.float32)
    ix = oracle.Index(d, dtype, R, L, 1.2, n, batch_growth=0.0)
    ix.insert(x[:200])
    ix.insert(x[200:])      # a second call continues the same schedule
    got, _ = ix.graph()
    want = _sequential_vamana(x, R, L, 1.2, ix.entry)
    assert np.array_equal(got, want)
    # and a real batch schedule does change the graph: the pin above is not vacuous
    iy = oracle.Index(d, dtype, R, L, 1.2, n, batch_growth=1.0)
    iy.insert(x)
    assert not np.array_equal(iy.graph()[0], want)
    # expansion-list candidates (the list holds min(512, 4 L rounded up to a power of two) = 64 entries for L = 12)
    iv = oracle.Index(d, dtype, R, L, 1.2, n, batch_growth=0.0, cand_mode=oracle.CAND_VISITED)
    iv.insert(x)
    want_v = _sequential_vamana(x, R, L, 1.2, iv.entry, v_cap=64)
    assert np.array_equal(iv.graph()[0], want_v)
    assert not np.array_equal(want_v, want)


def _edge_set(adj):
    src, col = np.nonzero(adj != oracle.NONE)
    return set(zip(src.tolist(), adj[src, col].tolist()))


def test_an_insertion_adds_at_most_2R_edges():
    """Sec. 3.4: inserting a point adds at most 2R edges -- its own row (<= R) and one reverse edge into each kept
    neighbour's row (<= R); pruning an overflowing row only removes edges.  Every edge that is new after a call
    therefore has a point of that call as source or target, and there are at most 2R of them per inserted point."""
    rng = np.random.default_rng(22)
    n0, d, R, L = 400, 16, 6, 16
    x = rng.integers(0, 256, (n0 + 60, d), dtype=np.uint8)
    ix = oracle.Index(d, np.uint8, R, L, 1.2, len(x), batch_growth=0.25)
    ix.insert(x[:n0])
    before = _edge_set(ix.graph()[0])
    # single points, then one batch of 40 (one internal batch: 0.25 * 420 > 40)
    for lo, hi in [(n0 + i, n0 + i + 1) for i in range(20)] + [(n0 + 20, n0 + 60)]:
        ix.insert(x[lo:hi])
        after = _edge_set(ix.graph()[0])
        new = after - before
        assert len(new) <= 2 * R * (hi - lo)
        assert all(lo <= s < hi or lo <= t < hi for s, t in new)
        # each new point has at most R out-edges and is named by at most R rows
        for p in range(lo, hi):
            assert sum(1 for s, t in new if s == p) <= R and sum(1 for s, t in new if t == p and not lo <= s < hi) <= R
        before = after


def test_recall_barely_depends_on_the_batch_size():
    """Sec. 6.2 (batch-size sweep): recall changes by less than two points between small and large batches.
    Workload 1, recall@10 at L = 64, internal batches of 0.5 % to 32 % of the linked points (the paper's range)."""
    n, nq, k = 10_000, 500, 10
    x = datagen.base(1, n)[datagen.insertion_order(1, n)]
    q = datagen.queries(1, nq)
    gt, _ = oracle.bruteforce(x, q, k)
    rec = {}
    for growth in (0.005, 0.02, 0.05, 0.25, 0.32):
        ix = oracle.Index(128, np.float32, 32, 64, 1.2, n, batch_growth=growth)
        ix.insert(x)
        rec[growth] = oracle.recall_at_k(ix.search(q, k, 64)["ids"], gt)
    assert max(rec.values()) - min(rec.values()) < 0.02, rec
    assert min(rec.values()) >= 0.95, rec
