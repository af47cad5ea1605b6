"""Pins for the oracle's batch deletion (Sec. 4.6).  No GPU."""
import os

import numpy as np

import oracle
from paper_2601_07048_amd import datagen


def test_delete_1d_golden(golden_dir):
    lines = [l for l in open(os.path.join(golden_dir, "delete_1d.txt")) if l.strip() and not l.startswith("#")]
    entry = int(lines[0].split()[1])
    rows = {int(l.split("|")[0]): [int(t) for t in l.split("|")[1].split()] for l in lines[1:]}
    base = np.zeros((5, 4), np.float32)
    base[:, 0] = [0, 10, 4, 5, 20]
    ix = oracle.Index(4, np.float32, 2, 4, 1.2, 8, batch_growth=1.0)
    ix.insert(base)
    ix.delete([1, 1, 77])  # repeated / unknown ids are ignored
    assert ix.n_deleted == 1
    # marked only: still traversed, never returned
    r = ix.search(np.array([[9.0, 0, 0, 0]], np.float32), 2, 4)
    assert r["ids"][0].tolist() == [3, 2]
    ix.consolidate()
    adj, deg = ix.graph()
    assert ix.entry == entry
    for i in range(5):
        assert adj[i, :deg[i]].tolist() == rows[i], (i, adj[i])


def test_delete_invariants_and_recall():
    n = 6000
    x = datagen.base(2, n)
    q = datagen.queries(2, 300)
    ix = oracle.Index(128, np.uint8, 32, 64, 1.2, n)
    ix.insert(x)
    rng = np.random.default_rng(1)
    dele = np.unique(np.concatenate([rng.choice(n, 600, replace=False), [ix.entry]])).astype(np.uint32)
    live = np.ones(n, bool)
    live[dele] = False
    lid = np.nonzero(live)[0]
    gt = lid[oracle.bruteforce(x[live], q, 10)[0]]
    before = oracle.recall_at_k(ix.search(q, 10, 64)["ids"], oracle.bruteforce(x, q, 10)[0])
    ix.delete(dele)
    r = ix.search(q, 10, 64, want_frontier=True)
    assert not np.isin(r["ids"], dele).any() and not np.isin(r["F_ids"], dele).any()
    marked = oracle.recall_at_k(r["ids"], gt)
    ix.consolidate()
    adj, deg = ix.graph()
    assert (deg[~live] == 0).all()
    assert not np.isin(adj[live][adj[live] != oracle.NONE], dele).any()
    assert live[ix.entry]
    for i in lid[::97]:
        row = adj[i, :deg[i]]
        assert i not in row and len(set(row.tolist())) == len(row)
    after = oracle.recall_at_k(ix.search(q, 10, 64)["ids"], gt)
    # Sec. 6.4: deletion + consolidation keeps recall (0.986 -> 0.988 in the paper's Table 2)
    assert marked >= before - 0.02 and after >= before - 0.02
    # a second consolidate changes nothing; inserts after it never link to deleted vertices
    ix.consolidate()
    adj2, _ = ix.graph()
    assert np.array_equal(adj, adj2)
    ix2 = oracle.Index(128, np.uint8, 32, 64, 1.2, n + 500)
    ix2.insert(x)
    ix2.delete(dele)
    ix2.insert(datagen.base(2, 500, start=n))
    a3, d3 = ix2.graph()
    assert not np.isin(a3[n:][a3[n:] != oracle.NONE], dele).any()


def test_consolidate_rows_equal_prune_of_stated_candidates():
    """Each row after consolidation = robustPrune (pinned on its own) of the candidate set assembled here in
    numpy from the graph before the call; rows without a deleted neighbour do not change."""
    n, R = 1500, 12
    x = datagen.base(2, n)
    ix = oracle.Index(128, np.uint8, R, 32, 1.2, n)
    ix.insert(x)
    adj0, deg0 = ix.graph()
    rng = np.random.default_rng(8)
    dele = rng.choice(n, 300, replace=False).astype(np.uint32)
    dead = np.zeros(n, bool)
    dead[dele] = True
    ix.delete(dele)
    ix.consolidate()
    adj1, deg1 = ix.graph()
    xi = x.astype(np.int64)
    touched = 0
    for v in range(n):
        row = adj0[v, :deg0[v]]
        if dead[v]:
            assert deg1[v] == 0
            continue
        if not dead[row].any():
            assert np.array_equal(adj1[v], adj0[v])
            continue
        touched += 1
        cand = []
        for u in row:
            if not dead[u]:
                cand.append(int(u))
            else:
                cand += [int(w) for w in adj0[u, :deg0[u]] if not dead[w] and w != v]
        cand = np.array(sorted(set(cand)), np.uint32)
        dist = ((xi[cand] - xi[v]) ** 2).sum(axis=1).astype(np.float64)
        want = oracle.robust_prune(v, cand, dist, x, R, 1.2)
        assert adj1[v, :deg1[v]].tolist() == want.tolist(), v
    assert touched > 300


def test_compact_1d_golden(golden_dir):
    lines = [l for l in open(os.path.join(golden_dir, "compact_1d.txt")) if l.strip() and not l.startswith("#")]
    want_map = [oracle.NONE if t == "x" else int(t) for t in lines[0].split()[1:]]
    entry = int(lines[1].split()[1])
    rows = {int(l.split("|")[0]): [int(t) for t in l.split("|")[1].split()] for l in lines[2:]}
    base = np.zeros((5, 4), np.float32)
    base[:, 0] = [0, 10, 4, 5, 20]
    ix = oracle.Index(4, np.float32, 2, 4, 1.2, 8, batch_growth=1.0)
    ix.insert(base)
    ix.delete([1])
    with np.testing.assert_raises(RuntimeError):
        ix.compact()  # rows still name vertex 1
    ix.consolidate()
    m = ix.compact()
    assert m.tolist() == want_map
    assert ix.n == 4 and ix.entry == entry and ix.n_deleted == 0
    adj, deg = ix.graph()
    for i in range(4):
        assert adj[i, :deg[i]].tolist() == rows[i]
    # the moved vectors: nearest neighbour of coordinate 19 is now vertex 3 (coordinate 20)
    r = ix.search(np.array([[19.0, 0, 0, 0]], np.float32), 1, 4)
    assert r["ids"][0].tolist() == [3] and r["dist"][0].tolist() == [1.0]


def test_compact_is_a_renaming():
    """Compaction changes names only: rows, vectors, codes and every search result are the consolidated
    index's under the order-preserving map; later inserts continue from the new size."""
    n = 5000
    x = datagen.base(1, n)
    q = datagen.queries(1, 200)
    ix = oracle.Index(128, np.float32, 24, 48, 1.2, n + 300)
    ix.insert(x)
    P = datagen.random_orthogonal(128, seed=3).astype(np.float32)
    ix.quantize(4, P)
    rng = np.random.default_rng(2)
    dele = np.unique(np.concatenate([rng.choice(n, 700, replace=False), [ix.entry]])).astype(np.uint32)
    ix.delete(dele)
    ix.consolidate()
    adj0, deg0 = ix.graph()
    e0 = ix.entry
    r0 = ix.search(q, 10, 48)
    q0 = ix.search(q, 10, 48, mode=1, rerank=20)
    m = ix.compact()
    live = np.setdiff1d(np.arange(n), dele)
    assert ix.n == live.size and ix.n_deleted == 0
    assert np.array_equal(m[live], np.arange(live.size)) and (m[dele] == oracle.NONE).all()
    assert ix.entry == m[e0]
    adj1, deg1 = ix.graph()
    assert np.array_equal(deg1, deg0[live])
    ren = np.where(adj0[live] == oracle.NONE, oracle.NONE, m[np.minimum(adj0[live], n - 1)])
    assert np.array_equal(adj1, ren)
    r1 = ix.search(q, 10, 48)
    assert np.array_equal(r1["ids"], m[r0["ids"]]) and np.array_equal(r1["dist"], r0["dist"])
    q1 = ix.search(q, 10, 48, mode=1, rerank=20)
    assert np.array_equal(q1["ids"], m[q0["ids"]]) and np.array_equal(q1["dist"], q0["dist"])
    assert r1["hops"] == r0["hops"] and r1["evals"] == r0["evals"]
    # nothing deleted: the identity
    assert np.array_equal(ix.compact(), np.arange(live.size))
    ix.insert(datagen.base(1, 300, start=n))
    assert ix.n == live.size + 300
    a2, d2 = ix.graph()
    assert (a2[a2 != oracle.NONE] < ix.n).all() and d2[live.size:].min() >= 1
