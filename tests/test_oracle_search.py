"""Pins for the oracle's distances, brute force and beamSearch (no GPU)."""
import os

import numpy as np
import pytest

import oracle
from paper_2601_07048_amd import datagen


def _path_graph(n, R=2):
    adj = np.full((n, R), oracle.NONE, np.uint32)
    for i in range(n):
        row = [j for j in (i - 1, i + 1) if 0 <= j < n]
        adj[i, : len(row)] = row
    return adj


def test_distance_matches_numpy():
    rng = np.random.default_rng(1)
    a = rng.integers(0, 256, 128, dtype=np.uint8)
    b = rng.integers(0, 256, 128, dtype=np.uint8)
    assert oracle.l2sq(a, b) == int(((a.astype(np.int64) - b.astype(np.int64)) ** 2).sum())
    # worst case fits the int32 the GPU accumulates in: 128 * 255^2
    z = np.zeros(128, np.uint8)
    f = np.full(128, 255, np.uint8)
    assert oracle.l2sq(z, f) == 128 * 255 * 255
    x = rng.standard_normal(960).astype(np.float32)
    y = rng.standard_normal(960).astype(np.float32)
    ref = float(((x.astype(np.float64) - y.astype(np.float64)) ** 2).sum())
    assert abs(oracle.l2sq(x, y) - ref) <= 1e-12 * ref
    assert oracle.l2sq(x, x) == 0.0


def test_oracle_half_distance_is_exact():
    rng = np.random.default_rng(0)
    a = rng.standard_normal(96).astype(np.float16)
    b = rng.standard_normal(96).astype(np.float16)
    assert oracle.l2sq(a, b) == float(((a.astype(np.float64) - b.astype(np.float64)) ** 2).sum())
    h = np.array([0, 1, 0x03FF, 0x0400, 0x7BFF, 0x8001, 0xFBFF], np.uint16).view(np.float16)  # subnormals, extremes
    assert oracle.l2sq(h, np.zeros(7, np.float16)) == float((h.astype(np.float64) ** 2).sum())


def test_oracle_half_conversion_all_bit_patterns():
    """Every finite binary16 value, one at a time: (h - 0)^2 and (h - 1)^2 against numpy's conversion."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    h = bits.view(np.float16)
    fin = np.isfinite(h)
    zero, one = np.zeros(1, np.float16), np.ones(1, np.float16)
    h64 = h.astype(np.float64)
    for i in np.nonzero(fin)[0]:
        assert oracle.l2sq(h[i:i + 1], zero) == h64[i] * h64[i], hex(i)
    for i in np.nonzero(fin)[0][::7]:
        assert oracle.l2sq(one, h[i:i + 1]) == (1.0 - h64[i]) ** 2, hex(i)


@pytest.mark.parametrize("dtype", [np.uint8, np.float32])
def test_bruteforce_matches_scipy(dtype):
    from scipy.spatial.distance import cdist

    rng = np.random.default_rng(2)
    if dtype == np.uint8:
        base = rng.integers(0, 256, (500, 32), dtype=np.uint8)
        q = rng.integers(0, 256, (20, 32), dtype=np.uint8)
    else:
        base = rng.standard_normal((500, 32)).astype(np.float32)
        q = rng.standard_normal((20, 32)).astype(np.float32)
    ids, dist = oracle.bruteforce(base, q, 7)
    D = cdist(q.astype(np.float64), base.astype(np.float64), "sqeuclidean")
    for i in range(20):
        order = np.lexsort((np.arange(500), D[i]))[:7]
        assert np.allclose(dist[i], D[i][order], rtol=1e-12)
        # ids must agree wherever the distance is unique
        for j in range(7):
            if (np.abs(D[i] - D[i][order[j]]) < 1e-9).sum() == 1:
                assert ids[i, j] == order[j]


def test_bruteforce_ties_by_id_and_padding():
    base = np.zeros((3, 4), np.uint8)
    base[1, 0] = 1
    q = np.zeros((1, 4), np.uint8)
    ids, dist = oracle.bruteforce(base, q, 5)
    assert ids[0].tolist() == [0, 2, 1, oracle.NONE, oracle.NONE]
    assert dist[0][:3].tolist() == [0.0, 0.0, 1.0] and np.isinf(dist[0][3:]).all()


def test_beam_path_graph_golden(golden_dir):
    """Hand-worked expansion orders (Alg. 1 / Alg. 2)."""
    n = 10
    base = np.zeros((n, 4), np.float32)
    base[:, 0] = np.arange(n)
    adj = _path_graph(n)
    for line in open(os.path.join(golden_dir, "beam_path_graph.txt")):
        if line.startswith("#") or not line.strip():
            continue
        head, v, f = [s.split() for s in line.split("|")]
        q = np.array([float(head[0]), 0, 0, 0], np.float32)
        L = int(head[1])
        for flt in (oracle.FILTER_EXACT, oracle.FILTER_NONE):
            r = oracle.beam_search(adj, base, q, L, 0, filter=flt, V_cap=64)
            assert r["V_ids"].tolist() == [int(t) for t in v], (line, flt)
            assert r["F_ids"].tolist() == [int(t) for t in f], (line, flt)
            assert r["hops"] == len(v)


def test_beam_star_graph():
    """Star: centre 0 -> all leaves, leaves -> nothing.  One expansion of the
    centre sees every leaf; the result is the exact top-L of {centre} U leaves."""
    rng = np.random.default_rng(3)
    n = 40
    base = rng.integers(0, 256, (n, 16), dtype=np.uint8)
    adj = np.full((n, n - 1), oracle.NONE, np.uint32)
    adj[0] = np.arange(1, n)
    q = rng.integers(0, 256, 16, dtype=np.uint8)
    r = oracle.beam_search(adj, base, q, 8, 0, V_cap=64)
    gt, gd = oracle.bruteforce(base, q[None], 8)
    assert r["F_ids"].tolist() == gt[0].tolist()
    assert r["V_ids"][0] == 0 and r["nV"] == 8 if 0 in gt[0] else r["nV"] == 9
    assert r["evals"] == n


@pytest.mark.parametrize("dtype", [np.uint8, np.float32])
def test_beam_L_ge_N_equals_bruteforce(dtype):
    """With L >= N nothing is ever truncated, so the search is a full traversal
    of everything reachable: on a connected graph F is the exact kNN order."""
    n, d, R = 300, 24, 6
    rng = np.random.default_rng(4)
    if dtype == np.uint8:
        base = rng.integers(0, 256, (n, d), dtype=np.uint8)
        qs = rng.integers(0, 256, (10, d), dtype=np.uint8)
    else:
        base = rng.standard_normal((n, d)).astype(np.float32)
        qs = rng.standard_normal((10, d)).astype(np.float32)
    # ring + random chords: strongly connected
    adj = np.full((n, R), oracle.NONE, np.uint32)
    for i in range(n):
        nb = {(i + 1) % n}
        while len(nb) < R - 1:
            j = int(rng.integers(0, n))
            if j != i:
                nb.add(j)
        nb = list(nb)
        adj[i, : len(nb)] = nb
    gt, gd = oracle.bruteforce(base, qs, n)
    for i, q in enumerate(qs):
        for flt in (oracle.FILTER_EXACT, oracle.FILTER_NONE):
            r = oracle.beam_search(adj, base, q, n + 5, 7, filter=flt, V_cap=n + 5)
            assert r["nF"] == n
            assert r["F_ids"].tolist() == gt[i].tolist()
            assert np.array_equal(r["F_dist"], gd[i])
            assert r["nV"] == n  # every entry of F gets expanded
            assert sorted(r["V_ids"].tolist()) == list(range(n))
        assert r["evals"] >= n


def _small_index(n=3000, workload=1, R=16, L=32):
    x = datagen.base(workload, n)
    ix = oracle.Index(x.shape[1], x.dtype, R, L, 1.2, n)
    ix.insert(x)
    return x, ix


def test_filter_equivalence_on_built_graph():
    """An exact visited set (Alg. 1), or no filter with duplicates dropped
    (Alg. 2), give the same frontier; only the number of distance evaluations
    differs.  Checked on a Vamana graph for several L."""
    x, ix = _small_index()
    q = datagen.queries(1, 100)
    for L in (4, 10, 33, 64):
        a = ix.search(q, min(10, L), L, want_frontier=True)
        b = ix.search(q, min(10, L), L, filter=oracle.FILTER_NONE, want_frontier=True)
        assert np.array_equal(a["F_ids"], b["F_ids"])
        assert np.array_equal(a["F_dist"], b["F_dist"])
        assert a["hops"] == b["hops"]
        assert a["evals"] <= b["evals"]


def test_search_structure_and_determinism():
    x, ix = _small_index(n=2000, workload=2, R=32, L=24)
    q = datagen.queries(2, 50)
    a = ix.search(q, 10, 24, want_frontier=True, nthreads=1)
    b = ix.search(q, 10, 24, want_frontier=True, nthreads=4)
    assert np.array_equal(a["ids"], b["ids"]) and np.array_equal(a["F_dist"], b["F_dist"])
    F, D = a["F_ids"], a["F_dist"]
    for i in range(len(q)):
        # sorted by (distance, id), no duplicates, distances are the true ones
        keys = list(zip(D[i].tolist(), F[i].tolist()))
        assert keys == sorted(keys)
        assert len(set(F[i].tolist())) == F.shape[1]
        for j in (0, 5, 23):
            assert D[i, j] == oracle.l2sq(q[i], x[F[i, j]])
    assert a["hops"] >= 24 * len(q)  # every final entry was expanded
    # per-query recall improves with L and reaches brute force for large L
    gt, _ = oracle.bruteforce(x, q, 10)
    r_small = oracle.recall_at_k(ix.search(q, 10, 10)["ids"], gt)
    r_big = oracle.recall_at_k(ix.search(q, 10, 200)["ids"], gt)
    assert r_big >= r_small and r_big >= 0.98


def test_recall_definition():
    t = np.array([[1, 2, 3, 4]], np.uint32)
    f = np.array([[4, 9, 1, 7]], np.uint32)
    assert oracle.recall_at_k(f, t) == 0.5


def test_mips_augment_is_inner_product_search():
    """Sec. 6.3: with one extra coordinate the L2 order of the augmented vectors is the inner-product order of the
    originals, and the distance has the closed form M^2 + |q|^2 - 2 <x, q>."""
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((400, 20)) * rng.uniform(0.2, 3.0, (400, 1))).astype(np.float32)
    q = rng.standard_normal((30, 20)).astype(np.float32)
    M = float(np.linalg.norm(x.astype(np.float64), axis=1).max())
    xa = oracle.mips_augment(x, M, dim_out=24)
    qa = oracle.mips_augment(q, M, is_query=True, dim_out=24)
    assert xa.shape == (400, 24) and (xa[:, 21:] == 0).all() and (qa[:, 20:] == 0).all()
    assert np.array_equal(xa[:, :20], x) and xa[:, 20].min() >= 0 and np.isclose(xa[:, 20].min(), 0, atol=2e-3)
    ip = x.astype(np.float64) @ q.astype(np.float64).T
    ids, dist = oracle.bruteforce(xa, qa, 10)
    want = np.argsort(-ip, axis=0, kind="stable")[:10].T
    assert np.array_equal(ids, want)
    closed = M * M + (q.astype(np.float64) ** 2).sum(axis=1)[:, None] - 2 * np.take_along_axis(ip.T, want, axis=1)
    assert np.allclose(dist, closed, rtol=1e-5)
