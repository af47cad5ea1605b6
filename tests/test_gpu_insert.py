"""GPU parity: batch insertion (beamSearch candidates, robustPrune, reverse-edge
merge) through the C ABI vs the CPU oracle.  Integer data must give the same
adjacency bit for bit, rows in the same order."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_07048_amd import datagen
from gpu_common import dev, u32, random_data

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def jx():
    from paper_2601_07048_amd import jx as m
    return m


def _build_both(jx, x, R, L, calls=None, alpha=1.2, growth=0.25, cand_mode=0):
    n, d = x.shape
    dt = jx.U8 if x.dtype == np.uint8 else jx.F32
    calls = calls or [n]
    ref = oracle.Index(d, x.dtype, R, L, alpha, n, batch_growth=growth, cand_mode=cand_mode)
    g = jx.Index(d, dt, R, L, alpha, capacity=n, max_batch=n, batch_growth=growth, cand_mode=cand_mode)
    pos = 0
    for c in calls:
        ref.insert(x[pos:pos + c])
        g.insert(dev(x[pos:pos + c]))
        pos += c
    torch.cuda.synchronize()
    return ref, g


def _graphs(ref, g):
    oadj, odeg = ref.graph()
    adj, deg = g.export_graph()
    return oadj, odeg, u32(adj), u32(deg)


@pytest.mark.parametrize("n,d,R,L,calls,growth", [
    (5, 16, 2, 4, None, 1.0),
    (700, 32, 8, 16, None, 0.25),
    (3000, 128, 32, 64, None, 0.25),
    (3000, 128, 32, 64, None, 1.0),
    (3000, 128, 32, 64, [1, 1, 2, 996, 2000], 0.5),
    (4000, 64, 16, 100, [1500, 2500], 0.25),
    (2500, 128, 70, 130, None, 0.3),      # R > 64: rows span two lane blocks
    (6000, 128, 20, 40, None, 0.25),      # small merges: one or two 32-slot tiles of the Gram-matrix path
    (6000, 128, 90, 128, None, 0.25),     # merges beyond 96 candidates: the global-memory path
    (5000, 128, 64, 64, [2500, 2500], 0.25),
    # 128-byte vectors take the lean prune and merge kernels: degenerate degrees and frontiers
    (600, 128, 1, 1, None, 0.25),
    (600, 128, 1, 4, [1, 599], 1.0),
    (800, 128, 2, 3, None, 0.25),
    (800, 128, 3, 8, None, 0.5),
    (1500, 128, 5, 128, None, 0.25),      # far more candidates than room: every round ends on the R cap
    (1200, 128, 127, 128, None, 0.25),    # rows of 127 + new edges: the 128-slot limit of the lean merge
    (1200, 128, 200, 128, None, 0.25),    # R above the frontier width: rows never fill from the forward prune
    (3000, 128, 12, 128, [100] * 30, 1.0),  # many small calls: appended tails between prunes
])
def test_insert_u8_graph_bit_exact(jx, n, d, R, L, calls, growth):
    x = random_data(n, d, np.uint8, seed=n + R)
    ref, g = _build_both(jx, x, R, L, calls, growth=growth)
    oadj, odeg, adj, deg = _graphs(ref, g)
    assert g.size() == (n, ref.entry)
    assert np.array_equal(deg, odeg)
    bad = np.nonzero((adj != oadj).any(axis=1))[0]
    assert bad.size == 0, f"{bad.size} rows differ, first {bad[:5]}"


def test_insert_u8_workload2_20k(jx):
    """Workload-2 generator and parameters (R=64, L_build=128, alpha=1.2) at
    N = 20,000, inserted in two calls."""
    n = 20000
    x = datagen.base(2, n)
    ref, g = _build_both(jx, x, 64, 128, [12000, 8000])
    oadj, odeg, adj, deg = _graphs(ref, g)
    assert g.size() == (n, ref.entry)
    assert np.array_equal(adj, oadj)
    q = datagen.queries(2, 500)
    ids, dist = g.search(dev(q), 10, 64)
    want = ref.search(q, 10, 64)
    assert np.array_equal(u32(ids), want["ids"])
    gt, _ = g.bruteforce(dev(q), 10)
    assert oracle.recall_at_k(u32(ids), u32(gt)) > 0.95


def test_insert_duplicate_points_and_hub(jx):
    """Many identical vectors: zero distances, ties broken by id, one hub that
    receives far more reverse edges than R."""
    rng = np.random.default_rng(3)
    x = rng.integers(0, 256, (1200, 16), dtype=np.uint8)
    x[200:700] = x[7]
    ref, g = _build_both(jx, x, 6, 24)
    oadj, odeg, adj, deg = _graphs(ref, g)
    assert np.array_equal(adj, oadj)


def test_insert_f32_dyadic_grid_bit_exact(jx):
    """On a dyadic grid every float32 distance is exact, so the float path must
    also reproduce the oracle's graph bit for bit."""
    x = datagen.dyadic_grid(3000, 64, seed=11)
    ref, g = _build_both(jx, x, 24, 48, [1000, 2000])
    oadj, odeg, adj, deg = _graphs(ref, g)
    assert g.size() == (3000, ref.entry)
    assert np.array_equal(adj, oadj)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("n,d,R,L,calls,growth", [
    (2500, 32, 8, 16, None, 0.25),          # prunes of 9..: one and two 32-row blocks of the Gram-matrix kernels
    (3000, 64, 40, 64, None, 0.25),         # 41.. candidates: two and three blocks
    (3000, 64, 64, 128, None, 0.5),         # frontier of 128 = four blocks; merges of 65..128 and beyond
    (2500, 40, 100, 128, None, 0.25),       # merges of 101..128 (four blocks) and > 128 (list-based kernel); ragged 160/80-byte vectors
    (2500, 64, 126, 128, None, 0.25),       # binary16: 127 candidates + the pruned vertex fill the 128 rows exactly
    (2500, 64, 127, 128, None, 0.25),       # binary16: one too many for the extra row -> list-based kernel
    (2000, 64, 24, 160, [800, 1200], 0.25), # frontier wider than 128: forward prune stays with the list-based kernel
    (6000, 32, 12, 24, [10, 5990], 1.0),    # doubling batches, small R: hubs collect hundreds of new edges (prefix pools)
])
def test_insert_float_dyadic_grid_gram_classes(jx, dtype, n, d, R, L, calls, growth):
    """Float builds on a dyadic grid (every distance exact in float32 in any summation order) must equal the
    oracle's graph bit for bit; the cases walk through every size class of the matrix-core robustPrune and
    its hand-over to the list-based kernel."""
    x = datagen.dyadic_grid(n, d, seed=n + R).astype(dtype)
    dt = jx.F32 if dtype == np.float32 else jx.F16
    ref = oracle.Index(d, x.dtype, R, L, 1.2, n, batch_growth=growth)
    g = jx.Index(d, dt, R, L, 1.2, capacity=n, max_batch=n, batch_growth=growth)
    pos = 0
    for c in calls or [n]:
        ref.insert(x[pos:pos + c])
        g.insert(dev(x[pos:pos + c]))
        pos += c
    oadj, odeg, adj, deg = _graphs(ref, g)
    assert g.size() == (n, ref.entry)
    assert np.array_equal(deg, odeg)
    bad = np.nonzero((adj != oadj).any(axis=1))[0]
    assert bad.size == 0, (bad[:5], adj[bad[:1]], oadj[bad[:1]])


def _invariants(adj, deg, n, R):
    for i in range(n):
        row = adj[i, :deg[i]]
        assert (adj[i, deg[i]:] == 0xFFFFFFFF).all()
        assert (row < n).all() and i not in row and len(set(row.tolist())) == len(row)


def test_insert_f32_workload1(jx):
    """Workload 1 (float32, N=10,000, R=32, L_build=64, seeded random order):
    float distances differ from the oracle's double in the last bits, so the
    graph is compared through its invariants and through recall, which must be
    within 0.002 of the oracle-built graph's and at least 0.95 at L=64."""
    n = 10000
    x = datagen.base(1, n)[datagen.insertion_order(1, n)]
    q = datagen.queries(1, 1000)
    ref, g = _build_both(jx, x, 32, 64)
    oadj, odeg, adj, deg = _graphs(ref, g)
    _invariants(adj, deg, n, 32)
    assert g.size() == (n, ref.entry)
    assert (adj == oadj).all(axis=1).mean() > 0.95  # most rows are identical
    gt, _ = oracle.bruteforce(x, q, 10)
    ids, dist = g.search(dev(q), 10, 64)
    r_gpu = oracle.recall_at_k(u32(ids), gt)
    r_ref = oracle.recall_at_k(ref.search(q, 10, 64)["ids"], gt)
    assert r_gpu >= 0.95 and abs(r_gpu - r_ref) <= 0.002, (r_gpu, r_ref)


def test_insert_errors(jx):
    x = random_data(100, 16, np.uint8, seed=1)
    g = jx.Index(16, jx.U8, 4, 8, 1.2, capacity=64, max_batch=64)
    with pytest.raises(jx.JxError) as e:
        g.insert(dev(x))
    assert e.value.code == -2  # capacity
    g2 = jx.Index(16, jx.U8, 4, 8, 1.2, capacity=100, max_batch=4, batch_growth=1.0)
    with pytest.raises(jx.JxError) as e:
        g2.insert(dev(x))      # an internal batch would exceed max_batch
    assert e.value.code == -2
    g2.insert(dev(x[:9]))      # batches of 1,1,2,4 fit
    assert g2.size()[0] == 9
    g2.insert(dev(x[:0]))      # empty insert is a no-op
    assert g2.size()[0] == 9


def test_matrix_core_prune_on_uint8_variant(jx):
    """The matrix-core robustPrune also has a uint8 instantiation (int8 MFMA, exact integers).  It is slower than
    the LDS-cached form for 128-byte vectors and therefore off by default (JX_FLAG_GRAM_U8 switches it on): the
    oracle's graph bit for bit, build and consolidation."""
    for (n, d, R, L, growth) in ((3000, 128, 32, 64, 0.25), (2500, 64, 100, 128, 0.25), (5000, 32, 12, 24, 1.0)):
        x = random_data(n, d, np.uint8, seed=n + R)
        ref = oracle.Index(d, np.uint8, R, L, 1.2, n, batch_growth=growth)
        ref.insert(x)
        g = jx.Index(d, jx.U8, R, L, 1.2, capacity=n, max_batch=n, batch_growth=growth, flags=jx.FLAG_GRAM_U8)
        g.insert(dev(x))
        assert g.size() == (n, ref.entry)
        assert np.array_equal(u32(g.export_graph()[0]), ref.graph()[0]), "build"
        dele = np.random.default_rng(n).choice(n, n // 3, replace=False).astype(np.uint32)
        ref.delete(dele); g.delete(dev(dele)); ref.consolidate(); g.consolidate()
        assert np.array_equal(u32(g.export_graph()[0]), ref.graph()[0]), "consolidate"


def test_incremental_prune_of_full_rows(jx):
    """uint8 rows remember which leading entries one robustPrune call selected together; the next prune of such a
    row evaluates only the pairs that involve an appended or new entry.  Small R makes nearly every reverse edge
    overflow its row; several insert calls, the oracle's graph bit for bit after each."""
    n, d, R, L = 6000, 128, 16, 32
    x = random_data(n, d, np.uint8, seed=77)
    ref = oracle.Index(d, np.uint8, R, L, 1.2, n)
    g = jx.Index(d, jx.U8, R, L, 1.2, capacity=n, max_batch=n)
    for lo, hi in ((0, 500), (500, 2500), (2500, 2600), (2600, 6000)):
        ref.insert(x[lo:hi])
        g.insert(dev(x[lo:hi]))
        assert np.array_equal(u32(g.export_graph()[0]), ref.graph()[0]), (lo, hi)
    # deletion rewrites rows through the same kernel; inserts after it go on from the rewritten rows
    dele = np.random.default_rng(5).choice(n, 900, replace=False).astype(np.uint32)
    ref.delete(dele); g.delete(dev(dele)); ref.consolidate(); g.consolidate()
    assert np.array_equal(u32(g.export_graph()[0]), ref.graph()[0])


def test_incremental_prune_switched_off_gives_the_same_graph(jx):
    """Streaming inserts with the incremental prune switched off (JX_FLAG_NO_INCR_PRUNE) and on: both graphs equal
    the oracle's after every call at N = 40,000, and each other at N = 200,000 (where the oracle is not run)."""
    import torch
    n = 40_000
    x = datagen.base(2, n)
    ref = oracle.Index(128, np.uint8, 64, 128, 1.2, n)
    gs = [jx.Index(128, jx.U8, 64, 128, 1.2, capacity=n, max_batch=n // 4 + 1, flags=fl) for fl in (0, jx.FLAG_NO_INCR_PRUNE)]
    for lo in range(0, n, 10_000):
        ref.insert(x[lo:lo + 10_000])
        want = ref.graph()[0]
        for g in gs:
            g.insert(dev(x[lo:lo + 10_000]))
            assert np.array_equal(u32(g.export_graph()[0]), want), (lo, g.params.flags)
    del gs, ref
    n = 200_000
    dx = torch.from_numpy(datagen.base(2, n)).cuda()
    tables = []
    for fl in (0, jx.FLAG_NO_INCR_PRUNE):
        g = jx.Index(128, jx.U8, 64, 128, 1.2, capacity=n, max_batch=n // 4 + 1, flags=fl)
        for lo in range(0, n, 50_000):
            g.insert(dx[lo:lo + 50_000])
        tables.append(g.export_graph()[0])
        del g
    assert torch.equal(tables[0], tables[1])


@pytest.mark.parametrize("n,d,R,L,calls,growth", [
    (700, 32, 8, 16, None, 0.25),            # expansion list of 64
    (3000, 128, 32, 64, None, 0.25),         # 256
    (3000, 128, 32, 64, [1, 1, 2, 996, 2000], 0.5),
    (2500, 128, 64, 128, [1500, 1000], 0.25),  # 512: the benchmark's R and L_build
    (4000, 64, 16, 100, [1500, 2500], 1.0),
    (3000, 128, 12, 5, None, 0.25),          # the list is cut at 64 expansions of a narrow beam
])
def test_insert_visited_candidates_u8_graph_bit_exact(jx, n, d, R, L, calls, growth):
    """JX_CAND_VISITED: robustPrune receives the expansion list V of Alg. 1 (what Alg. 4 prunes) instead of the final
    frontier.  Whole adjacency tables against the oracle in the same mode, and they differ from the frontier mode's."""
    x = random_data(n, d, np.uint8, seed=n + R + 1)
    ref, g = _build_both(jx, x, R, L, calls, growth=growth, cand_mode=jx.CAND_VISITED)
    oadj, odeg, adj, deg = _graphs(ref, g)
    assert g.size() == (n, ref.entry)
    bad = np.nonzero((adj != oadj).any(axis=1))[0]
    assert bad.size == 0, f"{bad.size} rows differ, first {bad[:5]}"
    if n >= 2500:
        ref_f = oracle.Index(d, np.uint8, R, L, 1.2, n, batch_growth=growth)
        pos = 0
        for c in (calls or [n]):
            ref_f.insert(x[pos:pos + c])
            pos += c
        assert not np.array_equal(ref_f.graph()[0], oadj)


def test_insert_visited_candidates_with_deletions(jx):
    n = 3000
    x = random_data(n, 128, np.uint8, seed=99)
    ref = oracle.Index(128, np.uint8, 24, 48, 1.2, n, cand_mode=oracle.CAND_VISITED)
    g = jx.Index(128, jx.U8, 24, 48, 1.2, capacity=n, max_batch=n, cand_mode=jx.CAND_VISITED)
    ref.insert(x[:2000])
    g.insert(dev(x[:2000]))
    dele = np.random.default_rng(7).choice(2000, 600, replace=False).astype(np.uint32)
    ref.delete(dele)
    g.delete(dev(dele))
    ref.insert(x[2000:])
    g.insert(dev(x[2000:]))
    oadj, odeg, adj, deg = _graphs(ref, g)
    assert np.array_equal(adj, oadj)
    assert not np.isin(adj[2000:][adj[2000:] != 0xFFFFFFFF], dele).any()


def test_insert_visited_candidates_float32(jx):
    """Dyadic-grid float32 data (exact partial sums): bit parity in the expansion-list mode, at d = 64, 960 and 1536;
    lists of 256 and 512 slots go through the block-row Gram-matrix forward prune."""
    for n, d, R, L in ((3000, 64, 24, 48), (1200, 960, 16, 32), (1500, 960, 16, 48), (1200, 1536, 12, 100)):
        x = datagen.dyadic_grid(n, d, seed=13 + d, step=0.25 if d > 64 else 0.125, lim=2.0 if d > 64 else 4.0)
        ref, g = _build_both(jx, x, R, L, [n // 3, n - n // 3], cand_mode=jx.CAND_VISITED)
        oadj, odeg, adj, deg = _graphs(ref, g)
        assert g.size() == (n, ref.entry)
        assert np.array_equal(adj, oadj), d


def test_workload1_frontier_vs_visited_candidates(jx):
    """Workload 1 (N = 10,000, R = 32, L_build = 64, seeded insertion order), both candidate modes on the GPU and in
    the oracle: recall@10 at L = 64 agrees with the oracle's within 0.002 in each mode; the difference between the
    modes is printed (Alg. 4 step 2 prunes V, Alg. 2 returns F)."""
    n = 10_000
    x = datagen.base(1, n)[datagen.insertion_order(1, n)]
    q = datagen.queries(1, 1000)
    gt, _ = oracle.bruteforce(x, q, 10)
    out = {}
    for name, mode in (("frontier", 0), ("visited", 1)):
        ref, g = _build_both(jx, x, 32, 64, None, cand_mode=mode)
        for L in (32, 64):
            r_o = oracle.recall_at_k(ref.search(q, 10, L)["ids"], gt)
            r_g = oracle.recall_at_k(u32(g.search(dev(q), 10, L)[0]), gt)
            assert abs(r_o - r_g) <= 0.002, (name, L, r_o, r_g)
            out[(name, L)] = (round(r_g, 4), round(r_o, 4), round(float(u32(g.export_graph()[1]).mean()), 1))
    print("workload 1, recall@10 (GPU, oracle, mean degree):", out, flush=True)
    assert out[("visited", 64)][0] >= 0.95 and out[("frontier", 64)][0] >= 0.95
