"""GPU parity: batch deletion (mark, consolidate; Sec. 4.6) through the C ABI vs
the CPU oracle.  On integer data the consolidated graph, the entry point and
every search result must equal the oracle's bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from gpu_common import dev, u32, random_data

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def jx():
    from paper_2601_07048_amd import jx as m
    return m


def _pair(jx, x, R, L, max_batch=None, alpha=1.2):
    """The same graph (the oracle's) on both sides."""
    n, d = x.shape
    dt = {np.dtype(np.uint8): jx.U8, np.dtype(np.float32): jx.F32, np.dtype(np.float16): jx.F16}[x.dtype]
    ref = oracle.Index(d, x.dtype, R, L, alpha, 2 * n)
    ref.insert(x)
    adj, _ = ref.graph()
    g = jx.Index(d, dt, R, L, alpha, capacity=2 * n, max_batch=max_batch or n)
    g.import_graph(dev(x), dev(adj), ref.entry)
    return ref, g


def _same_graph(ref, g):
    oadj, odeg = ref.graph()
    adj, deg = g.export_graph()
    adj, deg = u32(adj), u32(deg)
    assert np.array_equal(deg, odeg)
    bad = np.nonzero((adj != oadj).any(axis=1))[0]
    assert bad.size == 0, (bad[:5], adj[bad[:1]], oadj[bad[:1]])


def _same_search(ref, g, q, k, L):
    r = ref.search(q, k, L)
    oi, od = r["ids"], r["dist"]
    gi, gd = g.search(dev(q), k, L)
    assert np.array_equal(u32(gi), oi)
    fin = np.isfinite(od)
    assert np.array_equal(gd.cpu().numpy()[fin], od[fin].astype(np.float32))
    assert np.isinf(gd.cpu().numpy()[~fin]).all()
    return oi


@pytest.mark.parametrize("n,d,R,L,frac", [
    (600, 32, 8, 16, 0.1),
    (3000, 128, 32, 64, 0.05),
    (3000, 128, 32, 64, 0.5),        # many deleted neighbours per row: candidate sets far beyond 128
    (2500, 128, 70, 130, 0.2),       # R > 64
])
def test_mark_then_search_excludes_deleted(jx, n, d, R, L, frac):
    x = random_data(n, d, np.uint8, seed=7 * n + R)
    q = random_data(200, d, np.uint8, seed=n + 1)
    ref, g = _pair(jx, x, R, L)
    rng = np.random.default_rng(n)
    dele = rng.choice(n, int(frac * n), replace=False).astype(np.uint32)
    ref.delete(dele)
    g.delete(dev(dele))
    assert g.deleted_count() == ref.n_deleted == dele.size
    # repeated and unknown ids change nothing
    g.delete(dev(np.concatenate([dele[:10], np.array([n, n + 5, 2**31 - 2], np.uint32)])))
    assert g.deleted_count() == dele.size
    oi = _same_search(ref, g, q, 10, L)
    assert not np.isin(oi[oi != 0xFFFFFFFF], dele).any()
    # whole frontier
    fi, _ = g.beam_frontier(dev(q), L)
    fi = u32(fi)
    assert not np.isin(fi[fi != 0xFFFFFFFF], dele).any()
    # filtered entries are compacted to the left: no gap before the padding
    pad = fi == 0xFFFFFFFF
    assert (np.diff(pad.astype(np.int8), axis=1) >= 0).all()


@pytest.mark.parametrize("n,d,R,L,frac,max_batch", [
    (600, 32, 8, 16, 0.1, None),
    (3000, 128, 32, 64, 0.05, None),
    (3000, 128, 32, 64, 0.3, None),
    (3000, 128, 32, 64, 0.3, 64),     # small edge buffer: many vertex slices
    (3000, 128, 32, 64, 0.6, None),
    (2500, 128, 70, 130, 0.2, None),  # R > 64
    (4000, 64, 16, 40, 0.2, None),
])
def test_consolidate_u8_graph_bit_exact(jx, n, d, R, L, frac, max_batch):
    x = random_data(n, d, np.uint8, seed=3 * n + R)
    q = random_data(200, d, np.uint8, seed=n + 2)
    ref, g = _pair(jx, x, R, L, max_batch=max_batch)
    rng = np.random.default_rng(n + 1)
    dele = rng.choice(n, int(frac * n), replace=False).astype(np.uint32)
    dele[0] = ref.entry  # the entry point goes too
    dele = np.unique(dele)
    ref.delete(dele)
    g.delete(dev(dele))
    ref.consolidate()
    g.consolidate()
    assert g.size() == (n, ref.entry)
    assert ref.entry not in set(dele.tolist())
    _same_graph(ref, g)
    _same_search(ref, g, q, 10, L)
    # a second consolidation finds nothing to do
    g.consolidate()
    _same_graph(ref, g)


def test_delete_insert_interleaved_u8(jx):
    """Delete, consolidate, insert more, delete again without consolidating, insert, search."""
    n, d, R, L = 4000, 64, 24, 48
    x = random_data(n, d, np.uint8, seed=99)
    q = random_data(100, d, np.uint8, seed=98)
    ref = oracle.Index(d, x.dtype, R, L, 1.2, n)
    g = jx.Index(d, jx.U8, R, L, 1.2, capacity=n, max_batch=n)
    ref.insert(x[:2000])
    g.insert(dev(x[:2000]))
    rng = np.random.default_rng(5)
    d1 = rng.choice(2000, 300, replace=False).astype(np.uint32)
    ref.delete(d1)
    g.delete(dev(d1))
    ref.consolidate()
    g.consolidate()
    _same_graph(ref, g)
    ref.insert(x[2000:3000])
    g.insert(dev(x[2000:3000]))
    _same_graph(ref, g)
    d2 = rng.choice(3000, 400, replace=False).astype(np.uint32)
    ref.delete(d2)
    g.delete(dev(d2))
    # insertion candidates skip marked vertices even before consolidation
    ref.insert(x[3000:])
    g.insert(dev(x[3000:]))
    _same_graph(ref, g)
    adj, _ = g.export_graph()
    adj = u32(adj)
    assert not np.isin(adj[3000:], np.union1d(d1, d2)).any()
    _same_search(ref, g, q, 10, L)
    ref.consolidate()
    g.consolidate()
    assert g.size() == (n, ref.entry)
    _same_graph(ref, g)
    _same_search(ref, g, q, 10, L)
    assert g.deleted_count() == ref.n_deleted


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_consolidate_float_dyadic_bit_exact(jx, dtype):
    """Float data on a dyadic grid: every distance is exact in float32 whatever
    the summation order, so the float paths must reproduce the oracle too."""
    from paper_2601_07048_amd import datagen
    n, d, R, L = 2500, 64, 24, 48
    x = datagen.dyadic_grid(n, d, seed=11).astype(dtype)
    q = datagen.dyadic_grid(100, d, seed=12).astype(dtype)
    ref, g = _pair(jx, x, R, L)
    rng = np.random.default_rng(3)
    dele = rng.choice(n, 500, replace=False).astype(np.uint32)
    ref.delete(dele)
    g.delete(dev(dele))
    ref.consolidate()
    g.consolidate()
    assert g.size() == (n, ref.entry)
    _same_graph(ref, g)
    _same_search(ref, g, q, 10, L)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_consolidate_float_large_candidate_sets_bit_exact(jx, dtype):
    """Half of the vertices deleted with R = 40: candidate sets of several hundred, beyond the 256 rows of the
    matrix-core prune, which then works on the closest prefix (exact whenever R neighbours are found inside it)
    or hands the vertex to the list-based kernel.  Dyadic grid: the result must equal the oracle's bit for bit."""
    from paper_2601_07048_amd import datagen
    n, d, R, L = 3000, 64, 40, 80
    x = datagen.dyadic_grid(n, d, seed=21).astype(dtype)
    ref, g = _pair(jx, x, R, L)
    rng = np.random.default_rng(9)
    dele = rng.choice(n, n // 2, replace=False).astype(np.uint32)
    ref.delete(dele)
    g.delete(dev(dele))
    adj0, deg0 = ref.graph()
    dead = np.zeros(n, bool)
    dead[dele] = True
    sizes = [sum(int((~dead[adj0[u, :deg0[u]]]).sum()) if dead[u] else 1 for u in adj0[v, :deg0[v]]) for v in range(0, n, 50)
             if not dead[v]]
    assert max(sizes) > 300  # the case this test is about
    ref.consolidate()
    g.consolidate()
    assert g.size() == (n, ref.entry)
    _same_graph(ref, g)


def test_consolidate_float_quality(jx):
    """Generic float data: rounding differs, so compare what must hold: no edge
    to or from a deleted vertex, rows nearly equal, recall against brute force
    on the live set as good as the oracle's."""
    n, d, R, L = 4000, 96, 32, 64
    x = random_data(n, d, np.float32, seed=21)
    q = random_data(300, d, np.float32, seed=22)
    ref, g = _pair(jx, x, R, L)
    rng = np.random.default_rng(4)
    dele = rng.choice(n, 800, replace=False).astype(np.uint32)
    ref.delete(dele)
    g.delete(dev(dele))
    ref.consolidate()
    g.consolidate()
    oadj, _ = ref.graph()
    adj, _ = g.export_graph()
    adj = u32(adj)
    assert (adj[dele] == 0xFFFFFFFF).all()
    assert not np.isin(adj[adj != 0xFFFFFFFF], dele).any()
    assert (adj != oadj).any(axis=1).mean() < 0.01
    live = np.setdiff1d(np.arange(n), dele)
    gt = oracle.bruteforce(x[live], q, 10)[0]
    gt = live[gt]
    oi = ref.search(q, 10, L)["ids"]
    gi, _ = g.search(dev(q), 10, L)
    r_o = oracle.recall_at_k(oi, gt)
    r_g = oracle.recall_at_k(u32(gi), gt)
    assert abs(r_o - r_g) <= 0.002 and r_g > 0.75


def test_rabitq_search_skips_deleted(jx):
    from paper_2601_07048_amd import datagen
    n, d, R, L = 3000, 128, 32, 64
    x = random_data(n, d, np.float32, seed=31)
    q = random_data(2000, d, np.float32, seed=32)
    ref = oracle.Index(d, x.dtype, R, L, 1.2, n)
    ref.insert(x)
    adj, _ = ref.graph()
    g = jx.Index(d, jx.F32, R, L, 1.2, capacity=n, max_batch=n, quant_bits=4)
    g.import_graph(dev(x), dev(adj), ref.entry)
    P = datagen.random_orthogonal(d, seed=5)
    g.quantize(4, dev(P.astype(np.float32)))
    dele = np.random.default_rng(6).choice(n, 900, replace=False).astype(np.uint32)
    g.delete(dev(dele))
    ids, dist = g.search(dev(q), 10, L, mode=jx.RABITQ, rerank=L)
    ids = u32(ids)
    assert not np.isin(ids[ids != 0xFFFFFFFF], dele).any()
    live = np.setdiff1d(np.arange(n), dele)
    gt = live[oracle.bruteforce(x[live], q, 10)[0]]
    ref.quantize(4, P.astype(np.float32))
    ref.delete(dele)
    oi = ref.search(q, 10, L, mode=1, rerank=L)["ids"]
    r_g, r_o = oracle.recall_at_k(ids, gt), oracle.recall_at_k(oi, gt)
    assert abs(r_g - r_o) <= 0.002 and r_g > 0.7, (r_g, r_o)
    assert (ids == oi).all(axis=1).mean() > 0.95


def test_delete_everything(jx):
    n, d = 64, 16
    x = random_data(n, d, np.uint8, seed=41)
    ref, g = _pair(jx, x, 4, 8)
    every = np.arange(n, dtype=np.uint32)
    g.delete(dev(every))
    ids, _ = g.search(dev(x[:4]), 3, 8)
    assert (u32(ids) == 0xFFFFFFFF).all()
    g.consolidate()
    assert g.size() == (n, jx.NONE)
    adj, deg = g.export_graph()
    assert (u32(deg) == 0).all()
    with pytest.raises(jx.JxError):
        g.search(dev(x[:4]), 3, 8)
    with pytest.raises(jx.JxError):
        g.insert(dev(x[:4]))


def test_consolidate_capacity_error(jx):
    """A vertex whose candidate list exceeds the edge buffer is reported, not truncated."""
    n, d, R = 600, 32, 16
    x = random_data(n, d, np.uint8, seed=51)
    ref, g = _pair(jx, x, R, 32, max_batch=1)
    dele = np.random.default_rng(7).choice(n, 300, replace=False).astype(np.uint32)
    g.delete(dev(dele))
    with pytest.raises(jx.JxError) as e:
        g.consolidate()
    assert e.value.code == -2 and "candidates" in str(e.value)
    # nothing was changed
    adj, _ = g.export_graph()
    assert np.array_equal(u32(adj), ref.graph()[0])


@pytest.mark.parametrize("n,d,R,L,frac,quant", [
    (600, 32, 8, 16, 0.1, 0),
    (3000, 128, 32, 64, 0.3, 0),
    (2500, 128, 70, 130, 0.2, 0),
    (3000, 64, 13, 32, 0.25, 0),      # row of 52 bytes: moved in 4-byte units
])
def test_compact_u8_bit_exact(jx, n, d, R, L, frac, quant):
    x = random_data(n, d, np.uint8, seed=5 * n + R)
    q = random_data(200, d, np.uint8, seed=n + 3)
    ref, g = _pair(jx, x, R, L)
    rng = np.random.default_rng(n + 2)
    dele = np.unique(np.concatenate([rng.choice(n, int(frac * n), replace=False), [ref.entry]])).astype(np.uint32)
    ref.delete(dele)
    g.delete(dev(dele))
    with pytest.raises(jx.JxError) as e:
        g.compact()
    assert e.value.code == -3
    ref.consolidate()
    g.consolidate()
    before = u32(g.search(dev(q), 10, L)[0])
    want_map = ref.compact()
    got_map = u32(g.compact())
    assert np.array_equal(got_map, want_map)
    assert g.size() == (ref.n, ref.entry) and g.deleted_count() == 0
    _same_graph(ref, g)
    oi = _same_search(ref, g, q, 10, L)
    assert np.array_equal(oi, want_map[before])      # a renaming, nothing else
    bi, bd = g.bruteforce(dev(q[:20]), 5)             # the vectors moved with their ids
    oi2, od2 = oracle.bruteforce(x[np.setdiff1d(np.arange(n), dele)], q[:20], 5)
    assert np.array_equal(u32(bi), oi2)
    # the freed tail takes new points
    extra = random_data(400, d, np.uint8, seed=n + 9)
    ref.insert(extra)
    g.insert(dev(extra))
    _same_graph(ref, g)
    _same_search(ref, g, q, 10, L)


def test_compact_without_deletions_is_identity(jx):
    x = random_data(1000, 32, np.uint8, seed=77)
    ref, g = _pair(jx, x, 8, 16)
    m = u32(g.compact())
    assert np.array_equal(m, np.arange(1000))
    _same_graph(ref, g)


def test_compact_rabitq_records_move(jx):
    """Quantised float index: after delete / consolidate / compact the estimated-distance search with re-rank
    returns the renamed ids of what it returned before, with identical distances."""
    from paper_2601_07048_amd import datagen
    n, d, R, L = 3000, 128, 32, 64
    x = random_data(n, d, np.float32, seed=61)
    q = random_data(150, d, np.float32, seed=62)
    g = jx.Index(d, jx.F32, R, L, 1.2, capacity=n, max_batch=n, quant_bits=4)
    g.insert(dev(x))
    g.quantize(4, dev(datagen.random_orthogonal(d, seed=7).astype(np.float32)))
    dele = np.random.default_rng(8).choice(n, 600, replace=False).astype(np.uint32)
    g.delete(dev(dele))
    g.consolidate()
    b_ex = g.search(dev(q), 10, L)
    b_rq = g.search(dev(q), 10, L, mode=jx.RABITQ)
    b_rr = g.search(dev(q), 10, L, mode=jx.RABITQ, rerank=40)
    m = u32(g.compact())
    assert g.size()[0] == n - 600
    for (bi, bd), kw in ((b_ex, {}), (b_rq, dict(mode=jx.RABITQ)), (b_rr, dict(mode=jx.RABITQ, rerank=40))):
        ai, ad = g.search(dev(q), 10, L, **kw)
        assert np.array_equal(u32(ai), m[u32(bi)])
        assert np.array_equal(ad.cpu().numpy(), bd.cpu().numpy())
    codes, meta, _ = g.export_codes()
    assert codes.shape[0] == n - 600
