"""GPU parity for binary16 storage of float data (the format of the paper's
main evaluation, App. D): beamSearch, brute force, batch insertion, RaBitQ on
top of it.  The oracle converts halves exactly and accumulates in double."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_07048_amd import datagen
from gpu_common import dev, u32, random_data, oracle_index, gpu_index_from_oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def jx():
    from paper_2601_07048_amd import jx as m
    return m


def _half(n, d, seed):
    return random_data(n, d, np.float32, seed).astype(np.float16)


@pytest.mark.parametrize("d", [8, 64, 96, 128, 960, 1536])
def test_beam_f16(jx, d):
    n = 1500
    x = _half(n, d, d)
    q = _half(40, d, d + 1)
    ix = oracle_index(x, 20, 40)
    g = gpu_index_from_oracle(jx, x, ix, 20, 40)
    for L in (10, 70):
        ref = ix.search(q, 1, L, want_frontier=True)
        ids, dist = g.beam_frontier(dev(q), L)
        ids, dist = u32(ids), dist.cpu().numpy().astype(np.float64)
        fin = np.isfinite(ref["F_dist"])
        assert np.allclose(dist[fin], ref["F_dist"][fin], rtol=1e-4, atol=1e-5)
        assert (ids == ref["F_ids"]).mean() > 0.97


def test_f16_dyadic_grid_bit_exact_search_and_build(jx):
    """Multiples of 1/8 in [-4, 4] are exact in binary16 and every partial sum
    of the norm form is exact in float32: search and build must match the
    oracle bit for bit."""
    x = datagen.dyadic_grid(3000, 64, seed=21).astype(np.float16)
    q = datagen.dyadic_grid(80, 64, seed=22).astype(np.float16)
    ref = oracle.Index(64, np.float16, 24, 48, 1.2, 3000)
    g = jx.Index(64, jx.F16, 24, 48, 1.2, capacity=3000, max_batch=3000)
    for a, b in ((0, 1200), (1200, 3000)):
        ref.insert(x[a:b])
        g.insert(dev(x[a:b]))
    oadj, _ = ref.graph()
    adj, _ = g.export_graph()
    assert g.size() == (3000, ref.entry)
    assert np.array_equal(u32(adj), oadj)
    want = ref.search(q, 10, 64, want_frontier=True)
    ids, dist = g.beam_frontier(dev(q), 64)
    assert np.array_equal(u32(ids), want["F_ids"])
    assert np.array_equal(dist.cpu().numpy().astype(np.float64), want["F_dist"])


def test_bruteforce_f16(jx):
    n, d = 4000, 96
    x = _half(n, d, 3)
    q = _half(70, d, 4)
    g = jx.Index(d, jx.F16, 8, 8, 1.2, capacity=n)
    g.import_graph(dev(x), dev(np.full((n, 8), jx.NONE, np.uint32)), 0)
    ids, dist = g.bruteforce(dev(q), 10)
    rid, rd = oracle.bruteforce(x, q, 10)
    assert np.allclose(dist.cpu().numpy().astype(np.float64), rd, rtol=1e-4, atol=1e-5)
    assert (u32(ids) == rid).mean() > 0.99


def test_insert_f16_quality(jx):
    n = 6000
    x = datagen.base(1, n).astype(np.float16)
    q = datagen.queries(1, 1000).astype(np.float16)
    ref = oracle.Index(128, np.float16, 32, 64, 1.2, n)
    ref.insert(x)
    g = jx.Index(128, jx.F16, 32, 64, 1.2, capacity=n, max_batch=n)
    g.insert(dev(x))
    oadj, odeg = ref.graph()
    adj, deg = g.export_graph()
    adj, deg = u32(adj), u32(deg)
    assert g.size() == (n, ref.entry)
    for i in range(0, n, 37):
        row = adj[i, :deg[i]]
        assert (adj[i, deg[i]:] == 0xFFFFFFFF).all() and (row < n).all() and i not in row
        assert len(set(row.tolist())) == len(row)
    assert (adj == oadj).all(axis=1).mean() > 0.9
    gt, _ = oracle.bruteforce(x, q, 10)
    ids, _ = g.search(dev(q), 10, 64)
    r_gpu = oracle.recall_at_k(u32(ids), gt)
    r_ref = oracle.recall_at_k(ref.search(q, 10, 64)["ids"], gt)
    assert r_gpu >= 0.95 and abs(r_gpu - r_ref) <= 0.002, (r_gpu, r_ref)


def test_rabitq_on_f16_data(jx):
    """4-bit codes and exact re-rank on a binary16 store."""
    n, d = 3000, 960
    x = datagen.base(3, n).astype(np.float16)
    q = datagen.queries(3, 2000).astype(np.float16)
    P = datagen.rotation(3)
    ix = oracle_index(x, 32, 64)
    ix.quantize(4, P, qbits=8, rule=oracle.RULE_MAXCOS)
    g = gpu_index_from_oracle(jx, x, ix, 32, 64, quant_bits=4)
    g.quantize(4, dev(P), None, query_bits=8, rule=jx.RULE_MAXCOS)
    wc, wm, wcen = ix.codes()
    gc, gm, gcen = [t.cpu().numpy() for t in g.export_codes()]
    assert np.allclose(gcen, wcen, atol=1e-6)
    assert (gc == wc).all(axis=1).mean() > 0.9
    gt, _ = oracle.bruteforce(x, q, 10)
    want = ix.search(q, 10, 64, mode=1, rerank=40)
    ids, dist = g.search(dev(q), 10, 64, mode=jx.RABITQ, rerank=40)
    ids, dist = u32(ids), dist.cpu().numpy().astype(np.float64)
    assert abs(oracle.recall_at_k(ids, gt) - oracle.recall_at_k(want["ids"], gt)) <= 0.002
    for i in range(0, len(q), 170):
        for j in range(10):
            assert abs(dist[i, j] - oracle.l2sq(q[i], x[ids[i, j]])) <= 1e-4 * dist[i, j] + 1e-6


def test_f16_argument_errors(jx):
    with pytest.raises(jx.JxError):
        jx.Index(12, jx.F16, 8, 8, 1.2, capacity=16)  # dim must be a multiple of 8
