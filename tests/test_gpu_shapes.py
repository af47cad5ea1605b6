"""GPU parity on the further workload shapes the paper evaluates (Sec. 6.1: k in {1, 50, 100}; 96-dimensional
unit-norm descriptors; inner-product data searched through the one-extra-dimension transform of Sec. 6.3)."""
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


@pytest.mark.parametrize("k,L", [(1, 1), (1, 32), (50, 50), (50, 128), (100, 100), (100, 256)])
def test_search_k_values_u8_bit_exact(jx, k, L):
    x = random_data(6000, 128, np.uint8, seed=k + L)
    q = random_data(150, 128, np.uint8, seed=k + L + 1)
    ix = oracle_index(x, 32, 64)
    g = gpu_index_from_oracle(jx, x, ix, 32, 64)
    want = ix.search(q, k, L)
    ids, dist = g.search(dev(q), k, L)
    assert np.array_equal(u32(ids), want["ids"])
    assert np.array_equal(dist.cpu().numpy().astype(np.float64), want["dist"])


@pytest.mark.parametrize("k", [1, 50, 100])
def test_search_k_values_rabitq_rerank(jx, k):
    """Estimated-distance search with re-rank of max(k, 40): recall@k within 0.002 of the oracle's (2,000 queries)."""
    n, d, L = 4000, 128, 128
    x = random_data(n, d, np.float32, seed=70 + k)
    q = random_data(2000, d, np.float32, seed=71 + k)
    ref = oracle_index(x, 32, 64)
    g = gpu_index_from_oracle(jx, x, ref, 32, 64, quant_bits=4)
    P = datagen.random_orthogonal(d, seed=9).astype(np.float32)
    g.quantize(4, dev(P))
    ref.quantize(4, P)
    rr = max(k, 40)
    ids, _ = g.search(dev(q), k, L, mode=jx.RABITQ, rerank=rr)
    want = ref.search(q, k, L, mode=1, rerank=rr)["ids"]
    gt = oracle.bruteforce(x, q, k)[0]
    r_g, r_o = oracle.recall_at_k(u32(ids), gt), oracle.recall_at_k(want, gt)
    assert abs(r_g - r_o) <= 0.002 and r_g > 0.6, (r_g, r_o)
    assert (u32(ids) == want).all(axis=1).mean() > 0.9


def test_deep_like_96d_build_and_search(jx):
    """Workload 6 (96-d float32, unit norm): GPU build and search against the oracle's, through recall."""
    n = 20000
    x = datagen.base(6, n)
    q = datagen.queries(6, 2000)
    ref = oracle.Index(96, np.float32, 32, 64, 1.2, n)
    ref.insert(x)
    g = jx.Index(96, jx.F32, 32, 64, 1.2, capacity=n, max_batch=n)
    g.insert(dev(x))
    assert g.size() == (n, ref.entry)
    gt = oracle.bruteforce(x, q, 10)[0]
    for L in (32, 64):
        r_o = oracle.recall_at_k(ref.search(q, 10, L)["ids"], gt)
        r_g = oracle.recall_at_k(u32(g.search(dev(q), 10, L)[0]), gt)
        assert abs(r_o - r_g) <= 0.002, (L, r_o, r_g)
    assert r_g >= 0.95
    # same graph on both sides: ids agree except where float32 rounding reorders near-ties
    adj, _ = ref.graph()
    g2 = gpu_index_from_oracle(jx, x, ref, 32, 64)
    ids = u32(g2.search(dev(q), 10, 64)[0])
    assert (ids == ref.search(q, 10, 64)["ids"]).all(axis=1).mean() > 0.97


def test_mips_augment_parity_and_search(jx):
    """Workload 7 (200-d, varying norms, inner-product search): the transform against the oracle's definition,
    then build + search on the augmented vectors; the ground truth is the plain inner product."""
    n, d, dout = 20000, 200, 204
    x = datagen.base(7, n)
    q = datagen.queries(7, 2000)
    norms = jx.mips_augment(dev(x), want_norms=True).cpu().numpy()
    want_norms = np.linalg.norm(x.astype(np.float64), axis=1)
    assert np.allclose(norms, want_norms, rtol=1e-6)
    M = float(want_norms.max()) * (1 + 1e-6)
    xa = jx.mips_augment(dev(x), M, dim_out=dout)
    qa = jx.mips_augment(dev(q), M, is_query=True, dim_out=dout)
    oxa, oqa = oracle.mips_augment(x, M, dim_out=dout), oracle.mips_augment(q, M, is_query=True, dim_out=dout)
    assert np.array_equal(qa.cpu().numpy(), oqa)
    got = xa.cpu().numpy()
    assert np.array_equal(got[:, :d], oxa[:, :d]) and (got[:, d + 1:] == 0).all()
    assert np.allclose(got[:, d], oxa[:, d], rtol=1e-5, atol=1e-4 * M)
    # inner-product ground truth, independent of the transform
    gt = np.argsort(-(q.astype(np.float64) @ x.astype(np.float64).T), axis=1, kind="stable")[:, :10].astype(np.uint32)
    g = jx.Index(dout, jx.F32, 32, 64, 1.2, capacity=n, max_batch=n)
    g.insert(xa)
    bf, _ = g.bruteforce(qa, 10)
    assert oracle.recall_at_k(u32(bf), gt) > 0.999
    ref = oracle.Index(dout, np.float32, 32, 64, 1.2, n)
    ref.insert(oxa)
    r_o = oracle.recall_at_k(ref.search(oqa, 10, 64)["ids"], gt)
    r_g = oracle.recall_at_k(u32(g.search(qa, 10, 64)[0]), gt)
    assert abs(r_o - r_g) <= 0.002 and r_g > 0.8, (r_o, r_g)
