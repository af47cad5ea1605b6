"""GPU parity at the full size of the benchmark workload (N = 1,000,000,
d = 128, uint8, R = 64, L_build = 128, 10,000 queries), in the launch
configuration bench.py times.  The oracle is run where it finishes in seconds:
on sampled queries against the exported graph, on sampled brute-force rows, and
(one test, about a minute of host time) on the whole build."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_07048_amd import datagen
from gpu_common import dev, u32

pytestmark = pytest.mark.gpu

N, NQ, R, LB = 1_000_000, 10_000, 64, 128


@pytest.fixture(scope="module")
def jx():
    from paper_2601_07048_amd import jx as m
    return m


@pytest.fixture(scope="module")
def big(jx):
    x = datagen.base(2, N)
    q = datagen.queries(2, NQ)
    g = jx.Index(128, jx.U8, R, LB, 1.2, capacity=N, max_batch=N // 4 + 1)
    g.insert(dev(x))
    torch.cuda.synchronize()
    adj, deg = g.export_graph()
    return x, q, g, adj, deg


def test_fullsize_graph_invariants(jx, big):
    x, q, g, adj, deg = big
    n, entry = g.size()
    assert n == N and 0 <= entry < N
    a = adj.to(torch.int64) & 0xFFFFFFFF
    valid = a != 0xFFFFFFFF
    assert bool(((a < N) | ~valid).all())
    # rows are filled from the left and the degree matches
    assert bool((valid.sum(1) == deg).all())
    idx = torch.arange(R, device=a.device)[None, :]
    assert bool((valid == (idx < deg[:, None])).all())
    # no self loops, no duplicates
    assert not bool((a == torch.arange(N, device=a.device)[:, None]).any())
    s, _ = torch.sort(a, dim=1)
    dup = (s[:, 1:] == s[:, :-1]) & (s[:, 1:] != 0xFFFFFFFF)
    assert not bool(dup.any())
    assert int(deg.min()) >= 1 and 30 < float(deg.float().mean()) < 60


def test_fullsize_search_sampled_against_oracle(jx, big):
    """Sampled queries: the oracle's beamSearch on the exported graph must give
    the same ids and distances, bit for bit, at the benchmark's beam widths."""
    x, q, g, adj, deg = big
    ref = oracle.Index(128, np.uint8, R, LB, 1.2, N)
    ref.set_graph(x, u32(adj), g.size()[1])
    sample = np.random.default_rng(0).choice(NQ, 200, replace=False)
    dq = dev(q)
    for L in (32, 96, 256):
        ids, dist, st = g.search(dq, 10, L, stats=True)
        want = ref.search(q[sample], 10, L)
        assert np.array_equal(u32(ids)[sample], want["ids"])
        assert np.array_equal(dist.cpu().numpy().astype(np.float64)[sample], want["dist"])
        assert st["hops"] >= L * NQ * 0.9
    # recall target of the benchmark
    gt, gd = g.bruteforce(dq, 10)
    ids, _ = g.search(dq, 10, 96)
    assert oracle.recall_at_k(u32(ids)[:2000], u32(gt)[:2000]) >= 0.95
    # brute force itself, sampled rows against the CPU definition
    oid, od = oracle.bruteforce(x, q[sample[:16]], 10)
    assert np.array_equal(u32(gt)[sample[:16]], oid)
    assert np.array_equal(gd.cpu().numpy().astype(np.float64)[sample[:16]], od)


def test_fullsize_build_matches_oracle(jx, big):
    """The whole 1M-point adjacency table against the oracle's build with the
    same insertion order and batch schedule (about a minute on 16 host cores)."""
    x, q, g, adj, deg = big
    ref = oracle.Index(128, np.uint8, R, LB, 1.2, N)
    ref.insert(x)
    oadj, odeg = ref.graph()
    assert ref.entry == g.size()[1]
    bad = np.nonzero((u32(adj) != oadj).any(axis=1))[0]
    assert bad.size == 0, f"{bad.size} rows differ, first {bad[:5]}"
