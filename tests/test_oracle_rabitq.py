"""Pins for the oracle's RaBitQ encoder / estimator (Sec. 5.1).  No GPU.

The paper gives no worked numeric example, and its printed metadata formulas
are partly garbled, so the estimator is pinned by mathematics instead:
on-grid vectors (estimate must be exact), unbiasedness, the closed-form error
law over a random rotation, optimality of the code against brute force, and
deterministic rounding bounds of the integer-query form.
"""
import itertools

import numpy as np
import pytest

import oracle
from paper_2601_07048_amd import datagen


def test_record_size_and_packing():
    assert oracle.rabitq_code_bytes(960, 4) == 480   # + 2 floats = 488 B
    assert oracle.rabitq_code_bytes(1536, 1) == 192  # + 2 floats = 200 B
    r = np.array([[0.3, -0.1, 2.0, -3.0, 0.0, 1.0, -1.0, 0.5]], np.float32)
    codes, meta, _ = oracle.rabitq_encode(r, 1)
    assert oracle.rabitq_unpack(codes[0], 1, 8).tolist() == [1, 0, 1, 0, 1, 1, 0, 1]
    assert codes[0, 0] == 0b10110101  # coordinate i -> bit i of the byte
    # ||r||^2 and -4||r||^2/||r||_1 (1-bit closed form)
    l2 = float((r.astype(np.float64) ** 2).sum())
    l1 = float(np.abs(r.astype(np.float64)).sum())
    assert np.isclose(meta[0, 0], l2, rtol=1e-6) and np.isclose(meta[0, 1], -4 * l2 / l1, rtol=1e-6)
    c4, _, _ = oracle.rabitq_encode(np.array([[7.5, -7.5, 0.5, -0.5]], np.float32), 4, oracle.RULE_MAXABS)
    assert oracle.rabitq_unpack(c4[0], 4, 4).tolist() == [15, 0, 8, 7]
    assert c4[0].tolist() == [0x0F, 0x78]  # even coordinate -> low nibble


def test_rotate_matches_numpy():
    rng = np.random.default_rng(1)
    d = 48
    P = datagen.random_orthogonal(d, 5).astype(np.float32)
    v = rng.standard_normal((7, d)).astype(np.float32)
    c = rng.standard_normal(d).astype(np.float32)
    r32, r64 = oracle.rabitq_rotate(v, P, c)
    ref = (v.astype(np.float64) - c.astype(np.float64)) @ P.astype(np.float64).T
    assert np.allclose(r64, ref, rtol=0, atol=1e-12)
    assert np.array_equal(r32, r64.astype(np.float32))


@pytest.mark.parametrize("bits,rule", [(1, 0), (4, oracle.RULE_MAXCOS), (4, oracle.RULE_MAXABS), (2, oracle.RULE_MAXCOS),
                                       (2, oracle.RULE_MAXABS), (8, oracle.RULE_MAXCOS), (8, oracle.RULE_MAXABS)])
def test_on_grid_vector_estimate_is_exact(bits, rule):
    """If r lies exactly on a ray through a grid point the code is parallel to
    r, and est = ||r||^2 + ||q'||^2 - 2<r,q'> must hold exactly: this checks the
    signs and constants of all four metadata terms (c_b in particular)."""
    rng = np.random.default_rng(2)
    half = 1 << (bits - 1)
    d = max(64, 2 * half)
    lev = rng.integers(0, half, d)
    lev[:half] = np.arange(half)  # every level present
    sgn = rng.choice([-1.0, 1.0], d)
    scale = 0.37
    r = (sgn * (lev + 0.5) * scale).astype(np.float32)[None]
    codes, meta, cos = oracle.rabitq_encode(r, bits, rule)
    assert abs(cos[0] - 1.0) < 1e-9
    u = oracle.rabitq_unpack(codes[0], bits, d).astype(np.float64)
    assert np.array_equal(u - (2 ** bits - 1) / 2, sgn * (lev + 0.5))
    for _ in range(20):
        q = rng.standard_normal(d) * 3 + 1.5  # non-zero mean: a wrong c_b shows up
        est = oracle.rabitq_est_float(codes[0], bits, d, float(meta[0, 0]), float(meta[0, 1]), q)
        true = float(((r[0].astype(np.float64) - q) ** 2).sum())
        assert abs(est - true) <= 2e-6 * true  # only the float32 rounding of the two stored floats


def test_zero_vector_is_degenerate_but_finite():
    r = np.zeros((1, 16), np.float32)
    for bits in (1, 2, 4, 8):
        codes, meta, _ = oracle.rabitq_encode(r, bits)
        assert meta[0].tolist() == [0.0, 0.0]
        u = oracle.rabitq_unpack(codes[0], bits, 16)
        assert (u == (1 << (bits - 1))).all()
        q = np.arange(16, dtype=np.float64)
        assert oracle.rabitq_est_float(codes[0], bits, 16, 0.0, 0.0, q) == float((q ** 2).sum())


def _pairs(d, n, seed, bits, rule):
    rng = np.random.default_rng(seed)
    P = datagen.random_orthogonal(d, seed + 1).astype(np.float32)
    c = (rng.standard_normal(d) * 0.5).astype(np.float32)
    v = (rng.standard_normal((n, d)) * rng.uniform(0.5, 2.0, (n, 1)) + c).astype(np.float32)  # isotropic about c
    q = (rng.standard_normal((n, d)) + 0.8).astype(np.float32)  # non-centred queries
    r32, _ = oracle.rabitq_rotate(v, P, c)
    _, q64 = oracle.rabitq_rotate(q, P, c)
    codes, meta, cos = oracle.rabitq_encode(r32, bits, rule)
    return v, q, r32, q64, codes, meta, cos


@pytest.mark.parametrize("bits,rule", [(1, 0), (4, oracle.RULE_MAXCOS), (4, oracle.RULE_MAXABS), (2, oracle.RULE_MAXCOS),
                                       (8, oracle.RULE_MAXABS)])
def test_estimator_unbiased_and_error_law(bits, rule):
    """est - true = -2 ||r|| tan(theta) ||q_perp|| Z with Z one coordinate of a
    uniform unit vector of R^(d-1) (mean 0, variance 1/(d-1)): the normalised
    error must have mean ~0, std 1/sqrt(d-1) within 10 %, and stay below
    4/sqrt(d-1) for at least 99.9 % of the pairs."""
    d, n = 192, 6000
    v, q, r32, q64, codes, meta, cos = _pairs(d, n, 11, bits, rule)
    z = np.empty(n)
    err = np.empty(n)
    for i in range(n):
        est = oracle.rabitq_est_float(codes[i], bits, d, float(meta[i, 0]), float(meta[i, 1]), q64[i])
        true = oracle.l2sq(v[i], q[i])
        r = r32[i].astype(np.float64)
        nr = np.linalg.norm(r)
        o = r / nr
        qp = q64[i] - (q64[i] @ o) * o
        tan = np.sqrt(max(1 - cos[i] ** 2, 0)) / cos[i]
        err[i] = est - true
        z[i] = err[i] / (2 * nr * tan * np.linalg.norm(qp))
    assert abs(err.mean()) <= 3 * err.std() / np.sqrt(n)          # unbiased
    assert abs(z.mean()) <= 3 * z.std() / np.sqrt(n)
    assert abs(z.std() * np.sqrt(d - 1) - 1.0) < 0.10              # error law
    assert (np.abs(z) <= 4 / np.sqrt(d - 1)).mean() >= 0.999       # error bound


def test_one_bit_cosine_closed_form_and_coordinate_concentration():
    """E[cos theta] = E||o||_1/sqrt(d) -> sqrt(2/pi) for a uniformly random
    direction; rotated unit-vector coordinates exceed 2/sqrt(d) in about 4.6 %
    of the cases (Sec. 5.1 quotes this concentration)."""
    d = 512
    rng = np.random.default_rng(3)
    v = rng.standard_normal((400, d)).astype(np.float32)
    P = datagen.random_orthogonal(d, 9).astype(np.float32)
    r32, r64 = oracle.rabitq_rotate(v, P, np.zeros(d, np.float32))
    _, _, cos = oracle.rabitq_encode(r32, 1)
    assert abs(cos.mean() - np.sqrt(2 / np.pi)) < 0.005
    o = r64 / np.linalg.norm(r64, axis=1, keepdims=True)
    frac = (np.abs(o) > 2 / np.sqrt(d)).mean()
    assert 0.035 < frac < 0.055


def test_sweep_is_optimal():
    """Max-cosine rule: (a) on d<=4, m=2 it equals brute force over all 4^d grid
    points; (b) on real sizes it is never worse than max-abs scaling."""
    rng = np.random.default_rng(4)
    for d in (1, 2, 3, 4):
        r = rng.standard_normal((50, d)).astype(np.float32)
        _, _, cos = oracle.rabitq_encode(r, 2, oracle.RULE_MAXCOS)
        grid = np.array(list(itertools.product([-1.5, -0.5, 0.5, 1.5], repeat=d)))
        gn = grid / np.linalg.norm(grid, axis=1, keepdims=True)
        for i in range(50):
            o = r[i].astype(np.float64)
            o /= np.linalg.norm(o)
            assert abs(cos[i] - (gn @ o).max()) < 1e-12
    r = rng.standard_normal((200, 96)).astype(np.float32) * rng.uniform(0.1, 3, (200, 1)).astype(np.float32)
    ca, ma, cos_a = oracle.rabitq_encode(r, 4, oracle.RULE_MAXCOS)
    cb, mb, cos_b = oracle.rabitq_encode(r, 4, oracle.RULE_MAXABS)
    assert (cos_a >= cos_b - 1e-12).all() and cos_a.mean() > cos_b.mean()
    assert cos_a.min() > 0.98
    # the reported cosine is the cosine of the emitted code
    for i in range(0, 200, 17):
        u = oracle.rabitq_unpack(ca[i], 4, 96).astype(np.float64) - 7.5
        o = r[i].astype(np.float64)
        assert abs(u @ o / np.linalg.norm(u) / np.linalg.norm(o) - cos_a[i]) < 1e-12


@pytest.mark.parametrize("bits", [1, 2, 4, 8])
@pytest.mark.parametrize("qbits", [4, 8])
def test_integer_query_form(bits, qbits):
    """|<u,q'> - (delta <u,q_int> + lo sum u)| <= delta/2 * sum u, and the
    float32 estimate equals the same expression evaluated in double to float
    rounding."""
    d, n = 160, 300
    v, q, r32, q64, codes, meta, cos = _pairs(d, n, 21, bits, oracle.RULE_MAXCOS)
    cb = (2 ** bits - 1) / 2
    for i in range(n):
        qr = q64[i].astype(np.float32)
        qint, m4 = oracle.rabitq_query_prep(qr, bits, qbits)
        lo, delta, qadd, qsum = [float(t) for t in m4]
        assert qint.max() <= 2 ** qbits - 1 and qint.max() == 2 ** qbits - 1 and qint.min() == 0
        assert np.isclose(lo, qr.min()) and np.isclose(delta, (qr.max() - qr.min()) / (2 ** qbits - 1), rtol=1e-6)
        assert np.abs(lo + delta * qint.astype(np.float64) - qr).max() <= delta * 0.5 * (1 + 1e-4)
        assert np.isclose(qadd, (qr.astype(np.float64) ** 2).sum(), rtol=1e-6)
        assert np.isclose(qsum, cb * qr.astype(np.float64).sum(), rtol=1e-5, atol=1e-5)
        u = oracle.rabitq_unpack(codes[i], bits, d).astype(np.int64)
        I, S = oracle.rabitq_int_dot(codes[i], bits, d, qint)
        assert I == int((u * qint.astype(np.int64)).sum()) and S == int(u.sum())
        exact_ip = float(u @ qr.astype(np.float64))
        assert abs(exact_ip - (delta * I + lo * S)) <= 0.5 * delta * S * (1 + 1e-4) + 1e-9
        e32 = oracle.rabitq_est_int(codes[i], bits, d, meta[i, 0], meta[i, 1], qint, m4)
        e64 = float(meta[i, 0]) + qadd + float(meta[i, 1]) * (delta * I + lo * S - qsum)
        assert abs(e32 - e64) <= 1e-5 * (abs(float(meta[i, 0])) + qadd + abs(float(meta[i, 1]) * (delta * I + abs(lo) * S + abs(qsum))))


def test_query_prep_constant_query():
    qint, m4 = oracle.rabitq_query_prep(np.full(8, 2.5, np.float32), 1, 8)
    assert qint.tolist() == [0] * 8 and m4[1] == 0.0 and m4[0] == 2.5
    assert m4[2] == 50.0 and m4[3] == 0.5 * 20.0


def test_quantized_search_and_rerank():
    """Index-level: quantise, search with the estimator, re-rank exactly.
    L >= N with rerank = N must reproduce brute force (rerank is a plain
    definition); with the default 4k candidates recall must not drop."""
    n, d = 1500, 96
    rng = np.random.default_rng(7)
    cent = rng.standard_normal((8, d)) * 0.5
    x = (cent[rng.integers(0, 8, n)] + 0.3 * rng.standard_normal((n, d))).astype(np.float32)
    q = (cent[rng.integers(0, 8, 40)] + 0.3 * rng.standard_normal((40, d))).astype(np.float32)
    P = datagen.random_orthogonal(d, 77).astype(np.float32)
    ix = oracle.Index(d, np.float32, 24, 48, 1.2, n)
    ix.insert(x)
    gt, gd = oracle.bruteforce(x, q, 10)
    exact = oracle.recall_at_k(ix.search(q, 10, 48)["ids"], gt)
    for bits in (1, 4):
        ix.quantize(bits, P)
        codes, meta, cen = ix.codes()
        assert codes.shape == (n, d * bits // 8)
        assert np.allclose(cen, x.astype(np.float64).mean(0), atol=1e-6)
        full = ix.search(q, 10, n + 10, mode=1, rerank=n + 10)
        # the graph may leave a few vertices unreachable; compare where reached
        same = full["ids"] == gt
        assert same.mean() > 0.98
        assert np.allclose(full["dist"][same], gd[same], rtol=1e-12)
        raw = oracle.recall_at_k(ix.search(q, 10, 48, mode=1)["ids"], gt)
        rr = ix.search(q, 10, 48, mode=1, rerank=40)
        rer = oracle.recall_at_k(rr["ids"], gt)
        assert rer >= raw
        assert rer >= (0.85 if bits == 4 else 0.6) * exact
        # reranked distances are exact and sorted by (distance, id)
        for i in range(len(q)):
            keys = list(zip(rr["dist"][i].tolist(), rr["ids"][i].tolist()))
            assert keys == sorted(keys)
            assert rr["dist"][i, 0] == oracle.l2sq(q[i], x[rr["ids"][i, 0]])


def test_rabitq_on_uint8_equals_the_same_values_as_float32():
    """uint8 -> float32 is exact: an index on uint8 vectors must give the codes, the two floats and the search
    results of an index on the same values stored as float32 (whose path is pinned above)."""
    from paper_2601_07048_amd import datagen
    n, d = 2000, 64
    rng = np.random.default_rng(12)
    x = rng.integers(0, 256, (n, d), dtype=np.uint8)
    q = rng.integers(0, 256, (50, d), dtype=np.uint8)
    a = oracle.Index(d, np.uint8, 16, 32, 1.2, n)
    a.insert(x)
    adj, _ = a.graph()
    b = oracle.Index(d, np.float32, 16, 32, 1.2, n)
    b.set_graph(x.astype(np.float32), adj, a.entry)
    P = datagen.random_orthogonal(d, seed=2).astype(np.float32)
    for bits in (1, 4):
        a.quantize(bits, P)
        b.quantize(bits, P)
        ca, ma, cena = a.codes()
        cb, mb, cenb = b.codes()
        assert np.array_equal(ca, cb) and np.array_equal(ma, mb) and np.array_equal(cena, cenb)
        ra = a.search(q, 5, 32, mode=1, rerank=20)
        rb = b.search(q.astype(np.float32), 5, 32, mode=1, rerank=20)
        assert np.array_equal(ra["ids"], rb["ids"]) and np.array_equal(ra["dist"], rb["dist"])
