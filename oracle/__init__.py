"""CPU oracle for the Vamana beamSearch / robustPrune / RaBitQ path.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by ``bench.py``'s ``cpu_baseline`` leg, never by the product package.
The arithmetic lives in ``jx_oracle.c`` (plain C, built with gcc); this file
only marshals numpy arrays through ctypes.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libjx_oracle.so")
_SRC = os.path.join(_HERE, "jx_oracle.c")

U8, F32, F16 = 0, 1, 2
NONE = 0xFFFFFFFF
CAND_FRONTIER, CAND_VISITED = 0, 1
FILTER_EXACT, FILTER_NONE = 0, 1
RULE_MAXCOS, RULE_MAXABS = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle (gcc, -O2, OpenMP, no FMA contraction)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_SO)
        L = _lib
        L.orc_l2sq_u8.restype = C.c_int64
        L.orc_l2sq_f32.restype = C.c_double
        L.orc_l2sq_f16.restype = C.c_double
        L.orc_robust_prune.restype = C.c_int
        L.orc_index_create.restype = C.c_void_p
        L.orc_index_size.restype = C.c_int64
        L.orc_index_entry.restype = C.c_uint32
        L.orc_index_insert.restype = C.c_int
        L.orc_index_quantize.restype = C.c_int
        L.orc_index_search.restype = C.c_int
        L.orc_rabitq_code_bytes.restype = C.c_int
        L.orc_rabitq_est_float.restype = C.c_double
        L.orc_rabitq_est_int.restype = C.c_float
        L.orc_num_threads.restype = C.c_int
        L.orc_index_deleted_count.restype = C.c_int64
        L.orc_index_compact.restype = C.c_int64
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dt(a) -> int:
    if a.dtype == np.uint8:
        return U8
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.float16:
        return F16
    raise TypeError(a.dtype)


def num_threads() -> int:
    return lib().orc_num_threads()


def _nt(nthreads):
    return int(nthreads) if nthreads else num_threads()


# ---------------------------------------------------------------- distances
def l2sq(a: np.ndarray, b: np.ndarray):
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    if a.dtype == np.uint8:
        return int(lib().orc_l2sq_u8(_p(a), _p(b), C.c_int(a.size)))
    if a.dtype == np.float16:
        return float(lib().orc_l2sq_f16(_p(a), _p(b), C.c_int(a.size)))
    return float(lib().orc_l2sq_f32(_p(a), _p(b), C.c_int(a.size)))


def bruteforce(base, queries, k, nthreads=None):
    base = np.ascontiguousarray(base)
    queries = np.ascontiguousarray(queries)
    assert base.dtype == queries.dtype
    n, d = base.shape
    nq = queries.shape[0]
    ids = np.empty((nq, k), np.uint32)
    dist = np.empty((nq, k), np.float64)
    lib().orc_bruteforce(_p(base), C.c_int(_dt(base)), C.c_int64(n), C.c_int(d), _p(queries), C.c_int64(nq),
                         C.c_int(k), _p(ids), _p(dist), C.c_int(_nt(nthreads)))
    return ids, dist


def mips_augment(x, max_norm, is_query=False, dim_out=None):
    """Inner-product search as L2 search (Sec. 6.3): append sqrt(M^2 - |x|^2) to base rows, 0 to query rows,
    then zero padding up to dim_out.  Everything in float64, rounded to float32 at the end."""
    x = np.asarray(x, dtype=np.float64)
    n, d = x.shape
    dim_out = dim_out or d + 1
    out = np.zeros((n, dim_out), np.float64)
    out[:, :d] = x
    if not is_query:
        out[:, d] = np.sqrt(np.maximum(float(max_norm) ** 2 - (x * x).sum(axis=1), 0.0))
    return out.astype(np.float32)


# ---------------------------------------------------------------- beamSearch
def beam_search(adj, base, query, L, start, filter=FILTER_EXACT, V_cap=0):
    """One query on a caller-supplied graph.  Returns dict(F_ids, F_dist, nF,
    V_ids, V_dist, nV, hops, evals)."""
    adj = np.ascontiguousarray(adj, dtype=np.uint32)
    base = np.ascontiguousarray(base)
    query = np.ascontiguousarray(query, dtype=base.dtype)
    n, d = base.shape
    R = adj.shape[1]
    F_ids = np.empty(L, np.uint32)
    F_dist = np.empty(L, np.float64)
    V_ids = np.empty(max(V_cap, 1), np.uint32)
    V_dist = np.empty(max(V_cap, 1), np.float64)
    nF = C.c_int32(0)
    nV = C.c_int32(0)
    hops = C.c_int64(0)
    evals = C.c_int64(0)
    lib().orc_beam_search(_p(adj), C.c_int(R), _p(base), C.c_int(_dt(base)), C.c_int64(n), C.c_int(d), _p(query),
                          C.c_int(L), C.c_uint32(start), C.c_int(filter), _p(F_ids), _p(F_dist), C.byref(nF),
                          _p(V_ids), _p(V_dist), C.c_int32(V_cap), C.byref(nV), C.byref(hops), C.byref(evals))
    m = min(nV.value, V_cap)
    return dict(F_ids=F_ids[: nF.value], F_dist=F_dist[: nF.value], nF=nF.value, V_ids=V_ids[:m], V_dist=V_dist[:m],
                nV=nV.value, hops=hops.value, evals=evals.value)


# ---------------------------------------------------------------- robustPrune
def robust_prune(p_id, cand_ids, cand_dist, base, R, alpha):
    base = np.ascontiguousarray(base)
    cand_ids = np.ascontiguousarray(cand_ids, dtype=np.uint32)
    cand_dist = np.ascontiguousarray(cand_dist, dtype=np.float64)
    out = np.empty(R, np.uint32)
    k = lib().orc_robust_prune(C.c_uint32(p_id), _p(cand_ids), _p(cand_dist), C.c_int64(cand_ids.size), _p(base),
                               C.c_int(_dt(base)), C.c_int(base.shape[1]), C.c_int(R), C.c_float(alpha), _p(out))
    return out[:k].copy()


# ---------------------------------------------------------------- RaBitQ pieces
def rabitq_rotate(vecs, P, c, nthreads=None):
    vecs = np.ascontiguousarray(vecs, dtype=np.float32)
    P = np.ascontiguousarray(P, dtype=np.float32)
    c = np.ascontiguousarray(c, dtype=np.float32)
    n, d = vecs.shape
    o32 = np.empty((n, d), np.float32)
    o64 = np.empty((n, d), np.float64)
    lib().orc_rabitq_rotate(_p(vecs), C.c_int64(n), C.c_int(d), _p(P), _p(c), _p(o32), _p(o64), C.c_int(_nt(nthreads)))
    return o32, o64


def rabitq_code_bytes(d, bits):
    return lib().orc_rabitq_code_bytes(C.c_int(d), C.c_int(bits))


def rabitq_encode(r32, bits, rule=RULE_MAXCOS, nthreads=None):
    r32 = np.ascontiguousarray(r32, dtype=np.float32)
    n, d = r32.shape
    cb = rabitq_code_bytes(d, bits)
    codes = np.zeros((n, cb), np.uint8)
    meta = np.empty((n, 2), np.float32)
    cos = np.empty(n, np.float64)
    lib().orc_rabitq_encode(_p(r32), C.c_int64(n), C.c_int(d), C.c_int(bits), C.c_int(rule), _p(codes), _p(meta),
                            _p(cos), C.c_int(_nt(nthreads)))
    return codes, meta, cos


def rabitq_unpack(code, bits, d):
    code = np.ascontiguousarray(code, dtype=np.uint8)
    out = np.empty(d, np.uint8)
    lib().orc_rabitq_unpack(_p(code), C.c_int(bits), C.c_int(d), _p(out))
    return out


def rabitq_query_prep(qr32, bits, qbits):
    qr32 = np.ascontiguousarray(qr32, dtype=np.float32)
    d = qr32.size
    qint = np.empty(d, np.uint8)
    m4 = np.empty(4, np.float32)
    lib().orc_rabitq_query_prep(_p(qr32), C.c_int(d), C.c_int(bits), C.c_int(qbits), _p(qint), _p(m4))
    return qint, m4  # m4 = lo, delta, query_add, query_sumq


def rabitq_est_float(code, bits, d, data_add, data_rescale, qr64):
    code = np.ascontiguousarray(code, dtype=np.uint8)
    qr64 = np.ascontiguousarray(qr64, dtype=np.float64)
    return float(lib().orc_rabitq_est_float(_p(code), C.c_int(bits), C.c_int(d), C.c_double(data_add),
                                            C.c_double(data_rescale), _p(qr64)))


def rabitq_est_int(code, bits, d, data_add, data_rescale, qint, m4):
    code = np.ascontiguousarray(code, dtype=np.uint8)
    qint = np.ascontiguousarray(qint, dtype=np.uint8)
    return float(lib().orc_rabitq_est_int(_p(code), C.c_int(bits), C.c_int(d), C.c_float(data_add),
                                          C.c_float(data_rescale), _p(qint), C.c_float(m4[0]), C.c_float(m4[1]),
                                          C.c_float(m4[2]), C.c_float(m4[3])))


def rabitq_int_dot(code, bits, d, qint):
    code = np.ascontiguousarray(code, dtype=np.uint8)
    qint = np.ascontiguousarray(qint, dtype=np.uint8)
    I = C.c_int64(0)
    S = C.c_int64(0)
    lib().orc_rabitq_int_dot(_p(code), C.c_int(bits), C.c_int(d), _p(qint), C.byref(I), C.byref(S))
    return I.value, S.value


# ---------------------------------------------------------------- index
class Index:
    """Vector store + Vamana graph built by batch insertion (Alg. 4)."""

    def __init__(self, d, dtype, R, L_build, alpha, capacity, cand_mode=CAND_FRONTIER, batch_growth=0.25):
        self.d, self.R, self.L_build, self.alpha, self.capacity = d, R, L_build, alpha, capacity
        self.np_dtype = np.dtype(dtype)
        self.dtype = _dt(np.empty(0, self.np_dtype))
        self._h = C.c_void_p(lib().orc_index_create(C.c_int(d), C.c_int(self.dtype), C.c_int(R), C.c_int(L_build),
                                                    C.c_float(alpha), C.c_int64(capacity), C.c_int(cand_mode),
                                                    C.c_float(batch_growth)))
        self.bits = 0

    def __del__(self):
        if getattr(self, "_h", None):
            lib().orc_index_destroy(self._h)
            self._h = None

    @property
    def n(self):
        return int(lib().orc_index_size(self._h))

    @property
    def entry(self):
        return int(lib().orc_index_entry(self._h))

    def insert(self, vecs, nthreads=None):
        vecs = np.ascontiguousarray(vecs, dtype=self.np_dtype)
        assert vecs.shape[1] == self.d
        rc = lib().orc_index_insert(self._h, _p(vecs), C.c_int64(vecs.shape[0]), C.c_int(_nt(nthreads)))
        if rc != 0:
            raise RuntimeError("oracle insert failed: capacity")

    def set_graph(self, vecs, adj, entry):
        vecs = np.ascontiguousarray(vecs, dtype=self.np_dtype)
        adj = np.ascontiguousarray(adj, dtype=np.uint32)
        assert adj.shape == (vecs.shape[0], self.R)
        lib().orc_index_set_graph(self._h, _p(vecs), C.c_int64(vecs.shape[0]), _p(adj), C.c_uint32(entry))

    def graph(self):
        n = self.n
        adj = np.empty((n, self.R), np.uint32)
        deg = np.empty(n, np.uint32)
        lib().orc_index_get_graph(self._h, _p(adj), _p(deg))
        return adj, deg

    def delete(self, ids):
        ids = np.ascontiguousarray(ids, dtype=np.uint32)
        lib().orc_index_delete(self._h, _p(ids), C.c_int64(ids.size))

    @property
    def n_deleted(self):
        return int(lib().orc_index_deleted_count(self._h))

    def consolidate(self, nthreads=None):
        lib().orc_index_consolidate(self._h, C.c_int(_nt(nthreads)))

    def compact(self):
        """Remove the deleted vertices (after consolidate); returns old id -> new id (NONE for removed)."""
        m = np.empty(self.n, np.uint32)
        rc = lib().orc_index_compact(self._h, _p(m))
        if rc < 0:
            raise RuntimeError("compact needs a consolidated index")
        return m

    def quantize(self, bits, P, centroid=None, qbits=8, rule=RULE_MAXCOS, nthreads=None):
        P = np.ascontiguousarray(P, dtype=np.float32)
        c = None if centroid is None else np.ascontiguousarray(centroid, dtype=np.float32)
        rc = lib().orc_index_quantize(self._h, C.c_int(bits), C.c_int(qbits), C.c_int(rule), _p(P), _p(c),
                                      C.c_int(_nt(nthreads)))
        if rc != 0:
            raise RuntimeError("oracle quantize: float data only")
        self.bits = bits

    def set_codes(self, bits, P, centroid, codes, meta, qbits=8):
        P = np.ascontiguousarray(P, dtype=np.float32)
        centroid = np.ascontiguousarray(centroid, dtype=np.float32)
        codes = np.ascontiguousarray(codes, dtype=np.uint8)
        meta = np.ascontiguousarray(meta, dtype=np.float32)
        lib().orc_index_set_codes(self._h, C.c_int(bits), C.c_int(qbits), _p(P), _p(centroid), _p(codes), _p(meta))
        self.bits = bits

    def codes(self):
        n = self.n
        cb = rabitq_code_bytes(self.d, self.bits)
        codes = np.empty((n, cb), np.uint8)
        meta = np.empty((n, 2), np.float32)
        cen = np.empty(self.d, np.float32)
        lib().orc_index_get_codes(self._h, _p(codes), _p(meta), _p(cen))
        return codes, meta, cen

    def search(self, queries, k, L, mode=0, rerank=0, filter=FILTER_EXACT, want_frontier=False, nthreads=None):
        queries = np.ascontiguousarray(queries, dtype=self.np_dtype)
        nq = queries.shape[0]
        ids = np.empty((nq, k), np.uint32)
        dist = np.empty((nq, k), np.float64)
        F_ids = np.empty((nq, L), np.uint32) if want_frontier else None
        F_dist = np.empty((nq, L), np.float64) if want_frontier else None
        stats = np.zeros(2, np.int64)
        rc = lib().orc_index_search(self._h, _p(queries), C.c_int64(nq), C.c_int(k), C.c_int(L), C.c_int(mode),
                                    C.c_int(rerank), C.c_int(filter), _p(ids), _p(dist), _p(F_ids), _p(F_dist),
                                    _p(stats), C.c_int(_nt(nthreads)))
        if rc != 0:
            raise RuntimeError(f"oracle search failed rc={rc}")
        out = dict(ids=ids, dist=dist, hops=int(stats[0]), evals=int(stats[1]))
        if want_frontier:
            out["F_ids"], out["F_dist"] = F_ids, F_dist
        return out


def recall_at_k(found_ids, true_ids):
    """Sec. 6.1: fraction of the exact top-k that appear among the k returned."""
    k = true_ids.shape[1]
    hit = 0
    for f, t in zip(found_ids, true_ids):
        hit += len(set(f.tolist()) & set(t.tolist()))
    return hit / (k * len(true_ids))
