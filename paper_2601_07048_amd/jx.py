"""Thin ctypes binding of libjx's C ABI (include/jx.h).

Argument marshalling only: every function here forwards torch tensors' device
pointers and the current HIP stream to the entry point of the same name.  There
is no CPU path; importing this module without a built ``libjx.so`` raises.

The library is loaded from this directory; the environment variable ``JX_LIB`` names another build of it (a development
aid for comparing builds; it changes which file is loaded, nothing else).
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("JX_LIB", os.path.join(_HERE, "libjx.so"))

NONE = 0xFFFFFFFF
U8, F32, F16 = 0, 1, 2
EXACT, RABITQ = 0, 1
CAND_FRONTIER, CAND_VISITED = 0, 1
RULE_MAXCOS, RULE_MAXABS, RULE_DEFAULT = 0, 1, -1
# jx_params.flags / jx_set_flags (see include/jx.h)
FLAG_NO_PAIR, FLAG_NO_INCR_PRUNE, FLAG_NO_GRAM, FLAG_GRAM_U8 = 1 << 0, 1 << 1, 1 << 2, 1 << 3
FLAG_VISITED_IDS, FLAG_VISITED_NONE, FLAG_LANES_WIDE, FLAG_LANES_NARROW = 1 << 4, 1 << 5, 1 << 6, 1 << 7
FLAG_TILED_LOADS, FLAG_WAVES_2, FLAG_WAVES_4, FLAG_QPW_2, FLAG_QPW_4 = 1 << 8, 1 << 9, 1 << 10, 1 << 11, 1 << 12
MAX_L, MAX_R, MAX_BF_K = 512, 256, 128

EXPORTS = [
    "jx_arena_bytes", "jx_create", "jx_destroy", "jx_insert", "jx_quantize", "jx_search", "jx_beam_frontier",
    "jx_bruteforce", "jx_size", "jx_export_graph", "jx_import_graph", "jx_export_codes", "jx_import_codes", "jx_rotate",
    "jx_encode_rotated", "jx_delete", "jx_consolidate", "jx_compact", "jx_deleted_count", "jx_probe_gather", "jx_mips_augment", "jx_strerror", "jx_last_error",
    "jx_bruteforce_static", "jx_set_flags",
]


class Params(C.Structure):
    _fields_ = [
        ("dim", C.c_int32), ("dtype", C.c_int32), ("R", C.c_int32), ("L_build", C.c_int32), ("alpha", C.c_float),
        ("cand_mode", C.c_int32), ("capacity", C.c_int64), ("max_batch", C.c_int64), ("quant_bits", C.c_int32),
        ("batch_growth", C.c_float), ("flags", C.c_uint32),
    ]


class Stats(C.Structure):
    _fields_ = [("hops", C.c_uint64), ("dist_evals", C.c_uint64), ("adj_bytes", C.c_uint64),
                ("vec_bytes", C.c_uint64), ("rerank_bytes", C.c_uint64), ("rotate_ms", C.c_float),
                ("prep_ms", C.c_float), ("beam_ms", C.c_float), ("rerank_ms", C.c_float), ("beam_kernel", C.c_char * 96)]

    def as_dict(self):
        out = {k: (float if k.endswith("_ms") else int)(getattr(self, k)) for k, _ in self._fields_ if k != "beam_kernel"}
        out["beam_kernel"] = self.beam_kernel.decode()
        return out


class JxError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"libjx error {code}: {text}")
        self.code = code


def load_library(path: str = LIB_PATH) -> C.CDLL:
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2601_07048_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(path)
    lib.jx_arena_bytes.restype = C.c_int64
    lib.jx_strerror.restype = C.c_char_p
    lib.jx_last_error.restype = C.c_char_p
    for name in EXPORTS:
        getattr(lib, name)  # fail loudly on a missing symbol
    return lib


_lib = load_library()


def _check(rc):
    if rc != 0:
        raise JxError(rc, (_lib.jx_last_error() or b"").decode() or _lib.jx_strerror(rc).decode())


def _ptr(t):
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous()
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _torch_dtype(dtype):
    return {U8: torch.uint8, F32: torch.float32, F16: torch.float16}[dtype]


def jx_arena_bytes(params: Params) -> int:
    n = _lib.jx_arena_bytes(C.byref(params))
    if n < 0:
        _check(int(n))
    return int(n)


class Index:
    """Owns the arena tensor and the opaque handle; methods mirror the C ABI."""

    def __init__(self, dim, dtype, R, L_build, alpha=1.2, capacity=0, max_batch=0, quant_bits=0, batch_growth=0.25,
                 device="cuda:0", flags=0, cand_mode=CAND_FRONTIER):
        self.params = Params(dim=dim, dtype=dtype, R=R, L_build=L_build, alpha=alpha, cand_mode=cand_mode,
                             capacity=capacity, max_batch=max_batch or capacity, quant_bits=quant_bits, batch_growth=batch_growth,
                             flags=flags)
        self.device = torch.device(device)
        self.dim, self.dtype, self.R = dim, dtype, R
        nbytes = jx_arena_bytes(self.params)
        with torch.cuda.device(self.device):
            self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            h = C.c_void_p()
            _check(_lib.jx_create(C.byref(self.params), _ptr(self.arena), C.c_int64(nbytes), _stream(), C.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None) and _lib is not None:  # _lib is gone at interpreter shutdown
            _lib.jx_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    # -- jx_set_flags
    def set_flags(self, flags):
        _check(_lib.jx_set_flags(self._h, C.c_uint32(flags)))

    # -- jx_size
    def size(self):
        n = C.c_int64()
        e = C.c_uint32()
        _check(_lib.jx_size(self._h, C.byref(n), C.byref(e)))
        return n.value, e.value

    # -- jx_insert
    def insert(self, vecs: torch.Tensor):
        assert vecs.dtype == _torch_dtype(self.dtype) and vecs.shape[1] == self.dim
        with torch.cuda.device(self.device):
            _check(_lib.jx_insert(self._h, _ptr(vecs), C.c_int64(vecs.shape[0]), _stream()))

    # -- jx_import_graph / jx_export_graph
    def import_graph(self, vecs, adj, entry):
        assert vecs.dtype == _torch_dtype(self.dtype)
        assert adj.dtype in (torch.int32, torch.uint32)
        assert adj.shape == (vecs.shape[0], self.R)
        with torch.cuda.device(self.device):
            _check(_lib.jx_import_graph(self._h, _ptr(vecs), C.c_int64(vecs.shape[0]), _ptr(adj), C.c_uint32(entry),
                                        _stream()))

    def export_graph(self):
        n, _ = self.size()
        adj = torch.empty((n, self.R), dtype=torch.int32, device=self.device)
        deg = torch.empty(n, dtype=torch.int32, device=self.device)
        with torch.cuda.device(self.device):
            _check(_lib.jx_export_graph(self._h, _ptr(adj), _ptr(deg), _stream()))
        return adj, deg

    # -- jx_quantize / jx_export_codes / stage entry points
    def quantize(self, bits, rotation, centroid=None, query_bits=8, rule=RULE_DEFAULT):
        assert rotation.dtype == torch.float32 and rotation.shape == (self.dim, self.dim)
        with torch.cuda.device(self.device):
            _check(_lib.jx_quantize(self._h, C.c_int32(bits), _ptr(rotation), _ptr(centroid), C.c_int32(query_bits),
                                    C.c_int32(rule), _stream()))
        self.bits = bits

    def import_codes(self, bits, rotation, centroid, codes, meta, query_bits=8):
        assert codes.dtype == torch.uint8 and meta.dtype == torch.float32
        with torch.cuda.device(self.device):
            _check(_lib.jx_import_codes(self._h, C.c_int32(bits), _ptr(rotation), _ptr(centroid), C.c_int32(query_bits),
                                        _ptr(codes), _ptr(meta), _stream()))
        self.bits = bits

    def export_codes(self):
        n, _ = self.size()
        codes = torch.empty((n, self.dim * self.bits // 8), dtype=torch.uint8, device=self.device)
        meta = torch.empty((n, 2), dtype=torch.float32, device=self.device)
        cen = torch.empty(self.dim, dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            _check(_lib.jx_export_codes(self._h, _ptr(codes), _ptr(meta), _ptr(cen), _stream()))
        return codes, meta, cen

    def rotate(self, x):
        out = torch.empty_like(x)
        with torch.cuda.device(self.device):
            _check(_lib.jx_rotate(self._h, _ptr(x), C.c_int64(x.shape[0]), _ptr(out), _stream()))
        return out

    def encode_rotated(self, r):
        n = r.shape[0]
        codes = torch.empty((n, self.dim * self.bits // 8), dtype=torch.uint8, device=self.device)
        meta = torch.empty((n, 2), dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            _check(_lib.jx_encode_rotated(self._h, _ptr(r), C.c_int64(n), _ptr(codes), _ptr(meta), _stream()))
        return codes, meta

    # -- jx_search / jx_beam_frontier / jx_bruteforce
    def search(self, queries, k, L, mode=EXACT, rerank=0, stats=False, out=None):
        nq = queries.shape[0]
        if out is None:
            ids = torch.empty((nq, k), dtype=torch.int32, device=self.device)
            dist = torch.empty((nq, k), dtype=torch.float32, device=self.device)
        else:
            ids, dist = out
        st = Stats() if stats else None
        with torch.cuda.device(self.device):
            _check(_lib.jx_search(self._h, _ptr(queries), C.c_int64(nq), C.c_int32(k), C.c_int32(L), C.c_int32(mode),
                                  C.c_int32(rerank), _ptr(ids), _ptr(dist), C.byref(st) if stats else None, _stream()))
        return (ids, dist, st.as_dict()) if stats else (ids, dist)

    def beam_frontier(self, queries, L, mode=EXACT, stats=False):
        nq = queries.shape[0]
        ids = torch.empty((nq, L), dtype=torch.int32, device=self.device)
        dist = torch.empty((nq, L), dtype=torch.float32, device=self.device)
        st = Stats() if stats else None
        with torch.cuda.device(self.device):
            _check(_lib.jx_beam_frontier(self._h, _ptr(queries), C.c_int64(nq), C.c_int32(L), C.c_int32(mode),
                                         _ptr(ids), _ptr(dist), C.byref(st) if stats else None, _stream()))
        return (ids, dist, st.as_dict()) if stats else (ids, dist)

    def bruteforce(self, queries, k):
        nq = queries.shape[0]
        ids = torch.empty((nq, k), dtype=torch.int32, device=self.device)
        dist = torch.empty((nq, k), dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            _check(_lib.jx_bruteforce(self._h, _ptr(queries), C.c_int64(nq), C.c_int32(k), _ptr(ids), _ptr(dist),
                                      _stream()))
        return ids, dist

    # -- jx_delete / jx_consolidate / jx_deleted_count
    def delete(self, ids: torch.Tensor):
        assert ids.dtype == torch.int32 and ids.dim() == 1
        with torch.cuda.device(self.device):
            _check(_lib.jx_delete(self._h, _ptr(ids), C.c_int64(ids.shape[0]), _stream()))

    def consolidate(self):
        with torch.cuda.device(self.device):
            _check(_lib.jx_consolidate(self._h, _stream()))

    def compact(self, want_map=True):
        """jx_compact; returns old id -> new id (int32 tensor, -1 = NONE for removed vertices) if asked."""
        n_old, _ = self.size()
        m = torch.empty(n_old, dtype=torch.int32, device=self.device) if want_map else None
        with torch.cuda.device(self.device):
            _check(_lib.jx_compact(self._h, _ptr(m), _stream()))
        return m

    def deleted_count(self):
        n = C.c_int64()
        with torch.cuda.device(self.device):
            _check(_lib.jx_deleted_count(self._h, C.byref(n), _stream()))
        return n.value


STATIC_SCRATCH_BYTES = 16 << 20


def bruteforce_static(base: torch.Tensor, queries: torch.Tensor, k: int, out=None):
    """jx_bruteforce_static: exhaustive kNN without an index or an arena; the caller passes the output tensors
    (`out`) when it must not allocate either."""
    dtype = {torch.uint8: U8, torch.float32: F32, torch.float16: F16}[base.dtype]
    assert queries.dtype == base.dtype and queries.shape[1] == base.shape[1]
    nq = queries.shape[0]
    if out is None:
        out = (torch.empty((nq, k), dtype=torch.int32, device=base.device),
               torch.empty((nq, k), dtype=torch.float32, device=base.device))
    ids, dist = out
    with torch.cuda.device(base.device):
        _check(_lib.jx_bruteforce_static(_ptr(base), C.c_int64(base.shape[0]), C.c_int32(base.shape[1]), C.c_int32(dtype),
                                         _ptr(queries), C.c_int64(nq), C.c_int32(k), _ptr(ids), _ptr(dist), _stream()))
    return ids, dist


def mips_augment(x: torch.Tensor, max_norm: float = 0.0, is_query: bool = False, dim_out: int = 0, want_norms: bool = False):
    """jx_mips_augment.  Returns the augmented rows (if dim_out > 0) and / or the row norms."""
    assert x.dtype == torch.float32 and x.is_contiguous()
    n, dim = x.shape
    out = torch.empty((n, dim_out), dtype=torch.float32, device=x.device) if dim_out else None
    norms = torch.empty(n, dtype=torch.float32, device=x.device) if want_norms else None
    with torch.cuda.device(x.device):
        _check(_lib.jx_mips_augment(_ptr(x), C.c_int64(n), C.c_int32(dim), C.c_float(max_norm), C.c_int32(int(is_query)),
                                    _ptr(out), C.c_int32(dim_out), _ptr(norms), _stream()))
    if out is not None and norms is not None:
        return out, norms
    return out if out is not None else norms


def probe_gather(table: torch.Tensor, rec_bytes: int, ids: torch.Tensor, blocks: int = 4096):
    """jx_probe_gather: independent gathers of rec_bytes-byte records; returns the checksum words."""
    assert table.dtype == torch.uint8 and ids.dtype == torch.int32
    n_rec = table.numel() // rec_bytes
    assert 0 <= int(ids.min()) and int(ids.max()) < n_rec  # the device does not check
    sink = torch.empty(blocks * 256, dtype=torch.int32, device=table.device)
    with torch.cuda.device(table.device):
        _check(_lib.jx_probe_gather(_ptr(table), C.c_int64(n_rec), C.c_int32(rec_bytes), _ptr(ids), C.c_int64(ids.numel()),
                                    C.c_int32(blocks), _ptr(sink), _stream()))
    return sink


def ids_to_numpy(t: torch.Tensor):
    """int32 device tensor of ids -> uint32 numpy array."""
    import numpy as np

    return t.cpu().numpy().view(np.uint32)
