"""The C ABI without a GPU: libjx.so loads, exports every function include/jx.h declares, the Python binding names
the same set, and the host-only entry points (sizes, argument checks, error texts) behave as documented.  No kernel
is launched here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "jx.h")
LIB = os.path.join(ROOT, "paper_2601_07048_amd", "libjx.so")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(jx_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    return C.CDLL(LIB)


def test_every_declared_function_is_exported(lib):
    names = _declared()
    assert len(names) >= 20 and "jx_search" in names and "jx_insert" in names
    missing = [n for n in names if not hasattr(lib, n)]
    assert not missing, missing


def test_binding_names_the_same_functions():
    from paper_2601_07048_amd import jx
    assert sorted(jx.EXPORTS) == _declared()


def test_header_constants_match_binding():
    from paper_2601_07048_amd import jx
    text = open(HEADER).read()
    consts = dict(re.findall(r"#define\s+(JX_[A-Z0-9_]+)\s+\(?(-?\d+)\)?", text))
    assert int(consts["JX_U8"]) == jx.U8 and int(consts["JX_F32"]) == jx.F32 and int(consts["JX_F16"]) == jx.F16
    assert int(consts["JX_EXACT"]) == jx.EXACT and int(consts["JX_RABITQ"]) == jx.RABITQ
    assert int(consts["JX_RULE_MAXCOS"]) == jx.RULE_MAXCOS and int(consts["JX_RULE_MAXABS"]) == jx.RULE_MAXABS
    assert int(consts["JX_MAX_L"]) == jx.MAX_L and int(consts["JX_MAX_R"]) == jx.MAX_R
    assert int(consts["JX_MAX_BF_K"]) == jx.MAX_BF_K
    assert int(consts["JX_CAND_FRONTIER"]) == jx.CAND_FRONTIER and int(consts["JX_CAND_VISITED"]) == jx.CAND_VISITED
    assert int(consts["JX_RULE_DEFAULT"]) == jx.RULE_DEFAULT
    # the kernel-variant switches: bit positions in the header and in the binding
    flags = dict(re.findall(r"#define\s+(JX_FLAG_[A-Z0-9_]+)\s+\(1u << (\d+)\)", text))
    assert len(flags) == 13
    for name, bit in flags.items():
        assert getattr(jx, name[3:]) == 1 << int(bit), name


def _params(jx, **kw):
    base = dict(dim=128, dtype=jx.U8, R=64, L_build=128, alpha=1.2, cand_mode=jx.CAND_FRONTIER, capacity=1000,
                max_batch=1000, quant_bits=0, batch_growth=0.25)
    base.update(kw)
    return jx.Params(**base)


def test_arena_size_and_parameter_checks(lib):
    from paper_2601_07048_amd import jx
    lib.jx_arena_bytes.restype = C.c_int64
    lib.jx_last_error.restype = C.c_char_p
    lib.jx_strerror.restype = C.c_char_p
    p = _params(jx)
    n = lib.jx_arena_bytes(C.byref(p))
    # vectors + adjacency + marks at least, 256-byte granules, a workspace of at least 64 MiB
    assert n >= 1000 * 128 + 1000 * 64 * 4 + (64 << 20) and n % 256 == 0
    big = lib.jx_arena_bytes(C.byref(_params(jx, capacity=100000, max_batch=100000)))
    assert big > n
    q = lib.jx_arena_bytes(C.byref(_params(jx, dtype=jx.F32, dim=960, quant_bits=4)))
    assert q >= 1000 * (3840 + 512) + 960 * 960 * 4
    for bad in (dict(dim=0), dict(dim=100), dict(dtype=7), dict(R=0), dict(R=257), dict(L_build=513), dict(alpha=0.5),
                dict(capacity=0), dict(max_batch=0), dict(quant_bits=3), dict(quant_bits=4, dim=48),
                dict(batch_growth=1.5), dict(cand_mode=9), dict(dtype=jx.F16, dim=12), dict(flags=1 << 20)):
        rc = lib.jx_arena_bytes(C.byref(_params(jx, **bad)))
        assert rc == -1, bad
        assert lib.jx_last_error()
    assert lib.jx_strerror(0) == b"ok" and b"capacity" in lib.jx_strerror(-2)
    # NULL handles and pointers are rejected before anything touches a device
    out = C.c_void_p()
    assert lib.jx_create(C.byref(p), None, C.c_int64(n), None, C.byref(out)) == -1
    assert lib.jx_create(C.byref(p), C.c_void_p(256), C.c_int64(16), None, C.byref(out)) == -2
    assert lib.jx_insert(None, None, C.c_int64(1), None) == -1
    assert lib.jx_set_flags(None, 0) == -1
    assert lib.jx_search(None, None, C.c_int64(1), 1, 1, 0, 0, None, None, None, None) == -1
    assert lib.jx_delete(None, None, C.c_int64(1), None) == -1
    assert lib.jx_consolidate(None, None) == -1 and lib.jx_compact(None, None, None) == -1
    assert lib.jx_mips_augment(None, C.c_int64(1), 4, C.c_float(1.0), 0, None, 8, None, None) == -1


def test_product_path_never_imports_the_oracle():
    """The oracle is test infrastructure: nothing under the package may import or load it."""
    pkg = os.path.join(ROOT, "paper_2601_07048_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f), errors="ignore").read()
                assert "import oracle" not in text and "from oracle" not in text and "jx_oracle" not in text, f
