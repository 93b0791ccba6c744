"""The C-ABI library loads, exports every symbol the header declares, and rejects bad arguments
on the host before anything touches a GPU."""
import ctypes
import os
import re

import pytest

from paper_2604_18348_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2604_18348_amd import build
        build.build()
    return B.load_library()


def header_functions():
    src = open(os.path.join(ROOT, "include", "adacluster.h")).read()
    return sorted(set(re.findall(r"\bint\s+(adacluster_\w+)\s*\(", src)))


def test_every_declared_symbol_is_exported(lib):
    names = header_functions()
    assert set(names) == set(B.EXPORTED)
    for n in names:
        assert getattr(lib, n) is not None


def test_params_struct_matches_header():
    src = open(os.path.join(ROOT, "include", "adacluster.h")).read()
    body = src[src.index("typedef struct adacluster_params {"):src.index("} adacluster_params;")]
    fields = re.findall(r"\b(?:int32_t|float)\s+([^;]+);", body)
    names = [n.strip() for f in fields for n in f.split(",")]
    assert names == [f[0] for f in B.CParams._fields_]
    obody = src[src.index("typedef struct adacluster_outputs {"):src.index("} adacluster_outputs;")]
    onames = re.findall(r"\*\s*(\w+)\s*;", obody)
    assert onames == B.COutputs._names


def _rc(lib, **kw):
    p = B.Params(H=2, N=1000, d=64, **kw).c()
    out = ctypes.c_size_t(0)
    return lib.adacluster_workspace_bytes(ctypes.byref(p), ctypes.byref(out)), out.value


def test_workspace_query_and_argument_errors(lib):
    rc, n = _rc(lib)
    assert rc == 0 and n > 0
    assert _rc(lib, q_clusters=0)[0] == -2
    assert _rc(lib, q_clusters=2000)[0] == -2            # more query clusters than tokens
    assert _rc(lib, dtype=7)[0] == -3
    assert _rc(lib, topk=0)[0] == -1
    assert _rc(lib, top_p=0.0)[0] == -1
    assert _rc(lib, top_p=1.5)[0] == -1
    assert _rc(lib, k_m0=2000, k_max_clusters=100)[0] == -2 or _rc(lib, k_m0=2000, k_max_clusters=100)[0] == -1
    assert _rc(lib, k_m0=200, k_max_clusters=100)[0] == -1
    assert _rc(lib, score_mode=5)[0] == -1
    assert _rc(lib, k_max_stages=99)[0] == -1
    assert _rc(lib, tau_abs=0.0, tau_factor=0.0)[0] == -1
    p = B.Params(H=2, N=1000, d=96).c()
    out = ctypes.c_size_t(0)
    assert lib.adacluster_workspace_bytes(ctypes.byref(p), ctypes.byref(out)) == -2
    assert lib.adacluster_workspace_bytes(None, ctypes.byref(out)) == -1
    buf = ctypes.create_string_buffer(256)
    assert lib.adacluster_last_error(buf, 256) == 0 and b"NULL" in buf.value


def test_null_tensor_and_workspace_errors_launch_nothing(lib):
    p = B.Params(H=1, N=64, d=64, q_clusters=4, k_m0=4, k_m_min=2, k_max_clusters=16).c()
    z = ctypes.c_void_p(0)
    assert lib.adacluster_dense_attn(ctypes.byref(p), z, z, z, z, z, 0, z) == -1
    one = ctypes.c_void_p(256)
    assert lib.adacluster_dense_attn(ctypes.byref(p), one, one, one, one, z, 0, z) == -4
    assert lib.adacluster_dense_attn(ctypes.byref(p), one, one, one, one, ctypes.c_void_p(257), 1 << 40, z) == -4
    assert lib.adacluster_dense_attn(ctypes.byref(p), one, one, one, one, one, 16, z) == -4
    buf = ctypes.create_string_buffer(256)
    lib.adacluster_last_error(buf, 256)
    assert b"too small" in buf.value


def test_quest_scores_argument_errors_launch_nothing(lib):
    z, one = ctypes.c_void_p(0), ctypes.c_void_p(256)
    f = lib.adacluster_quest_scores
    assert f(1, 8, 8, 64, B.BF16, B.QUEST_MFMA, 0, z, one, one, one, z) == -1          # NULL tensor
    assert f(0, 8, 8, 64, B.BF16, B.QUEST_ALU, 0, one, one, one, one, z) == -2          # H < 1
    assert f(1, 8, 0, 64, B.BF16, B.QUEST_ALU, 0, one, one, one, one, z) == -2          # no pages
    assert f(1, 8, 8, 96, B.BF16, B.QUEST_ALU, 0, one, one, one, one, z) == -2          # head width
    assert f(1, 8, 8, 64, 9, B.QUEST_ALU, 0, one, one, one, one, z) == -3               # dtype
    assert f(1, 8, 8, 64, B.BF16, 2, 0, one, one, one, one, z) == -1                    # form
    assert f(1, 8, 8, 64, B.F32, B.QUEST_MFMA, 0, one, one, one, one, z) == -5          # matrix cores: bf16 only
