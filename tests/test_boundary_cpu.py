"""CPU-side checks of the C boundary: the library loads and exports every
entry point that include/kvp.h declares.  No compute call is made here."""
import ctypes
import os
import re

import paper_2508_13231_amd as K

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "kvp.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(kvp_[a-z_]+)\s*\(", src)))


def test_header_and_binding_agree():
    assert _declared() == sorted(K.EXPORTS)


def test_library_exports_every_declared_symbol():
    lib = K.lib()
    for name in _declared():
        assert hasattr(lib, name), name
    assert K.strerror(0) == "ok" and "trace" in K.strerror(K.KVP_ENOTRACE)


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(K.kvp_problem) == 24 + 64 + 16 + 24 + 8
    assert ctypes.sizeof(K.kvp_anneal_params) == 8 + 8 + 8 + 8 + 8 + 16 + 24
    assert ctypes.sizeof(K.kvp_chain_stats_t) == 80
    assert K.kvp_problem.plane_bytes.offset == 24 and K.kvp_problem.bw_hbm.offset == 104
    assert K.kvp_anneal_params.p0.offset == 40


def test_enumerators_match_the_header():
    """Every `NAME = value` of the header's enums has the same value in the binding."""
    src = open(os.path.join(ROOT, "include", "kvp.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    seen = 0
    for body in re.findall(r"enum\s*\w*\s*\{(.*?)\}", src, flags=re.S):
        for name, value in re.findall(r"\b(KVP_[A-Z0-9_]+)\s*=\s*(-?\d+)", body):
            assert getattr(K, name) == int(value), name
            seen += 1
    assert seen >= 25 and K.KVP_SCORE_ROWLANE == 13
