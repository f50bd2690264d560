"""CPU-side checks of the boundary: the shared library loads without a GPU and
exports every function that include/prs.h declares; host-only entry points
behave."""
from __future__ import annotations

import os
import re

import paper_1310_4645_amd as prs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "prs.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(?:int|size_t)\s+(\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert {"simulate_completion_batch", "greedy_schedule_batch", "replay_reduction"} <= set(names)
    lib = prs.load_library()
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(prs.binding.EXPORTS) == names
    assert lib.prs_abi_version() == 2


def test_workspace_sizes_are_monotone_and_bounded():
    w = prs.prs_workspace_bytes
    # small machines keep their state in LDS; beyond 1024 processors it moves to the workspace
    assert w(prs.PRS_CALL_SIMULATE, prs.PRS_UNI, 1, 10, 64, 8) <= w(prs.PRS_CALL_SIMULATE, prs.PRS_UNI, 1, 10, 1024, 8)
    assert w(prs.PRS_CALL_SIMULATE, prs.PRS_UNI, 1, 10, 1024, 8) < w(prs.PRS_CALL_SIMULATE, prs.PRS_UNI, 1, 10, 4096, 8)
    assert w(prs.PRS_CALL_SIMULATE, prs.PRS_BI, 1, 10, 64, 8) < w(prs.PRS_CALL_SIMULATE, prs.PRS_BI, 1, 10, 64, 512)
    assert w(prs.PRS_CALL_SCHEDULE, prs.PRS_UNI, 1, 10, 1024, 8) < w(prs.PRS_CALL_SCHEDULE, prs.PRS_UNI, 1, 10, 4096, 8)
    assert w(prs.PRS_CALL_SIMULATE, prs.PRS_BI, 1, 10_000, 65536, 4096) <= 20 << 30
    assert w(prs.PRS_CALL_REPLAY, 0, 0, 1, 256, 64) > 256 * 64 * 4
    assert w(99, 0, 0, 1, 256, 64) == 0 and w(0, 0, 0, -1, 256, 64) == 0
    # every segmentation of a message: 2^(m_max-1) configurations per problem, at most 24 units, fewer than 2^31 in all
    u = prs.PRS_CALL_UNEQUAL
    assert 0 < w(u, prs.PRS_UNI, 0, 986, 1024, 10) < w(u, prs.PRS_UNI, 0, 986, 1024, 14)
    assert w(u, prs.PRS_UNI, 0, 986, 1024, 25) == 0 and w(u, prs.PRS_UNI, 0, 1 << 20, 1024, 24) == 0


def test_calls_reject_bad_arguments_before_touching_the_gpu():
    import ctypes as C
    lib = prs.load_library()
    cfg = prs.binding._Configs(0, 0, 0, 0, 0, 0)
    out = prs.binding._Unequal(*([None] * 8))
    rc = lib.unequal_segmentation_batch(C.byref(cfg), 4, prs.PRS_COST_I64, 64, 10, C.byref(out), None, 0, None, None)
    assert rc == 1                                                  # PRS_EINVAL: null arrays with n > 0
    assert lib.unequal_segmentation_batch(C.byref(cfg), 0, prs.PRS_COST_I64, 64, 30, C.byref(out), None, 0, None, None) == 1
    assert lib.unequal_segmentation_batch(C.byref(cfg), 0, prs.PRS_COST_I64, 64, 10, C.byref(out), None, 0, None, None) == 0
    # replay: unknown element type or operation
    off = (C.c_int64 * 2)(0, 8)
    one = C.c_void_p(256)                                            # never dereferenced: the call fails first
    assert lib.replay_reduction(4, 1, off, one, one, one, 3, one, 8, 8, 7, one, None, one, 1 << 20, None) == 1
    assert lib.replay_reduction(4, 1, off, one, one, one, 3, one, 8, 8, prs.PRS_F64 | 0x200, one, None, one, 1 << 20, None) == 1


def test_product_path_has_no_oracle_dependency():
    pkg = os.path.join(ROOT, "paper_1310_4645_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "from oracle" not in src and "prs_oracle" not in src, f
