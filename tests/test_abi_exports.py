"""The C-ABI library loads and exports every symbol include/hb.h declares; its host-only entry
points agree with the oracle.  No kernel is launched here (no GPU needed)."""
import ctypes
import os
import re

import pytest

import oracle
from paper_2309_04875_amd import hb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "hb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return re.findall(r"HB_API\s+[\w\s\*]+?\b(hb_\w+)\s*\(", text)


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert sorted(names) == sorted(hb.EXPORTS)
    lib = ctypes.CDLL(hb.LIBRARY)
    for name in names:
        assert getattr(lib, name) is not None


def test_binding_has_the_same_names():
    for name in hb.EXPORTS:
        if name in ("hb_strerror", "hb_last_hip_error"):
            continue
        assert callable(getattr(hb, name))


def test_tensor_seed_matches_oracle():
    for root in (0, 1, 0x2309048750000001, 2**64 - 1):
        for t in range(20):
            assert hb.hb_tensor_seed(root, t) == oracle.tensor_seed(root, t)


def test_opened_bits_matches_oracle():
    for k in range(0, 64, 3):
        for m in range(k + 1, 65):
            for relu in (0, 1):
                assert hb.hb_opened_bits(relu, k, m, 1000) == oracle.opened_bits(relu, k, m, 1000)
    for (k, m) in [(-1, 3), (4, 4), (9, 2), (0, 65)]:
        assert hb.hb_opened_bits(1, k, m, 10) == 0


def test_strerror_texts():
    assert hb.strerror(0) == "success"
    for st in (-1, -2, -3, -99):
        assert hb.strerror(st)
    assert hb.last_hip_error() == ""


def test_eco_choose_matches_oracle():
    import ctypes
    import numpy as np
    rng = np.random.default_rng(3)
    for _ in range(50):
        c = np.zeros(64, dtype=np.uint64)
        top = int(rng.integers(0, 63))
        c[:top] = rng.integers(0, 5, top)
        arr = (ctypes.c_uint64 * 64)(*[int(v) for v in c])
        assert hb.raw("hb_eco_choose", arr) == oracle.eco_choose(c)
    assert hb.raw("hb_eco_choose", None) == hb.HB_EINVAL
