"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and its host logic (packing, size queries, argument
errors) behaves as documented."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2408_12526_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sp():
    from paper_2408_12526_amd import sp as binding
    return binding


def declared_symbols():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if header.endswith(".h"):
            text = open(os.path.join(ROOT, "include", header)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(sp_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol(sp):
    names = declared_symbols()
    assert {"sp_load_students", "sp_forward", "sp_pack", "sp_free", "sp_strerror", "sp_arena_bytes",
            "sp_workspace_bytes", "sp_blob_floats", "sp_workspace_layout", "sp_forward_partial", "sp_lab_create",
            "sp_lab_push", "sp_lab_pop", "sp_ctl_create", "sp_ctl_on_buffered", "sp_ctl_on_tick",
            "sp_dispatch_simulate"} <= set(names)
    lib = sp.raw_lib()
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/ but not exported"


def test_pack_matches_oracle_bit_for_bit(sp, oracle64):
    rng = np.random.default_rng(0)
    for B in (1, 2, 31, 256, 1000):
        lengths = rng.integers(1, 513, size=B).astype(np.int32)
        got = sp.sp_pack(lengths)
        assert got.dtype == np.int32 and np.array_equal(got, oracle64.pack(lengths))
    assert sp.sp_pack([512]).tolist() == [0, 512]
    assert sp.sp_pack([7] * 5).tolist() == [0, 7, 14, 21, 28, 35]


def test_pack_rejects_bad_lengths(sp):
    with pytest.raises(sp.SpError) as e:
        sp.sp_pack([4, 0, 2])
    assert e.value.code == -2
    with pytest.raises(sp.SpError):
        sp.sp_pack([2**31 - 1, 2**31 - 1])


def test_size_queries(sp):
    for n, w in synth.WORKLOADS.items():
        cfg = sp.config_from_shape(w.shape)
        assert sp.sp_blob_floats(cfg) == synth.blob_floats(w.shape)
        elem = 2 if w.shape.dtype == "bf16" else 4
        assert sp.sp_arena_bytes(cfg) >= synth.blob_floats(w.shape) * elem * 0.99
        a, b = sp.sp_workspace_bytes(cfg, 100, 4), sp.sp_workspace_bytes(cfg, 5000, 64)
        assert 0 < a <= b
        lay = sp.sp_workspace_layout(cfg, 300, 3)
        assert lay.rows >= 300 and lay.rows % 64 == 0 and lay.act_bytes == elem
    bad = sp.make_config(0, 2, 128, 2, 512, 100, 64, 2)
    assert sp.sp_blob_floats(bad) == 0 and sp.sp_arena_bytes(bad) == 0


def test_argument_errors_without_touching_a_gpu(sp):
    lib = sp.raw_lib()
    assert lib.sp_forward(None, None, None, 1, 1, 1, 1, None, 0, None, None) == -1
    cfg = sp.config_from_shape(synth.WORKLOADS[1].shape)
    out = C.c_void_p()
    assert lib.sp_load_students(C.byref(cfg), None, 0, None, 0, None, C.byref(out)) == -1
    assert b"k_active" in lib.sp_strerror(-3)
    assert lib.sp_strerror(-99) is not None
