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


def test_e4m3_encoder_matches_the_library_conversion_bit_for_bit(sp):
    """The fp8 weight loader's float32 -> e4m3 rounding (host code) against torch's float8_e4m3fn conversion: every
    code exactly, on a dense sweep of the whole finite range including the subnormal codes, exact ties, both signs
    and the saturation point (the loader never produces magnitudes above 448: it scales each row so that its largest
    weight is 448)."""
    import numpy as np
    import torch
    rng = np.random.default_rng(5)
    codes = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy()
    finite = np.sort(codes[np.isfinite(codes)])
    mids = (finite[1:] + finite[:-1]) / 2                      # exact ties between neighbouring codes
    x = np.concatenate([finite, mids, np.nextafter(mids, np.inf).astype(np.float32),
                        np.nextafter(mids, -np.inf).astype(np.float32),
                        rng.uniform(-448, 448, 200_000), rng.normal(0, 1, 200_000), rng.normal(0, 0.01, 100_000),
                        rng.uniform(-2.0 ** -6, 2.0 ** -6, 100_000), [0.0, -0.0, 448.0, -448.0, 2.0 ** -9, 2.0 ** -10,
                                                                       1.5 * 2.0 ** -10, 2.0 ** -11]]).astype(np.float32)
    got = sp.sp_probe_e4m3(x)
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    bad = np.flatnonzero(got != want)
    # (-0.0 and +0.0: both conversions keep the sign bit)
    assert bad.size == 0, f"{bad.size} codes differ, first at x = {x[bad[0]]!r}: {got[bad[0]]:#x} vs {want[bad[0]]:#x}"
    assert sp.sp_probe_e4m3(np.array([1e9, -1e9, 464.0], np.float32)).tolist() == [0x7e, 0xfe, 0x7e]   # saturating


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits (before anything touches a GPU)."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
