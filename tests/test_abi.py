"""CPU-side checks of the C ABI: the library loads, exports every declared symbol, and rejects bad
arguments on the host before anything is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2310_14997_amd import binding as bd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "spcfg.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spcfg_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = bd.load()
    names = declared_symbols()
    assert {"spcfg_inside", "spcfg_inside_backward", "spcfg_workspace_bytes", "spcfg_strerror"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/spcfg.h but not exported"


def test_strerror_is_total():
    lib = bd.load()
    for code in range(-8, 2):
        assert isinstance(lib.spcfg_strerror(code), bytes) and len(lib.spcfg_strerror(code)) > 0


def test_workspace_query_and_monotonicity():
    cfg = bd.make_config(30, 60, 4, 10)
    exact = bd.spcfg_workspace_bytes_for(cfg, [10, 10, 10, 10], 10)
    assert 0 < exact <= bd.spcfg_workspace_bytes(cfg)
    assert bd.spcfg_workspace_bytes_for(cfg, [2, 3, 10, 4], 10) < exact
    big = bd.make_config(2048, 2048, 64, 40)
    assert bd.spcfg_workspace_bytes(big) < 8 << 30


@pytest.mark.parametrize("kwargs,code", [
    (dict(N=0), -2), (dict(P=0), -2), (dict(max_B=0), -2), (dict(max_B=5000), -2), (dict(max_n=1), -2),
    (dict(precision=7), -5), (dict(flags=64), -5), (dict(flags=16), -5),
])
def test_bad_config_is_rejected(kwargs, code):
    base = dict(N=8, P=8, max_B=2, max_n=6, precision=0, flags=0)
    base.update(kwargs)
    cfg = bd.make_config(**base)
    with pytest.raises(bd.SpcfgError) as e:
        bd.spcfg_workspace_bytes(cfg)
    assert e.value.code == code


def test_every_documented_flag_is_accepted():
    for flags in (0, bd.FLAG_ACCUMULATE_GRADS, bd.FLAG_PER_SENTENCE_GRAMMAR, bd.FLAG_FP32_MFMA,
                  bd.FLAG_BF16_SINGLE_FORWARD,
                  bd.FLAG_ACCUMULATE_GRADS | bd.FLAG_PER_SENTENCE_GRAMMAR | bd.FLAG_FP32_MFMA | bd.FLAG_BF16_SINGLE_FORWARD):
        for precision in (bd.PRECISION_FP32, bd.PRECISION_BF16):
            cfg = bd.make_config(8, 8, 2, 6, precision, flags)
            assert bd.spcfg_workspace_bytes(cfg) > 0


def test_bad_struct_size_and_lengths():
    cfg = bd.make_config(8, 8, 4, 6)
    for lens, n_max, code in [([1, 3], 6, -3), ([7, 3], 6, -3), ([3, 3], 9, -2), ([3] * 5, 6, -2)]:
        with pytest.raises(bd.SpcfgError) as e:
            bd.spcfg_workspace_bytes_for(cfg, lens, n_max)
        assert e.value.code == code
    cfg.struct_size = 4
    with pytest.raises(bd.SpcfgError) as e:
        bd.spcfg_workspace_bytes(cfg)
    assert e.value.code == -1


def test_null_pointers_are_rejected_before_any_launch():
    lib = bd.load()
    cfg = bd.make_config(8, 8, 2, 6)
    lens = np.array([3, 4], dtype=np.int32)
    rc = lib.spcfg_inside(C.byref(cfg), None, None, None, None, lens.ctypes.data, 2, 6, None, None, 0, None)
    assert rc == -1
    # non-null (never dereferenced) data pointers, null workspace -> argument error; tiny workspace -> workspace error
    fake = C.c_void_p(4096)
    rc = lib.spcfg_inside(C.byref(cfg), fake, fake, fake, fake, lens.ctypes.data, 2, 6, fake, None, 0, None)
    assert rc == -1
    rc = lib.spcfg_inside(C.byref(cfg), fake, fake, fake, fake, lens.ctypes.data, 2, 6, fake, C.c_void_p(256), 16, None)
    assert rc == -4
    rc = lib.spcfg_inside(C.byref(cfg), fake, fake, fake, fake, lens.ctypes.data, 2, 6, fake, C.c_void_p(100), 1 << 40, None)
    assert rc == -4  # misaligned


def test_static_scratch_entry_point_checks_its_arguments_on_the_host():
    """spcfg_inside_static refuses bad arguments and batches beyond its static buffer before anything is launched."""
    lib = bd.load()
    fake = C.c_void_p(4096)
    cfg = bd.make_config(8, 8, 2, 6)
    lens = np.array([3, 4], dtype=np.int32)
    assert lib.spcfg_inside_static(C.byref(cfg), None, fake, fake, fake, lens.ctypes.data, 2, 6, fake, None) == -1
    bad = np.array([1, 4], dtype=np.int32)
    assert lib.spcfg_inside_static(C.byref(cfg), fake, fake, fake, fake, bad.ctypes.data, 2, 6, fake, None) == -3
    big = bd.make_config(2048, 2048, 64, 40)
    full = np.full(64, 40, dtype=np.int32)
    assert lib.spcfg_inside_static(C.byref(big), fake, fake, fake, fake, full.ctypes.data, 64, 40, fake, None) == -7
    assert b"static" in lib.spcfg_strerror(-7)


def test_decode_argument_checks_run_before_any_launch():
    lib = bd.load()
    fake = C.c_void_p(4096)
    lens = np.array([3, 4], dtype=np.int32)
    out = C.c_size_t(0)
    assert lib.spcfg_mbr_decode_scratch_bytes(2, 6, C.byref(out)) == 0 and out.value == 2 * 36 * 12
    assert lib.spcfg_mbr_decode_scratch_bytes(2, 1, C.byref(out)) == -2
    assert lib.spcfg_mbr_decode_scratch_bytes(961, 6, C.byref(out)) == -2
    assert lib.spcfg_mbr_decode_scratch_bytes(2, 6, None) == -1
    assert lib.spcfg_mbr_decode(None, lens.ctypes.data, 2, 6, fake, fake, fake, 1 << 20, None) == -1
    assert lib.spcfg_mbr_decode(fake, lens.ctypes.data, 2, 6, fake, fake, fake, 16, None) == -4
    assert lib.spcfg_mbr_decode(fake, lens.ctypes.data, 2, 6, fake, fake, C.c_void_p(4100), 1 << 20, None) == -4
    bad = np.array([3, 7], dtype=np.int32)
    assert lib.spcfg_mbr_decode(fake, bad.ctypes.data, 2, 6, fake, fake, fake, 1 << 20, None) == -3
    cfg = bd.make_config(8, 8, 2, 6)
    assert lib.spcfg_span_marginals(C.byref(cfg), lens.ctypes.data, 2, 6, fake, 1 << 30, None, None, None) == -1
    assert lib.spcfg_span_marginals(C.byref(cfg), lens.ctypes.data, 2, 6, C.c_void_p(4096), 16, fake, None, None) == -4


def test_header_is_valid_c99_and_cpp():
    """The boundary is a C ABI: the header must compile as plain C (and as C++) on its own."""
    import subprocess
    import tempfile
    hdr = os.path.join(ROOT, "include", "spcfg.h")
    with tempfile.TemporaryDirectory() as tmp:
        src = os.path.join(tmp, "t.c")
        with open(src, "w") as f:
            f.write(f'#include "{hdr}"\nint main(void) {{ spcfg_config c; c.struct_size = sizeof c; return (int)c.struct_size == 0; }}\n')
        subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-fsyntax-only", src])
        subprocess.check_call(["g++", "-std=c++11", "-Wall", "-Werror", "-x", "c++", "-fsyntax-only", src])
