"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and its host-side
logic (sizes, validation, error strings) behaves; no kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lpc():
    from paper_1901_08924_amd import lpc as mod
    return mod


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "lpc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lpc_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lpc):
    names = _declared_functions()
    assert len(names) >= 15
    for name in names:
        assert hasattr(lpc.lib, name), name
    assert sorted(lpc.EXPORTS) == names      # the binding covers exactly the header


def test_no_oracle_in_the_product_path():
    # the package must not import, link or read anything under oracle/
    pkg = os.path.join(ROOT, "paper_1901_08924_amd")
    for dirpath, _dirs, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "lpco" not in text and "oracle" not in text.lower(), os.path.join(dirpath, f)


def test_sizes_and_strings(lpc):
    assert lpc.d_pad(1) == 32 and lpc.d_pad(64) == 64 and lpc.d_pad(65) == 96
    assert lpc.words_per_msg(64, 2) == 4 and lpc.words_per_msg(4096, 4) == 512 and lpc.words_per_msg(33, 3) == 6
    for code in (0, -1, -2, -3, -4, -5, -6, -7):
        assert len(lpc.lib.lpc_status_string(code)) > 0
    # message size of Sec. 4.2: b*d_pad code bits in the buffer, the 32-bit scale factor beside it
    assert lpc.words_per_msg(4096, 4) * 32 + 32 == 32 + 4 * 4096


def _problem(lpc, n=1024, d=64, X=0x1000, y=0x2000):
    p = lpc.Problem()
    p.n, p.d, p.loss, p.X, p.ldx, p.y = n, d, lpc.LOSS_LOGISTIC, X, d, y
    return p


def test_workspace_size_grows_with_the_problem(lpc):
    small = lpc.lib.lpc_workspace_bytes(C.byref(_problem(lpc)), C.byref(lpc.make_config(N=4, B=16, m=16, bits=2)))
    big = lpc.lib.lpc_workspace_bytes(C.byref(_problem(lpc, n=65536, d=4096)),
                                      C.byref(lpc.make_config(N=8, B=64, m=128, bits=4)))
    assert 0 < small < big
    # at least U (N+1 rows), the messages and the cached margins must fit
    assert big >= 9 * 4096 * 4 + 8 * 512 * 4 + 65536 * 4


@pytest.mark.parametrize("field,value,code", [
    ("bits", 1, -1),      # 2^(b-1)-1 = 0 in eq. (3)
    ("bits", 0, -1), ("bits", 17, -1), ("bits", 31, -1),
    ("N", 0, -1), ("B", 0, -1), ("m", 0, -1),
    ("B", 1024, -1),      # N*B > n contradicts Theorem 1's N*B <= n
    ("clip", 0.0, -1), ("clip", 1.5, -1),   # lambda in (0,1]
    ("eta", 0.0, -1), ("clip_mode", 7, -1), ("algo", 9, -1), ("scheme", 5, -1),
])
def test_create_rejects_bad_config(lpc, field, value, code):
    cfg = lpc.make_config(N=4, B=16, m=16, bits=2)
    setattr(cfg, field, value)
    handle = C.c_void_p()
    rc = lpc.lib.lpc_create(C.byref(handle), C.byref(_problem(lpc)), C.byref(cfg), 0x10000, 1 << 30)
    assert rc == code and not handle.value
    assert lpc.lib.lpc_workspace_bytes(C.byref(_problem(lpc)), C.byref(cfg)) == 0


def test_create_rejects_bad_problem_and_workspace(lpc):
    cfg = lpc.make_config(N=4, B=16, m=16, bits=2)
    handle = C.c_void_p()
    assert lpc.lib.lpc_create(C.byref(handle), None, C.byref(cfg), 0x10000, 1 << 30) == lpc.ENULL
    assert lpc.lib.lpc_create(C.byref(handle), C.byref(_problem(lpc, y=0)), C.byref(cfg), 0x10000, 1 << 30) == lpc.ENULL
    assert lpc.lib.lpc_create(C.byref(handle), C.byref(_problem(lpc, n=0)), C.byref(cfg), 0x10000, 1 << 30) == lpc.ESHAPE
    p = _problem(lpc)
    p.ldx = 32                                              # leading dimension shorter than a row
    assert lpc.lib.lpc_create(C.byref(handle), C.byref(p), C.byref(cfg), 0x10000, 1 << 30) == lpc.ESHAPE
    p = _problem(lpc)
    p.lambda1 = -1.0
    assert lpc.lib.lpc_create(C.byref(handle), C.byref(p), C.byref(cfg), 0x10000, 1 << 30) == lpc.EINVAL
    good = _problem(lpc)
    assert lpc.lib.lpc_create(C.byref(handle), C.byref(good), C.byref(cfg), None, 1 << 30) == lpc.EWORKSPACE
    assert lpc.lib.lpc_create(C.byref(handle), C.byref(good), C.byref(cfg), 0x10000, 16) == lpc.EWORKSPACE
    assert lpc.lib.lpc_create(C.byref(handle), C.byref(good), C.byref(cfg), 0x10001, 1 << 30) == lpc.EWORKSPACE
    alpc = lpc.make_config(algo=lpc.ALGO_ALPC_SC, N=4, B=16, m=16, bits=2)     # ALPC needs L
    assert lpc.lib.lpc_create(C.byref(handle), C.byref(good), C.byref(alpc), 0x10000, 1 << 30) == lpc.EINVAL


def test_calls_reject_null_handles(lpc):
    assert lpc.lib.lpc_full_grad(None, None, None, None, None, None) == lpc.ENULL
    assert lpc.lib.lpc_epoch(None, None, None, None, 0, None) == lpc.ENULL
    assert lpc.lib.lpc_prox_step(None, None, None, None, 0.1, None) == lpc.ENULL
    out = C.c_double()
    assert lpc.lib.lpc_objective(None, None, C.byref(out), None) == lpc.ENULL


def test_theorem2_and_huffman_host_entry_points():
    """Host arithmetic inside the HIP library (no GPU needed): eq. (6)/(7) and optimal prefix-code sizes."""
    from fractions import Fraction
    from paper_1901_08924_amd import lpc
    exact = Fraction(8 * 4, 100) * (Fraction(64, 4 * 49) + Fraction(1, 64)) + Fraction(1, 10)
    assert abs(lpc.theorem2_lhs(64, 4, 1.0, 0, 4, 16, 2, 0.1, lpc.SCHEME_A) - float(exact)) < 1e-12
    exact_c = Fraction(8 * 4, 100) * (Fraction(3 * 64, 8 * 49) + Fraction(1, 64)) + Fraction(1, 10)
    assert abs(lpc.theorem2_lhs(64, 4, 1.0, 0, 4, 16, 2, 0.1, lpc.SCHEME_C) - float(exact_c)) < 1e-12
    exact_l = Fraction(8 * 4, 100) * (Fraction(64, 4 * 49) / 4 + Fraction(3, 4) + Fraction(1, 64)) + Fraction(1, 10)
    assert abs(lpc.theorem2_lhs(64, 4, 0.5, 3, 4, 16, 2, 0.1, lpc.SCHEME_B) - float(exact_l)) < 1e-12
    with pytest.raises(lpc.LpcError):
        lpc.theorem2_lhs(64, 1, 1.0, 0, 4, 16, 2, 0.1, lpc.SCHEME_A)
    bits, lens = lpc.huffman_bits([45, 13, 12, 16, 9, 5])
    assert bits == 224 and sorted(lens) == [1, 3, 3, 3, 4, 4]
    assert lpc.huffman_bits([0, 9, 0]) == (9, [0, 1, 0])
    assert lpc.huffman_bits([0, 0]) == (0, [0, 0])
    bits, lens = lpc.huffman_bits([3] * 8)
    assert bits == 72 and lens == [3] * 8


def test_table1_bits_per_iteration(lpc):
    """lpc_bits_per_iteration against the values worked out by hand from Table 1's formulas (tests/golden)."""
    with open(os.path.join(ROOT, "tests", "golden", "table1_bits.txt")) as f:
        rows = [[int(t) for t in line.split()] for line in f if line.strip() and not line.startswith("#")]
    assert len(rows) >= 4
    for d, b, N, bits_a, bits_b, bits_c, _msg in rows:
        assert lpc.bits_per_iteration(d, b, N, lpc.SCHEME_A) == bits_a
        assert lpc.bits_per_iteration(d, b, N, lpc.SCHEME_B) == bits_b
        assert lpc.bits_per_iteration(d, b, N, lpc.SCHEME_C) == bits_c
    assert lpc.bits_per_iteration(20, 32, 4) == 32 * 20 * 4 * 3
    for bad in ((10, 1, 4, 0), (10, 17, 4, 0), (10, 4, 0, 0), (10, 4, 4, 3)):
        with pytest.raises(lpc.LpcError):
            lpc.bits_per_iteration(*bad)
