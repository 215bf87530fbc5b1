"""Pins for the oracle's operand decoding (Sec. II-A, Fig. 1; Table IV; Sec. V-B)."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import pyoracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_table_iv_values():
    # Every printed value of Table IV, to the digits the paper prints.
    for e, m, printed in _rows("table_iv_bf16.txt"):
        w = (int(e, 2) << 7) | int(m, 2)
        got = orc.decode16(w, orc.BF16)
        want = float(printed)
        digits = len(printed.split("e")[0].replace(".", "").lstrip("0")) if "e" in printed else 6
        assert abs(got - want) <= abs(want) * 10.0 ** (1 - digits), (e, m, got, want)
    # BoundCheck threshold: exponent 10010000 with zero mantissa is exactly 2^17.
    assert orc.decode16(0b0100100000000000, orc.BF16) == 131072.0


def test_subnormal_examples():
    for fmt, pat, printed in _rows("subnormal_examples.txt"):
        got = orc.decode16(int(pat, 2), orc.FP16 if fmt == "fp16" else orc.BF16)
        if fmt == "fp16":
            assert got == 2.0 ** -15
            assert round(got, 8) == float(printed)
        else:
            assert got == 2.0 ** -127 == float(printed)


def _closed_form(w, ebits, mbits):
    """(-1)^s 2^(E-bias) (1+m/2^p), subnormal 2^(1-bias) m/2^p, as exact fractions."""
    bias = (1 << (ebits - 1)) - 1
    s = w >> 15
    E = (w >> mbits) & ((1 << ebits) - 1)
    m = w & ((1 << mbits) - 1)
    if E == (1 << ebits) - 1:
        return None if m else (Fraction(-1) if s else Fraction(1), "inf")
    if E == 0:
        v = Fraction(m, 1 << mbits) * Fraction(2) ** (1 - bias)
    else:
        v = (1 + Fraction(m, 1 << mbits)) * Fraction(2) ** (E - bias)
    return -v if s else v


@pytest.mark.parametrize("fmt,ebits,mbits", [(orc.FP16, 5, 10), (orc.BF16, 8, 7)])
def test_all_patterns_closed_form_and_library(fmt, ebits, mbits):
    words = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = orc.decode_array(words, fmt)
    # library routine / format identity
    if fmt == orc.FP16:
        lib = words.view(np.float16).astype(np.float32)
    else:
        lib = (words.astype(np.uint32) << 16).view(np.float32)
    nan = np.isnan(lib)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), lib[~nan].view(np.uint32))
    # closed form on a stride of patterns plus all the edge exponents
    probe = list(range(0, 65536, 101)) + [0, 1, 0x8000, 0x8001, 0x03FF, 0x0400, 0x007F, 0x0080,
                                          0x7BFF, 0x7C00, 0xFC00, 0x7F7F, 0x7F80, 0xFF80]
    for w in probe:
        cf = _closed_form(w, ebits, mbits)
        g = float(got[w])
        if cf is None:
            assert np.isnan(g)
        elif isinstance(cf, tuple):
            assert np.isinf(g) and (g > 0) == (cf[0] > 0)
        else:
            assert Fraction(g) == cf, (hex(w), g, cf)
    # sign of zero is kept
    assert np.signbit(got[0x8000]) and not np.signbit(got[0])


def test_input_rounding_helpers_match_library():
    from paper_2311_05782_amd import workloads as wl
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(4096).astype(np.float32) * np.float32(s)
                        for s in (1e-8, 1e-3, 1.0, 300.0)])
    # ties and edge cases for bf16: exactly halfway patterns
    ties = (np.array([0x3F808000, 0x3F818000, 0x3F807FFF, 0x3F808001, 0x00008000, 0x7F7F7FFF],
                     np.uint32)).view(np.float32)
    x = np.concatenate([x, ties])
    w = wl.to_bf16_words(x)
    back = orc.decode_array(w, orc.BF16)
    # RNE: the decoded value is the nearest bf16, ties to even mantissa
    n = len(x) - len(ties)          # the random part: all normal, far from the format's ends
    up = ((w[:n].astype(np.uint32) + 1) << 16).view(np.float32)
    dn = ((w[:n].astype(np.uint32) - 1) << 16).view(np.float32)
    err = np.abs(back[:n].astype(np.float64) - x[:n])
    assert np.all(err <= np.abs(up.astype(np.float64) - x[:n]))
    assert np.all(err <= np.abs(dn.astype(np.float64) - x[:n]))
    assert w[-6] == 0x3F80 and w[-5] == 0x3F82 and w[-4] == 0x3F80 and w[-3] == 0x3F81
    # fp16 goes through NumPy's own conversion; decoding it again is the identity on fp16 values
    w16 = wl.to_fp16_words(x[:-1])
    assert np.array_equal(orc.decode_array(w16, orc.FP16).view(np.uint32),
                          x[:-1].astype(np.float16).astype(np.float32).view(np.uint32))
