"""Pins for the exponent-only detection / correction techniques of Sec. VI-A (BoundCheck,
RangeCheck-max, RangeCheck-flip) as the oracle applies them to the erroneous product."""
import os

import numpy as np
import pytest

import np_reference as ref
from oracle import pyoracle as orc
from paper_2311_05782_amd import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))
BF, FP = orc.BF16, orc.FP16


def _rows():
    out = []
    for ln in open(os.path.join(HERE, "golden", "exponent_checks.txt")):
        ln = ln.split("#")[0].split()
        if len(ln) >= 7:
            out.append(ln[:7])
    return out


@pytest.mark.parametrize("row", _rows())
def test_worked_examples(row):
    w_err = int(row[0], 16)
    a, b = 0x3FC0, 0x4000
    for mode, wcol, fcol in ((orc.PCHECK_BOUND, 1, 2), (orc.PCHECK_RANGE_MAX, 3, 4), (orc.PCHECK_RANGE_FLIP, 5, 6)):
        if row[wcol] == "-":
            continue
        assert orc.product_check(w_err, a, b, BF, mode) == (int(row[wcol], 16), int(row[fcol])), (row, mode)
    assert orc.product_check(w_err, a, b, BF, orc.PCHECK_NONE) == (w_err, 0)


def test_bound_check_fires_exactly_from_131072_up_and_confines_the_value():
    # Table IV: exponent 10010000, mantissa 0000000 is 131072, the smallest value the check rejects.
    words = np.arange(65536, dtype=np.uint16)
    vals = orc.decode_array(words, BF)
    for w, v in zip(words.tolist(), vals.tolist()):
        cw, fired = orc.product_check(w, 0, 0, BF, orc.PCHECK_BOUND)
        assert fired == int(not (abs(v) < 131072.0)), hex(w)          # NaN and Inf fire too
        if fired:
            cv = orc.decode16(cw, BF)
            assert abs(cv) < 4.0 * 32768 and abs(cv) >= 2.0           # exponent 1000xxxx: [2, 131072)
            assert (cw & 0x807F) == (w & 0x807F) and ((cw >> 7) & 0x0F) == ((w >> 7) & 0x0F)
        else:
            assert cw == w
    # the table's 261120 -> 3.98438
    assert orc.decode16(0x487F, BF) == 261120.0
    assert abs(orc.decode16(orc.product_check(0x487F, 0, 0, BF, orc.PCHECK_BOUND)[0], BF) - 3.98438) < 5e-6
    # not defined for FP16: never fires
    assert all(orc.product_check(w, 0, 0, FP, orc.PCHECK_BOUND) == (w, 0) for w in range(0, 65536, 97))


@pytest.mark.parametrize("fmt", [FP, BF])
def test_range_check_never_fires_on_a_correct_product(fmt):
    # e_m <= e_1 + e_2 + 1 (Sec. VI-A) holds for every correctly rounded product, including
    # overflow to Inf only when the bound itself is at the top, subnormals and zeros.
    rng = np.random.default_rng(9)
    words = rng.integers(0, 65536, size=(20000, 2)).astype(np.uint16)
    scale = 0x7C00 if fmt == FP else 0x7F80
    for wa, wb in words.tolist():
        if (wa & 0x7FFF) >= scale or (wb & 0x7FFF) >= scale:
            continue
        prod = np.float32(orc.decode16(wa, fmt)) * np.float32(orc.decode16(wb, fmt))
        w = orc.round16(float(prod), fmt)
        for mode in (orc.PCHECK_RANGE_MAX, orc.PCHECK_RANGE_FLIP):
            assert orc.product_check(w, wa, wb, fmt, mode) == (w, 0), (hex(wa), hex(wb), hex(w))


@pytest.mark.parametrize("fmt", [FP, BF])
def test_range_check_corrections_respect_the_bound_and_touch_only_the_exponent(fmt):
    rng = np.random.default_rng(10)
    mb, eb, bias = (10, 5, 15) if fmt == FP else (7, 8, 127)
    emask = (1 << eb) - 1
    for _ in range(20000):
        wa, wb, we = (int(x) for x in rng.integers(0, 65536, 3))
        bound = max(((wa >> mb) & emask) + ((wb >> mb) & emask) - bias + 1, 0)
        e = (we >> mb) & emask
        for mode in (orc.PCHECK_RANGE_MAX, orc.PCHECK_RANGE_FLIP):
            cw, fired = orc.product_check(we, wa, wb, fmt, mode)
            ce = (cw >> mb) & emask
            assert fired == int(e > bound)
            assert (cw & ~(emask << mb)) == (we & ~(emask << mb))
            if not fired:
                assert cw == we
            elif mode == orc.PCHECK_RANGE_MAX:
                assert ce == min(bound, emask)
            else:
                assert ce <= bound and (ce & ~e) == 0                      # only 1s were cleared
                cleared = e & ~ce
                last = 1 << (cleared.bit_length() - 1)                     # the leftmost bit it cleared
                assert cleared == e & (2 * last - 1)                       # every 1 from the right up to it
                assert ce + last > bound                                   # and it stopped as soon as it could


def test_checks_inside_a_trial_confine_the_deviation():
    # Sec. VI-B, Fig. 9: with a technique applied the difference is confined; corrections happen
    # only where detection fired.
    fmt = BF
    M, N, K, kb = 4, 4, 64, 16
    Aw, Bw = wl.gaussian(M, N, K, fmt, seed=77)
    worst = {}
    for mode in (orc.PCHECK_NONE, orc.PCHECK_BOUND, orc.PCHECK_RANGE_MAX, orc.PCHECK_RANGE_FLIP):
        p = orc.problem(M, N, K, kb, fmt, product_check=mode)
        devs, fired = [], 0
        for k in range(K):
            for bit in range(7, 15):                                    # exponent bits of the product
                r = orc.trial(p, Aw, Bw, (orc.SITE_PRODUCT, 1, 2, k, 1 << bit), orc.CORRECT_NONE, orc.MODE_AFFECTED)
                devs.append(float(r["max_dev_pre"]))
                fired += int(r["product_flag"])
                if mode == orc.PCHECK_NONE:
                    assert r["product_flag"] == 0
        worst[mode] = (max(devs), fired)
    assert worst[orc.PCHECK_NONE][0] > 1e30 and worst[orc.PCHECK_NONE][1] == 0
    assert worst[orc.PCHECK_BOUND][0] < 2.0 * 131072 and worst[orc.PCHECK_BOUND][1] > 0
    for mode in (orc.PCHECK_RANGE_MAX, orc.PCHECK_RANGE_FLIP):
        # corrected |re_err| < 2^(e1+e2+2) <= 4 |a| |b| ... bounded by the operands
        assert worst[mode][0] < 64.0 and worst[mode][1] >= worst[orc.PCHECK_BOUND][1]


def test_full_and_affected_modes_agree_with_a_check_enabled():
    fmt = BF
    Aw, Bw = wl.gaussian(3, 3, 32, fmt, seed=78)
    for mode in (orc.PCHECK_BOUND, orc.PCHECK_RANGE_MAX, orc.PCHECK_RANGE_FLIP):
        p = orc.problem(3, 3, 32, 16, fmt, product_check=mode)
        for k in (0, 15, 16, 31):
            for mask in (0x4000, 0x2000, 0x0080, 0x7F80):
                f = (orc.SITE_PRODUCT, 2, 0, k, mask)
                a = orc.trial(p, Aw, Bw, f, orc.CORRECT_ZERO, orc.MODE_AFFECTED)
                b = orc.trial(p, Aw, Bw, f, orc.CORRECT_ZERO, orc.MODE_FULL)
                for name in a.dtype.names:
                    assert a[name] == b[name] or (np.isnan(a[name]) and np.isnan(b[name])), (name, f, mode)
