"""Pins for the bound check of Sec. VI-A used as an output-side detector on binary32 words
(exponent 1eeexxxx with a 1 among eee; Table IV: every such value is at least 131072)."""
import numpy as np

from oracle import pyoracle as orc
from paper_2311_05782_amd import workloads as wl


def pattern_fires(words):
    """The rule as the paper words it, on the 8-bit exponent field of each word."""
    e = (np.asarray(words, np.uint32) >> 23) & 0xFF
    return ((e & 0x80) != 0) & ((e & 0x70) != 0)


def test_fires_on_exactly_the_exponent_pattern_over_every_exponent_sign_and_mantissa_edge():
    M, N, K, kb = 32, 48, 32, 16
    p = orc.problem(M, N, K, kb, orc.BF16, bound_mode=orc.BOUND_EXPONENT)
    words = []
    for sign in (0, 1):
        for e in range(256):
            for man in (0, 1, 0x7FFFFF):
                words.append((sign << 31) | (e << 23) | man)
    words = np.array(words, np.uint32)
    assert words.size == M * N
    ra = np.zeros(M, np.float32); cb = np.zeros(N, np.float32)     # no operand statistics are used
    out, flags, n = orc.detect_correct(p, ra, cb, words.view(np.float32).reshape(1, M, N), orc.CORRECT_ZERO)
    want = pattern_fires(words)
    assert np.array_equal(flags.reshape(-1).astype(bool), want) and int(n[0]) == int(want.sum())
    # Inf and NaN carry the pattern; the smallest flagged magnitude is Table IV's 131072
    mags = np.abs(words.view(np.float32)[want & np.isfinite(words.view(np.float32))])
    assert mags.min() == 131072.0
    assert np.abs(words.view(np.float32)[~want]).max() == np.nextafter(np.float32(131072.0), np.float32(0))
    assert np.all(out.reshape(-1).view(np.uint32)[want] == 0)
    assert np.array_equal(out.reshape(-1).view(np.uint32)[~want], words[~want])


def test_in_a_trial_the_last_block_flip_is_flagged_by_its_exponent_alone():
    # a fault after the last k-block leaves word(C*) XOR mask in the output: the flag is then a
    # function of that word only, whatever the operands are.
    M, N, K, kb = 4, 4, 64, 32
    Aw, Bw = wl.gaussian(M, N, K, orc.FP16, seed=12)
    p = orc.problem(M, N, K, kb, orc.FP16, bound_mode=orc.BOUND_EXPONENT)
    cstar = orc.gemm(p, Aw, Bw).view(np.uint32)
    for (i, j) in ((0, 0), (3, 2)):
        for bit in range(32):
            rec, cf, cc = orc.trial(p, Aw, Bw, (orc.SITE_ACC, i, j, K // kb - 1, 1 << bit), orc.CORRECT_ZERO,
                                    want_outputs=True)
            w = int(cstar[i, j]) ^ (1 << bit)
            assert int(cf.view(np.uint32)[i, j]) == w == int(rec["site_word_after"])
            assert int(rec["n_flagged"]) == int(pattern_fires([w])[0]), (i, j, bit, hex(w))
            assert int(rec["cls"]) == (orc.DETECTED if pattern_fires([w])[0] else
                                       (orc.SDC if int(rec["n_dev_pre"]) else orc.MASKED))


def test_coverage_is_a_subset_of_the_magnitude_bound_when_every_threshold_is_below_2_pow_17():
    M, N, K, kb = 16, 16, 128, 32
    Aw, Bw = wl.gaussian(M, N, K, orc.BF16, seed=13)
    pm = orc.problem(M, N, K, kb, orc.BF16)
    pe = orc.problem(M, N, K, kb, orc.BF16, bound_mode=orc.BOUND_EXPONENT)
    ra, cb, _ = orc.rowcol_absmax(pm, Aw, Bw)
    assert float(K * ra.max() * cb.max()) * 1.001 < 2.0 ** 17
    faults = orc.sample_faults(3, 0, 600, pm, orc.KIND_ALL_ACC, 1)
    rm = orc.campaign(pm, Aw, Bw, faults, orc.CORRECT_ZERO)
    re = orc.campaign(pe, Aw, Bw, faults, orc.CORRECT_ZERO)
    fm, fe = rm["n_flagged"] > 0, re["n_flagged"] > 0
    assert np.all(fm[fe]) and fe.sum() > 0 and fm.sum() > fe.sum()
    # what the exponent rule misses and the magnitude bound catches lies between T and 2^17
    missed = fm & ~fe
    assert np.all(rm["max_dev_pre"][missed] < 2.0 ** 17 + float(K * ra.max() * cb.max()))
    # no false positive on fault-free trials
    none = orc.make_faults([(orc.SITE_NONE, 0, 0, 0, 0)] * 3)
    assert np.all(orc.campaign(pe, Aw, Bw, none, orc.CORRECT_ZERO)["cls"] == orc.MASKED)
