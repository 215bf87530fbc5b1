"""Pins for the oracle's product-term fault (the paper's own fault model: Sec. III-E write-back,
Eq. 1-2; Sec. IV-A one term of one 16-term MMA step; Sec. IV-C a bit flip in the result of a
multiplication) and for the conversion that holds a product in the operand format."""
import itertools
import os

import numpy as np
import pytest

import np_reference as ref
from oracle import pyoracle as orc
from paper_2311_05782_amd import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))
FIELDS = ("n_flagged", "n_bitdiff", "n_dev_pre", "n_dev_post", "site_word_before", "site_word_after", "cls")


def _f32(words):
    return np.asarray(words, np.uint32).view(np.float32)


def _same_fields(got, want, ctx):
    """Integer fields equal; a NaN site word is compared as "is a NaN" (payloads are not defined)."""
    for name in FIELDS:
        g, w = int(got[name]), int(want[name])
        if name == "site_word_after" and np.isnan(_f32([g])[0]) and np.isnan(_f32([w])[0]):
            continue
        assert g == w, (name, ctx)


# ------------------------------------------------------------ round to the operand format

def test_round16_is_the_identity_on_every_representable_value():
    for fmt in (orc.FP16, orc.BF16):
        words = np.arange(65536, dtype=np.uint16)
        vals = orc.decode_array(words, fmt)
        for w, v in zip(words.tolist(), vals.tolist()):
            if np.isnan(v):
                assert np.isnan(orc.decode16(orc.round16(v, fmt), fmt))
            else:
                assert orc.round16(v, fmt) == w, (fmt, hex(w))


def test_round16_fp16_equals_numpy_conversion_on_midpoints_and_random_values():
    rng = np.random.default_rng(5)
    xs = [0.0, -0.0, 65504.0, 65519.99, 65520.0, 65536.0, 1e9, -1e9, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.5,
          2.0 ** -26, 2.0 ** -14, np.nextafter(np.float32(2.0 ** -14), np.float32(0)), np.inf, -np.inf]
    # every midpoint between neighbouring FP16 values (ties must go to the even word)
    pos = np.arange(0, 0x7C00, dtype=np.uint16)
    v = pos.view(np.float16).astype(np.float64)
    nxt = np.append(v[1:], 65536.0)
    xs += ((v + nxt) / 2).astype(np.float32).tolist()
    xs += (rng.standard_normal(4000) * 10.0 ** rng.uniform(-9, 6, 4000)).astype(np.float32).tolist()
    xs = np.array(xs, np.float32)
    with np.errstate(all="ignore"):
        want = xs.astype(np.float16).view(np.uint16)
    for x, w in zip(xs.tolist(), want.tolist()):
        assert orc.round16(x, orc.FP16) == w, (x, hex(w), hex(orc.round16(x, orc.FP16)))


def test_round16_bf16_picks_the_nearest_value_ties_to_even():
    rng = np.random.default_rng(6)
    xs = (rng.standard_normal(3000) * 10.0 ** rng.uniform(-38, 38, 3000)).astype(np.float32)
    # exact midpoints: a BF16 word followed by 0x8000 in the dropped half
    mids = ((rng.integers(0, 0x7F7F, 500).astype(np.uint32) << 16) | 0x8000).view(np.float32)
    for x in np.concatenate([xs, mids, -mids]).tolist():
        if not np.isfinite(x):
            continue
        got = orc.round16(x, orc.BF16)
        sign = got & 0x8000
        mag = abs(np.float64(x))
        lo = (np.array([abs(np.float32(x))], np.float32).view(np.uint32)[0] >> 16)      # truncation
        cands = [int(lo), int(lo) + 1]
        vals = [np.float64(_f32([c << 16])[0]) for c in cands]                            # Inf for 0x7F80
        d = [abs(mag - val) if np.isfinite(val) else (abs(mag - 2.0 ** 128)) for val in vals]
        best = cands[0] if d[0] < d[1] else cands[1] if d[1] < d[0] else (cands[0] if cands[0] % 2 == 0 else cands[1])
        assert got == (sign | best), (x, hex(got), hex(best))
    assert orc.round16(np.inf, orc.BF16) == 0x7F80 and orc.round16(3.4e38, orc.BF16) == 0x7F80
    assert orc.round16(-0.0, orc.BF16) == 0x8000


# ------------------------------------------------------------ the write-back, by hand

def _golden_rows():
    rows = []
    for ln in open(os.path.join(HERE, "golden", "writeback_examples.txt")):
        if ln.startswith("#") or not ln.strip():
            continue
        fmt, a0, b0, mask, re_w, err_w, final = ln.split()
        rows.append((orc.FP16 if fmt == "fp16" else orc.BF16, float(a0), float(b0), int(mask, 16), int(re_w, 16),
                     int(err_w, 16), float(final)))
    return rows


@pytest.mark.parametrize("row", _golden_rows())
def test_write_back_examples_worked_by_hand(row):
    fmt, a0, b0, mask, re_w, err_w, final = row
    a = np.ones((1, 16), np.float32); a[0, 0] = a0
    b = np.ones((1, 16), np.float32); b[0, 0] = b0
    Aw, Bw = wl.to_words(a, fmt), wl.to_words(b, fmt)
    p = orc.problem(1, 1, 16, 16, fmt)
    assert orc.round16(a0 * b0, fmt) == re_w and re_w ^ mask == err_w
    rec, cf, cc = orc.trial(p, Aw, Bw, (orc.SITE_PRODUCT, 0, 0, 0, mask), orc.CORRECT_NONE, orc.MODE_FULL,
                            want_outputs=True)
    assert float(cf[0, 0]) == final
    re_sum = np.float32(a0 * b0)
    for _ in range(15):
        re_sum = np.float32(re_sum + np.float32(1.0))
    assert _f32([rec["site_word_before"]])[0] == re_sum
    assert _f32([rec["site_word_after"]])[0] == np.float32(final)
    # Sec. V-B: a trial whose destination register ends up unchanged has a site word that does not change
    assert (rec["site_word_before"] == rec["site_word_after"]) == (np.float32(final) == re_sum)


def test_fault_acts_after_the_step_that_holds_the_term_and_later_steps_accumulate_on_it():
    # K = 48 = three steps of 16; all products are 1 except the faulted one (2*4 = 8, k = 20).
    fmt = orc.BF16
    a = np.ones((1, 48), np.float32); a[0, 20] = 2
    b = np.ones((1, 48), np.float32); b[0, 20] = 4
    Aw, Bw = wl.to_words(a, fmt), wl.to_words(b, fmt)
    for kb in (16, 48):
        p = orc.problem(1, 1, 48, kb, fmt)
        # 8.0 = 0x4100; flipping exponent bit 7 (mask 0x0080) gives 0x4180 = 16.0
        rec, cf, _ = orc.trial(p, Aw, Bw, (orc.SITE_PRODUCT, 0, 0, 20, 0x0080), orc.CORRECT_NONE, orc.MODE_FULL,
                               want_outputs=True)
        assert _f32([rec["site_word_before"]])[0] == 16 + 15 + 8      # after the second step
        assert _f32([rec["site_word_after"]])[0] == 16 + 15 + 16
        assert float(cf[0, 0]) == 16 + 15 + 16 + 16                    # third step added on top


def test_exponent_flip_of_the_product_can_overflow_and_is_flagged():
    fmt = orc.BF16
    Aw, Bw = wl.gaussian(4, 4, 32, fmt, seed=3)
    p = orc.problem(4, 4, 32, 16, fmt)
    k = 5
    w = orc.round16(float(orc.decode16(int(Aw[1, k]), fmt)) * float(orc.decode16(int(Bw[2, k]), fmt)), fmt)
    assert (w & 0x4000) == 0                       # |product| < 2: exponent MSB clear
    rec = orc.trial(p, Aw, Bw, (orc.SITE_PRODUCT, 1, 2, k, 0x4000), orc.CORRECT_ZERO, orc.MODE_FULL)
    assert rec["n_flagged"] == 1 and rec["cls"] == orc.DETECTED and rec["n_dev_post"] == 1


# ------------------------------------------------------------ brute force against the NumPy statement

@pytest.mark.parametrize("fmt", [orc.FP16, orc.BF16])
def test_brute_force_every_term_and_bit(fmt):
    M, N, K, kb = 2, 2, 48, 16
    Aw, Bw = wl.gaussian(M, N, K, fmt, seed=31)
    Aw = Aw.copy(); Aw[1, 3] = 0; Aw[0, 17] = 0          # zero activations (Sec. V-B scenario i)
    p = orc.problem(M, N, K, kb, fmt)
    seen = set()
    zero_diff = 0
    for (i, j), k, bit in itertools.product([(0, 1), (1, 0)], range(K), range(16)):
        f = (orc.SITE_PRODUCT, i, j, k, 1 << bit)
        want = ref.run_trial(Aw, Bw, fmt, kb, f, orc.CORRECT_ZERO)
        full, cf, cc = orc.trial(p, Aw, Bw, f, orc.CORRECT_ZERO, orc.MODE_FULL, want_outputs=True)
        _same_fields(full, want, f)
        nan = np.isnan(want["C_f"])
        assert np.array_equal(np.isnan(cf), nan)
        assert np.array_equal(cf[~nan].view(np.uint32), want["C_f"][~nan].view(np.uint32))
        aff = orc.trial(p, Aw, Bw, f, orc.CORRECT_ZERO, orc.MODE_AFFECTED)
        for name in aff.dtype.names:
            assert aff[name] == full[name] or (np.isnan(aff[name]) and np.isnan(full[name])), (name, f)
        seen.add(int(full["cls"]))
        zero_diff += int(full["site_word_before"] == full["site_word_after"])
    assert seen == {orc.MASKED, orc.SDC, orc.DETECTED}
    assert 0 < zero_diff < 2 * K * 16


def test_multi_bit_masks_and_validity():
    fmt = orc.FP16
    M, N, K, kb = 3, 3, 32, 32
    Aw, Bw = wl.gaussian(M, N, K, fmt, seed=32)
    p = orc.problem(M, N, K, kb, fmt)
    for mask in (0x3, 0xF, 0xF000, 0x0180):
        f = (orc.SITE_PRODUCT, 2, 1, 30, mask)
        want = ref.run_trial(Aw, Bw, fmt, kb, f, orc.CORRECT_RECOMPUTE)
        full = orc.trial(p, Aw, Bw, f, orc.CORRECT_RECOMPUTE, orc.MODE_FULL)
        _same_fields(full, want, mask)
    # the high half of the mask is ignored; a term index beyond K is not a site
    a = orc.trial(p, Aw, Bw, (orc.SITE_PRODUCT, 2, 1, 30, 0x0180), orc.CORRECT_NONE, orc.MODE_AFFECTED)
    b = orc.trial(p, Aw, Bw, (orc.SITE_PRODUCT, 2, 1, 30, 0xABCD0180), orc.CORRECT_NONE, orc.MODE_AFFECTED)
    assert a["site_word_after"] == b["site_word_after"]
    bad = orc.trial(p, Aw, Bw, (orc.SITE_PRODUCT, 2, 1, K, 1), orc.CORRECT_NONE, orc.MODE_AFFECTED)
    assert bad["valid"] == 0 and bad["cls"] == orc.MASKED


def test_zero_products_fp16_changes_the_sum_far_more_often_than_bf16():
    # Sec. V-B: a zero product in FP16 becomes at least 2^-24 after one flip, in BF16 a number
    # near 2^-133 .. 2^-126 unless an exponent bit flips: with sums of order 1 the BF16 mantissa
    # flips are all absorbed, FP16's upper ones are not.
    K = 64
    counts = {}
    for fmt in (orc.FP16, orc.BF16):
        Aw, Bw = wl.gaussian(1, 1, K, fmt, seed=40)
        Aw = Aw.copy(); Aw[0, ::2] = 0                         # half of the activations are zero
        p = orc.problem(1, 1, K, 16, fmt)
        nz = 0
        for k in range(0, K, 2):
            for bit in range(16):
                r = orc.trial(p, Aw, Bw, (orc.SITE_PRODUCT, 0, 0, k, 1 << bit), orc.CORRECT_NONE, orc.MODE_AFFECTED)
                nz += int(r["site_word_before"] != r["site_word_after"])
        counts[fmt] = nz
    assert counts[orc.FP16] > 2 * counts[orc.BF16] > 0


# ------------------------------------------------------------ sampler

def test_product_site_sampler_ranges_and_spread():
    p = orc.problem(40, 24, 96, 32, orc.BF16)
    for nbits in (1, 2, 4):
        f = orc.sample_faults(11, 0, 6000, p, orc.KIND_ALL_PRODUCT, nbits)
        assert (f["kind"] == orc.SITE_PRODUCT).all()
        assert f["row"].max() == 39 and f["col"].max() == 23 and f["kblock"].max() == 95
        assert f["row"].min() == 0 and f["col"].min() == 0 and f["kblock"].min() == 0
        assert (f["xor_mask"] < 65536).all()
        pops = np.array([bin(int(m)).count("1") for m in f["xor_mask"]])
        assert (pops == nbits).all()
        pos = np.array([(int(m) & -int(m)).bit_length() - 1 for m in f["xor_mask"]])
        assert set(pos.tolist()) == set(range(16 - nbits + 1))
    a = orc.sample_faults(11, 100, 50, p, orc.KIND_ALL_PRODUCT, 1)
    b = orc.sample_faults(11, 0, 150, p, orc.KIND_ALL_PRODUCT, 1)[100:]
    assert (a == b).all()


# ------------------------------------------------------------ deviation histogram (Fig. 7 / Fig. 9)

def test_deviation_histogram_bins_are_binary32_exponents():
    recs = np.zeros(9, orc.RECORD_DTYPE)
    faults = orc.make_faults([(orc.SITE_ACC, 0, 0, 0, 1)] * 6 + [(orc.SITE_PRODUCT, 0, 0, 0, 1), (orc.SITE_A, 0, 0, 0, 1),
                              (orc.SITE_ACC, 0, 0, 0, 1)])
    recs["valid"] = 1
    recs["valid"][8] = 0                                           # invalid site: skipped everywhere
    pairs = [(17.0, 17.0), (17.0, 15.0), (1.0, 4.0), (1.0, np.inf), (0.0, 2.0 ** -130), (2.0 ** 100, -2.0 ** 100),
             (15.0, 15.000030517578125), (3.0, 5.0), (1.0, 2.0)]
    for t, (b, a) in enumerate(pairs):
        recs["site_word_before"][t] = np.array([b], np.float32).view(np.uint32)[0]
        recs["site_word_after"][t] = np.array([a], np.float32).view(np.uint32)[0]
    recs["max_dev_pre"] = [0.0, 0.75, 1.0, np.inf, 1e-50, 3.0, 1e39, 2.0, 8.0]
    recs["max_dev_post"] = 0.0
    h = orc.deviation_histogram(recs, faults, orc.HIST_SITE)
    # diffs: 0 | 2 | 3 | Inf | subnormal | 2^101 | 2^-15 ; the operand trial and the invalid one are skipped
    want = {0: 2, 128: 2, 255: 1, 127 + 101: 1, 127 - 15: 1}
    assert {int(b): int(c) for b, c in enumerate(h) if c} == want
    h = orc.deviation_histogram(recs, faults, orc.HIST_DEV_PRE)
    # 0 | 0.75 | 1 | Inf | 1e-50 -> 0 in binary32 | 3 | 1e39 -> Inf in binary32 | 2
    assert {int(b): int(c) for b, c in enumerate(h) if c} == {0: 2, 126: 1, 127: 1, 128: 2, 255: 2}
    assert int(orc.deviation_histogram(recs, faults, orc.HIST_DEV_POST)[0]) == 8


def test_deviation_histogram_of_a_campaign_matches_frexp_binning():
    fmt = orc.BF16
    Aw, Bw = wl.gaussian(24, 16, 64, fmt, seed=91)
    p = orc.problem(24, 16, 64, 16, fmt)
    faults = orc.sample_faults(3, 0, 1500, p, orc.KIND_ALL_PRODUCT, 2)
    recs = orc.campaign(p, Aw, Bw, faults, orc.CORRECT_ZERO, orc.MODE_AFFECTED)
    h = orc.deviation_histogram(recs, faults, orc.HIST_SITE)
    b = recs["site_word_before"].view(np.float32)
    a = recs["site_word_after"].view(np.float32)
    with np.errstate(all="ignore"):
        d = np.abs(a - b).astype(np.float32)
    want = np.zeros(256, np.uint64)
    for x in d.tolist():
        if not np.isfinite(x):
            want[255] += 1
        elif x < 2.0 ** -126:
            want[0] += 1
        else:
            m, e = np.frexp(x)                       # x = m * 2^e, m in [0.5, 1): floor(log2 x) = e - 1
            want[e - 1 + 127] += 1
    assert np.array_equal(h, want) and int(h.sum()) == 1500
    # the ECDF reaches 1 and the zero-difference share is Table III's statistic
    assert int(h[0]) == int((recs["site_word_before"] == recs["site_word_after"]).sum() + ((d > 0) & (d < 2.0 ** -126)).sum())
