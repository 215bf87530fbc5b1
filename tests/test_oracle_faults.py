"""Pins for fault application, detector, corrector, counters and classes
(Sec. III-E write target, Sec. IV-C fault model, Sec. VI-A/B detection then correction)."""
import itertools

import numpy as np
import pytest

from oracle import pyoracle as orc
from paper_2311_05782_amd import workloads as wl
import np_reference as ref


def ones_problem(K=128, kb=32, first_only=False, fmt=orc.FP16):
    """Row 0 of A and column 0 of B all ones (or a = e_0): acc after block s is 32(s+1)."""
    M = N = 2
    a = np.ones((M, K), np.float32)
    b = np.ones((N, K), np.float32)
    if first_only:
        a[0, 1:] = 0
    return orc.problem(M, N, K, kb, fmt), wl.to_words(a, fmt), wl.to_words(b, fmt)


# ---- worked flips: known accumulator value, known result ---------------------------------

@pytest.mark.parametrize("bit,after,final,flag", [
    (23, 0x42800000, 160.0, 1),     # 32 -> 64, three more blocks of 32; 160 > T = 128.0625
    (31, 0xC2000000, 64.0, 0),      # 32 -> -32
    (30, 0x02000000, 96.0, 0),      # 32 -> 2^-123, vanishes in the next addition
    (22, 0x42400000, 144.0, 1),     # 32 -> 48
])
def test_worked_single_bit_flips(bit, after, final, flag):
    p, Aw, Bw = ones_problem()
    rec, cf, cc = orc.trial(p, Aw, Bw, (orc.SITE_ACC, 0, 0, 0, 1 << bit), orc.CORRECT_NONE,
                            orc.MODE_FULL, want_outputs=True)
    assert rec["site_word_before"] == 0x42000000
    assert rec["site_word_after"] == after
    assert cf[0, 0] == final and cf[0, 1] == 128.0 and cf[1, 0] == 128.0 and cf[1, 1] == 128.0
    assert rec["n_bitdiff"] == 1 and rec["n_flagged"] == flag
    assert rec["cls"] == (orc.DETECTED if flag else orc.SDC)
    assert rec["max_dev_pre"] == abs(final - 128.0) and rec["n_dev_pre"] == 1


def test_worked_flip_threshold_side():
    # T = 128.0625 for all-ones operands; 160 exceeds it.  Zeroing leaves |C*| as the
    # residual, recomputation leaves none.
    p, Aw, Bw = ones_problem()
    rec = orc.trial(p, Aw, Bw, (orc.SITE_ACC, 0, 0, 0, 1 << 23), orc.CORRECT_ZERO)
    assert rec["n_flagged"] == 1 and rec["cls"] == orc.DETECTED
    assert rec["n_dev_pre"] == 1 and rec["max_dev_pre"] == 32.0
    assert rec["max_dev_post"] == 128.0 and rec["n_dev_post"] == 1     # zeroing leaves |C*|
    rec = orc.trial(p, Aw, Bw, (orc.SITE_ACC, 0, 0, 0, 1 << 23), orc.CORRECT_RECOMPUTE)
    assert rec["n_flagged"] == 1 and rec["n_dev_post"] == 0 and rec["max_dev_post"] == 0.0


def test_low_mantissa_flip_is_absorbed():
    # 32 + 2^-18 is carried exactly through 33..63 and lost to round-to-even at 64.
    p, Aw, Bw = ones_problem()
    rec, cf, _ = orc.trial(p, Aw, Bw, (orc.SITE_ACC, 0, 0, 0, 1), orc.CORRECT_ZERO,
                           orc.MODE_FULL, want_outputs=True)
    assert rec["site_word_after"] == 0x42000001
    assert cf[0, 0] == 128.0 and rec["n_bitdiff"] == 0
    assert rec["n_dev_pre"] == 0 and rec["n_flagged"] == 0 and rec["cls"] == orc.MASKED
    # injected in the LAST block it survives, but stays inside the tolerance: still masked
    rec, cf, _ = orc.trial(p, Aw, Bw, (orc.SITE_ACC, 0, 0, 3, 1), orc.CORRECT_ZERO,
                           orc.MODE_FULL, want_outputs=True)
    assert cf.view(np.uint32)[0, 0] == 0x43000001 and rec["n_bitdiff"] == 1
    assert rec["max_dev_pre"] == 2.0 ** -16 and rec["cls"] == orc.MASKED


def test_exponent_msb_flip_up_is_flagged_down_is_not():
    # acc = 1.0 = 0x3F800000; bit 30: 0 -> 1 gives +Inf, which any bound flags.
    p, Aw, Bw = ones_problem(first_only=True)
    for policy in (orc.CORRECT_ZERO, orc.CORRECT_RECOMPUTE):
        rec, cf, cc = orc.trial(p, Aw, Bw, (orc.SITE_ACC, 0, 1, 0, 1 << 30), policy,
                                orc.MODE_FULL, want_outputs=True)
        assert rec["site_word_before"] == 0x3F800000 and rec["site_word_after"] == 0x7F800000
        assert np.isinf(cf[0, 1]) and rec["n_flagged"] == 1 and rec["cls"] == orc.DETECTED
        assert np.isinf(rec["max_dev_pre"])
        assert cc[0, 1] == (0.0 if policy == orc.CORRECT_ZERO else 1.0)
    # NaN after the flip (exponent all ones, mantissa non-zero) is flagged too
    a = np.zeros((2, 128), np.float32); a[0, 0] = 1.5
    Aw2 = wl.to_fp16_words(a)
    rec = orc.trial(p, Aw2, Bw, (orc.SITE_ACC, 0, 0, 0, 1 << 30), orc.CORRECT_ZERO)
    assert rec["site_word_after"] == 0x7FC00000 and rec["n_flagged"] == 1
    # 1 -> 0 on |acc| >= 2 shrinks the value by 2^128: never flagged, an SDC
    p2, A2, B2 = ones_problem()
    rec = orc.trial(p2, A2, B2, (orc.SITE_ACC, 1, 1, 2, 1 << 30), orc.CORRECT_ZERO)
    assert rec["site_word_before"] == 0x42C00000 and rec["n_flagged"] == 0 and rec["cls"] == orc.SDC
    assert rec["max_dev_pre"] == 96.0
    # acc = +0 (first two k-blocks of the row are zero) -> 2.0, final 66: not flagged
    z = np.ones((2, 128), np.float32); z[0, :64] = 0
    rec = orc.trial(p2, wl.to_fp16_words(z), B2, (orc.SITE_ACC, 0, 0, 1, 1 << 30), orc.CORRECT_ZERO)
    assert rec["site_word_before"] == 0 and rec["site_word_after"] == 0x40000000
    assert rec["n_flagged"] == 0 and rec["cls"] == orc.SDC and rec["max_dev_pre"] == 2.0
    # an all-zero row has bound T = 0: any non-zero output there is flagged
    z[0, :] = 0
    rec = orc.trial(p2, wl.to_fp16_words(z), B2, (orc.SITE_ACC, 0, 0, 1, 1 << 30), orc.CORRECT_ZERO)
    assert rec["n_flagged"] == 1 and rec["cls"] == orc.DETECTED


def test_bf16_and_k_block_position():
    # Same worked example in BF16 with kb = 64: acc after block 0 is 64 = 0x42800000.
    p, Aw, Bw = ones_problem(kb=64, fmt=orc.BF16)
    rec, cf, _ = orc.trial(p, Aw, Bw, (orc.SITE_ACC, 1, 0, 0, 1 << 24), orc.CORRECT_NONE,
                           orc.MODE_FULL, want_outputs=True)
    assert rec["site_word_before"] == 0x42800000 and rec["site_word_after"] == 0x43800000
    assert cf[1, 0] == 256.0 + 64.0
    rec, cf, _ = orc.trial(p, Aw, Bw, (orc.SITE_ACC, 1, 0, 1, 1 << 24), orc.CORRECT_NONE,
                           orc.MODE_FULL, want_outputs=True)
    assert rec["site_word_before"] == 0x43000000 and cf[1, 0] == 32.0   # 128 -> 2^(134-127-2)=32


# ---- operand faults -----------------------------------------------------------------------

def test_operand_fault_reaches_exactly_one_row_or_column():
    M, N, K, kb = 6, 7, 64, 32
    Aw, Bw = wl.gaussian(M, N, K, orc.FP16, seed=2)
    p = orc.problem(M, N, K, kb, orc.FP16)
    gold = orc.gemm(p, Aw, Bw)
    rec, cf, _ = orc.trial(p, Aw, Bw, (orc.SITE_A, 4, 37, 0, 1 << 13), orc.CORRECT_NONE,
                           orc.MODE_FULL, want_outputs=True)
    diff = cf.view(np.uint32) != gold.view(np.uint32)
    assert diff[4].all() and not np.delete(diff, 4, axis=0).any()
    assert rec["site_word_before"] == Aw[4, 37] and rec["site_word_after"] == Aw[4, 37] ^ (1 << 13)
    A2 = Aw.copy(); A2[4, 37] ^= 1 << 13
    assert np.array_equal(cf.view(np.uint32), orc.gemm(p, A2, Bw).view(np.uint32))
    rec, cf, _ = orc.trial(p, Aw, Bw, (orc.SITE_B, 50, 3, 0, 1 << 15), orc.CORRECT_NONE,
                           orc.MODE_FULL, want_outputs=True)
    diff = cf.view(np.uint32) != gold.view(np.uint32)
    assert diff[:, 3].all() and not np.delete(diff, 3, axis=1).any()
    B2 = Bw.copy(); B2[3, 50] ^= 1 << 15
    assert np.array_equal(cf.view(np.uint32), orc.gemm(p, Aw, B2).view(np.uint32))
    # only the low 16 bits of the mask apply to an operand
    r1 = orc.trial(p, Aw, Bw, (orc.SITE_A, 1, 2, 0, 0xABCD0004), orc.CORRECT_NONE)
    assert r1["site_word_after"] == Aw[1, 2] ^ 0x0004


def test_fp16_exponent_flip_to_inf_propagates_as_ieee():
    # |a| in [1,2): flipping the FP16 exponent MSB gives Inf; Inf*0 = NaN; all flagged.
    M, N, K = 2, 3, 32
    a = np.ones((M, K), np.float32); b = np.ones((N, K), np.float32); b[1, 0] = 0.0
    p = orc.problem(M, N, K, 32, orc.FP16)
    rec, cf, cc = orc.trial(p, wl.to_fp16_words(a), wl.to_fp16_words(b),
                            (orc.SITE_A, 0, 0, 0, 1 << 14), orc.CORRECT_RECOMPUTE,
                            orc.MODE_FULL, want_outputs=True)
    assert rec["site_word_after"] == 0x7C00
    assert np.isinf(cf[0, 0]) and np.isnan(cf[0, 1]) and np.isinf(cf[0, 2])
    assert rec["n_flagged"] == 3 and rec["cls"] == orc.DETECTED
    assert np.array_equal(cc[0], [32.0, 31.0, 32.0]) and rec["n_dev_post"] == 0


# ---- invariants ---------------------------------------------------------------------------

def test_invariants_on_random_problem():
    M, N, K, kb = 5, 6, 96, 32
    Aw, Bw = wl.gaussian(M, N, K, orc.BF16, seed=9)
    p = orc.problem(M, N, K, kb, orc.BF16)
    gold = orc.gemm(p, Aw, Bw)
    S = K // kb
    # no fault / zero mask => masked, nothing differs
    for f in [(orc.SITE_NONE, 0, 0, 0, 0), (orc.SITE_ACC, 1, 1, 1, 0), (orc.SITE_A, 2, 3, 0, 0)]:
        rec, cf, cc = orc.trial(p, Aw, Bw, f, orc.CORRECT_ZERO, orc.MODE_FULL, want_outputs=True)
        assert rec["cls"] == orc.MASKED and rec["n_bitdiff"] == 0 and rec["n_flagged"] == 0
        assert np.array_equal(cf.view(np.uint32), gold.view(np.uint32))
        assert np.array_equal(cc.view(np.uint32), gold.view(np.uint32))
    for bit in range(32):
        # last block: the output word is the golden word with the mask applied
        rec, cf, _ = orc.trial(p, Aw, Bw, (orc.SITE_ACC, 3, 2, S - 1, 1 << bit), orc.CORRECT_NONE,
                               orc.MODE_FULL, want_outputs=True)
        assert cf.view(np.uint32)[3, 2] == gold.view(np.uint32)[3, 2] ^ (1 << bit)
        d = cf.view(np.uint32) != gold.view(np.uint32)
        assert d.sum() == 1 and d[3, 2]
        assert rec["site_word_before"] == gold.view(np.uint32)[3, 2]
    # sign flip in the last block: c^f = -C*, never flagged
    rec, cf, _ = orc.trial(p, Aw, Bw, (orc.SITE_ACC, 0, 5, S - 1, 1 << 31), orc.CORRECT_ZERO,
                           orc.MODE_FULL, want_outputs=True)
    assert cf[0, 5] == -gold[0, 5] and rec["n_flagged"] == 0
    # out-of-range site: trial runs fault-free and says so
    for f in [(orc.SITE_ACC, M, 0, 0, 1), (orc.SITE_ACC, 0, N, 0, 1), (orc.SITE_ACC, 0, 0, S, 1),
              (orc.SITE_A, 0, K, 0, 1), (orc.SITE_B, K, 0, 0, 1), (7, 0, 0, 0, 1)]:
        rec = orc.trial(p, Aw, Bw, f, orc.CORRECT_ZERO)
        assert rec["valid"] == 0 and rec["cls"] == orc.MASKED and rec["n_bitdiff"] == 0


def test_recompute_restores_and_zero_writes_plus_zero():
    M, N, K, kb = 4, 4, 64, 32
    Aw, Bw = wl.gaussian(M, N, K, orc.FP16, seed=4)
    p = orc.problem(M, N, K, kb, orc.FP16)
    gold = orc.gemm(p, Aw, Bw)
    f = (orc.SITE_ACC, 2, 1, 1, 1 << 29)
    rz, cf, cz = orc.trial(p, Aw, Bw, f, orc.CORRECT_ZERO, orc.MODE_FULL, want_outputs=True)
    rr, _, cr = orc.trial(p, Aw, Bw, f, orc.CORRECT_RECOMPUTE, orc.MODE_FULL, want_outputs=True)
    rn, _, cn = orc.trial(p, Aw, Bw, f, orc.CORRECT_NONE, orc.MODE_FULL, want_outputs=True)
    assert rz["n_flagged"] == 1
    assert cz.view(np.uint32)[2, 1] == 0 and cr[2, 1] == gold[2, 1] and cn[2, 1] == cf[2, 1]
    assert rr["n_dev_post"] == 0 and rr["n_dev_post"] <= rr["n_dev_pre"]
    assert rn["n_dev_post"] == rn["n_dev_pre"] and rn["max_dev_post"] == rn["max_dev_pre"]
    # XOR is an involution: applying the same operand mask to the already faulted matrix gives C*
    A2 = Aw.copy(); A2[1, 7] ^= 0x0100
    r = orc.trial(p, A2, Bw, (orc.SITE_A, 1, 7, 0, 0x0100), orc.CORRECT_NONE, orc.MODE_FULL, want_outputs=True)
    assert np.array_equal(r[1].view(np.uint32), gold.view(np.uint32))


def test_flag_is_monotone_in_gamma_and_global_bound_is_looser():
    M, N, K, kb = 6, 6, 64, 32
    Aw, Bw = wl.gaussian(M, N, K, orc.FP16, seed=6)
    f = (orc.SITE_A, 2, 9, 0, 1 << 13)          # scales one operand by 2^8: some of the row exceeds T
    counts = []
    for g in (1.0, 1.5, 4.0, 64.0, 1e6):
        p = orc.problem(M, N, K, kb, orc.FP16, gamma=g)
        counts.append(int(orc.trial(p, Aw, Bw, f, orc.CORRECT_ZERO)["n_flagged"]))
    assert counts == sorted(counts, reverse=True) and counts[-1] == 0
    pr = orc.problem(M, N, K, kb, orc.FP16)
    pg = orc.problem(M, N, K, kb, orc.FP16, bound_mode=orc.BOUND_GLOBAL)
    assert orc.trial(pg, Aw, Bw, f, orc.CORRECT_ZERO)["n_flagged"] <= \
        orc.trial(pr, Aw, Bw, f, orc.CORRECT_ZERO)["n_flagged"]


# ---- brute force against the independent NumPy reference -----------------------------------

FIELDS = ["n_flagged", "n_bitdiff", "n_dev_pre", "n_dev_post", "site_word_before",
          "site_word_after", "cls"]


def _same(rec, want):
    for k in FIELDS:
        assert int(rec[k]) == int(want[k]), (k, int(rec[k]), int(want[k]))
    for k in ("max_dev_pre", "max_dev_post"):
        assert float(rec[k]) == float(want[k]), k


@pytest.mark.parametrize("fmt,policy", [(orc.FP16, orc.CORRECT_ZERO), (orc.BF16, orc.CORRECT_RECOMPUTE)])
def test_brute_force_all_accumulator_sites_and_bits(fmt, policy):
    M, N, K, kb = 3, 2, 64, 16
    Aw, Bw = wl.gaussian(M, N, K, fmt, seed=21)
    p = orc.problem(M, N, K, kb, fmt)
    seen = set()
    for i, j, s, bit in itertools.product(range(M), range(N), range(K // kb), range(32)):
        f = (orc.SITE_ACC, i, j, s, 1 << bit)
        want = ref.run_trial(Aw, Bw, fmt, kb, f, policy)
        full, cf, cc = orc.trial(p, Aw, Bw, f, policy, orc.MODE_FULL, want_outputs=True)
        _same(full, want)
        assert np.array_equal(cf.view(np.uint32), want["C_f"].view(np.uint32))
        assert np.array_equal(cc.view(np.uint32), want["C_c"].view(np.uint32))
        aff = orc.trial(p, Aw, Bw, f, policy, orc.MODE_AFFECTED)
        for k in aff.dtype.names:
            a, b = aff[k], full[k]
            assert a == b or (np.isnan(a) and np.isnan(b)), k
        seen.add(int(full["cls"]))
    assert seen == {orc.MASKED, orc.SDC, orc.DETECTED}


def test_brute_force_operand_sites_and_bursts():
    M, N, K, kb = 3, 4, 32, 16
    fmt = orc.FP16
    Aw, Bw = wl.gaussian(M, N, K, fmt, seed=22, scale_b=0.05)
    p = orc.problem(M, N, K, kb, fmt)
    cases = [(orc.SITE_A, i, k, 0, m << pos) for i in range(M) for k in (0, 15, 16, 31)
             for m in (1, 3, 15) for pos in range(0, 17 - 4)]
    cases += [(orc.SITE_B, k, j, 0, 1 << pos) for j in range(N) for k in (3, 30) for pos in range(16)]
    cases += [(orc.SITE_ACC, 1, 2, 1, 3 << pos) for pos in range(31)]
    for f in cases:
        want = ref.run_trial(Aw, Bw, fmt, kb, f, orc.CORRECT_RECOMPUTE)
        full = orc.trial(p, Aw, Bw, f, orc.CORRECT_RECOMPUTE, orc.MODE_FULL)
        _same(full, want)
        aff = orc.trial(p, Aw, Bw, f, orc.CORRECT_RECOMPUTE, orc.MODE_AFFECTED)
        for k in aff.dtype.names:
            assert aff[k] == full[k] or (np.isnan(aff[k]) and np.isnan(full[k])), (k, f)
    # global bound against the reference too
    pg = orc.problem(M, N, K, kb, fmt, bound_mode=orc.BOUND_GLOBAL)
    for f in cases[::17]:
        want = ref.run_trial(Aw, Bw, fmt, kb, f, orc.CORRECT_ZERO, bound_global=True)
        _same(orc.trial(pg, Aw, Bw, f, orc.CORRECT_ZERO, orc.MODE_FULL), want)


def test_campaign_equals_single_trials_and_classify_counts():
    M, N, K, kb = 8, 8, 64, 32
    Aw, Bw = wl.gaussian(M, N, K, orc.BF16, seed=30)
    p = orc.problem(M, N, K, kb, orc.BF16)
    faults = orc.sample_faults(77, 0, 96, p, orc.KIND_MIX_ACC_A, 1)
    aff = orc.campaign(p, Aw, Bw, faults, orc.CORRECT_ZERO, orc.MODE_AFFECTED)
    full = orc.campaign(p, Aw, Bw, faults, orc.CORRECT_ZERO, orc.MODE_FULL)
    assert aff.tobytes() == full.tobytes()
    for t in (0, 1, 50, 95):
        one = orc.trial(p, Aw, Bw, faults[t:t + 1], orc.CORRECT_ZERO, orc.MODE_FULL)
        assert one.tobytes() == full[t].tobytes()
    cls, counts = orc.classify(full)
    assert np.array_equal(cls, full["cls"].astype(np.uint8))
    assert counts.sum() == 96 and all(int(counts[c]) == int((cls == c).sum()) for c in range(3))


# ---- standalone detector -------------------------------------------------------------------

def test_standalone_detector_edges():
    M, N, K = 2, 2, 128
    p, Aw, Bw = ones_problem()
    ra, cb, _ = orc.rowcol_absmax(p, Aw, Bw)
    T = np.float32(128.0625)
    Cb = np.array([[[T, np.nextafter(T, np.float32(np.inf))], [-T, -np.nextafter(T, np.float32(np.inf))]],
                   [[np.nan, np.inf], [-np.inf, 0.0]]], np.float32)
    cs = np.full((M, N), 128.0, np.float32)
    out, flags, n = orc.detect_correct(p, ra, cb, Cb, orc.CORRECT_ZERO)
    assert flags.tolist() == [[[0, 1], [0, 1]], [[1, 1], [1, 0]]] and n.tolist() == [2, 3]
    assert out[0, 0, 0] == T and out.view(np.uint32)[0, 0, 1] == 0 and out.view(np.uint32)[1, 0, 0] == 0
    out, _, _ = orc.detect_correct(p, ra, cb, Cb, orc.CORRECT_RECOMPUTE, c_star=cs)
    assert out[1].tolist() == [[128.0, 128.0], [128.0, 0.0]]
    out, _, n = orc.detect_correct(p, ra, cb, Cb, orc.CORRECT_NONE)
    assert np.array_equal(out.view(np.uint32), Cb.view(np.uint32)) and n.tolist() == [2, 3]


def test_guard_band_counters():
    # acc = 32 after block 0; T = 128.0625.  A flip of bit 24 gives 128 (+96 = 224): far from T.
    p, Aw, Bw = ones_problem()
    r = orc.trial(p, Aw, Bw, (orc.SITE_ACC, 0, 0, 0, 1 << 24), orc.CORRECT_ZERO)
    assert r["n_border_T"] == 0 and r["n_border_tau"] == 0
    # last block, bit 0 set on 128.0: |c| - T = 0.0625 - tiny, inside 2^-6*T -> borderline for T
    r = orc.trial(p, Aw, Bw, (orc.SITE_ACC, 0, 0, 3, 1), orc.CORRECT_ZERO)
    assert r["n_border_T"] == 1
    # tau = 2^-12 * 128 = 2^-5: a last-block flip of bit 11 changes 128 by 2^-5 -> on the band
    r = orc.trial(p, Aw, Bw, (orc.SITE_ACC, 0, 0, 3, 1 << 11), orc.CORRECT_ZERO)
    assert r["max_dev_pre"] == 2.0 ** -5 and r["n_dev_pre"] == 0 and r["n_border_tau"] == 1
    r = orc.trial(p, Aw, Bw, (orc.SITE_ACC, 0, 0, 3, 1 << 12), orc.CORRECT_ZERO)
    assert r["n_dev_pre"] == 1 and r["n_border_tau"] == 1
    r = orc.trial(p, Aw, Bw, (orc.SITE_ACC, 0, 0, 3, 1 << 14), orc.CORRECT_ZERO)
    assert r["n_dev_pre"] == 1 and r["n_border_tau"] == 0
