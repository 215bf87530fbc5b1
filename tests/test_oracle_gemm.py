"""Pins for the oracle's fault-free GEMM (Sec. II-B D = A x B; Sec. IV-C FP32 accumulation)."""
import numpy as np
import pytest

from oracle import pyoracle as orc
from paper_2311_05782_amd import workloads as wl
import np_reference as ref


@pytest.mark.parametrize("fmt", [orc.FP16, orc.BF16])
@pytest.mark.parametrize("kb", [16, 32, 48, 96])
def test_small_integer_operands_equal_integer_matmul(fmt, kb):
    # |a|,|b| <= 4, K = 96: all partial sums are integers below 2^24, so the
    # blocked FP32 accumulation is exact whatever the k-block.
    M, N, K = 7, 5, 96
    Aw, Bw = wl.small_integers(M, N, K, fmt, seed=kb)
    A = ref.decode(Aw, fmt).astype(np.int64)
    Bt = ref.decode(Bw, fmt).astype(np.int64)
    want = A @ Bt.T
    got = orc.gemm(orc.problem(M, N, K, kb, fmt), Aw, Bw)
    assert got.shape == (M, N)
    assert np.array_equal(got.astype(np.int64), want)
    assert np.all(got == want.astype(np.float32))


def test_b_layouts_and_leading_dimensions_agree():
    M, N, K, kb = 6, 9, 64, 32
    Aw, Bw = wl.gaussian(M, N, K, orc.FP16, seed=3)
    base = orc.gemm(orc.problem(M, N, K, kb, orc.FP16), Aw, Bw)
    # B stored as K rows of N
    Bkn = np.ascontiguousarray(Bw.T)
    alt = orc.gemm(orc.problem(M, N, K, kb, orc.FP16, b_layout=1), Aw, Bkn)
    assert np.array_equal(base.view(np.uint32), alt.view(np.uint32))
    # padded leading dimensions
    Ap = np.zeros((M, K + 8), np.uint16); Ap[:, :K] = Aw
    Bp = np.zeros((N, K + 24), np.uint16); Bp[:, :K] = Bw
    pad = orc.gemm(orc.problem(M, N, K, kb, orc.FP16, lda=K + 8, ldb=K + 24), Ap, Bp)
    assert np.array_equal(base.view(np.uint32), pad.view(np.uint32))


@pytest.mark.parametrize("fmt", [orc.FP16, orc.BF16])
def test_matches_stepwise_numpy_float32(fmt):
    M, N, K, kb = 5, 4, 96, 32
    Aw, Bw = wl.gaussian(M, N, K, fmt, seed=11)
    got = orc.gemm(orc.problem(M, N, K, kb, fmt), Aw, Bw)
    A, Bt = ref.decode(Aw, fmt), ref.decode(Bw, fmt)
    for i in range(M):
        for j in range(N):
            want = ref.dot(A[i], Bt[j], kb)[0]
            assert np.float32(got[i, j]).view(np.uint32) == np.float32(want).view(np.uint32)
            assert orc.dot(orc.problem(M, N, K, kb, fmt), Aw, Bw, i, j) == got[i, j]


@pytest.mark.parametrize("fmt", [orc.FP16, orc.BF16])
def test_within_tolerance_of_float64_matmul(fmt):
    # |C* - sum_k a b| <= 2^-12 * sum_k |a b| against an independent float64 matmul.
    M, N, K, kb = 48, 40, 1024, 64
    Aw, Bw = wl.gaussian(M, N, K, fmt, seed=7)
    Cm, R, S = orc.gemm(orc.problem(M, N, K, kb, fmt), Aw, Bw, want_double=True)
    A = ref.decode(Aw, fmt).astype(np.float64)
    Bt = ref.decode(Bw, fmt).astype(np.float64)
    R64 = A @ Bt.T
    S64 = np.abs(A) @ np.abs(Bt).T
    assert np.allclose(R, R64, rtol=0, atol=1e-9 * S64.max())
    assert np.allclose(S, S64, rtol=1e-12)
    assert np.all(np.abs(Cm.astype(np.float64) - R64) <= 2.0 ** -12 * S64)
    # and it is not trivially far inside: the fp32 sum differs from the exact one somewhere
    assert np.any(Cm.astype(np.float64) != R64)


def test_products_of_operands_obey_exponent_bound():
    # Sec. VI-A: m1*m2 < 4  =>  e_m <= e1 + e2 + 1, for every pair of finite operands.
    rng = np.random.default_rng(0)
    for fmt in (orc.FP16, orc.BF16):
        w1 = rng.integers(0, 65536, 20000).astype(np.uint16)
        w2 = rng.integers(0, 65536, 20000).astype(np.uint16)
        x1 = orc.decode_array(w1, fmt).astype(np.float64)
        x2 = orc.decode_array(w2, fmt).astype(np.float64)
        ok = np.isfinite(x1) & np.isfinite(x2) & (x1 != 0) & (x2 != 0)
        e1 = np.floor(np.log2(np.abs(x1[ok])))
        e2 = np.floor(np.log2(np.abs(x2[ok])))
        em = np.floor(np.log2(np.abs(x1[ok] * x2[ok])))
        assert np.all(em <= e1 + e2 + 1)
        assert np.any(em == e1 + e2 + 1)


def test_clean_outputs_never_exceed_threshold():
    # |C*_ij| <= K*ra_i*cb_j*gamma even when every product in a row is maximal.
    M, N, K, kb = 4, 4, 4096, 64
    for fmt in (orc.FP16, orc.BF16):
        a = np.full((M, K), 1.9921875, np.float32)       # same sign, all at the row maximum
        b = np.full((N, K), 1.9921875, np.float32)
        a[1] *= -1
        Aw, Bw = wl.to_words(a, fmt), wl.to_words(b, fmt)
        p = orc.problem(M, N, K, kb, fmt)
        Cm = orc.gemm(p, Aw, Bw)
        ra, cb, finite = orc.rowcol_absmax(p, Aw, Bw)
        assert finite
        for i in range(M):
            for j in range(N):
                assert abs(Cm[i, j]) <= orc.threshold(K, ra[i], cb[j])
                assert abs(Cm[i, j]) > 0.99 * orc.threshold(K, ra[i], cb[j], 1.0)


def test_default_slack_grows_with_K_and_covers_a_long_accumulation():
    # 1 + 2^-11 up to K = 4096, one more 2^-11 per further 4096 terms.
    assert orc.default_gamma(16) == 1 + 2.0 ** -11 and orc.default_gamma(4096) == 1 + 2.0 ** -11
    assert orc.default_gamma(4097) == 1 + 2.0 ** -10 and orc.default_gamma(8192) == 1 + 2.0 ** -10
    assert orc.default_gamma(65536) == 1 + 2.0 ** -7
    # Why: 65536 equal products (143/128)^2, added one by one in binary32, round upwards step
    # after step and end 8.9e-4 above the exact sum - more than the 4.9e-4 the short-K slack allows.
    K, kb, fmt = 65536, 64, orc.BF16
    a = np.full((1, K), 143.0 / 128.0, np.float32)
    Aw, Bw = wl.to_words(a, fmt), wl.to_words(a, fmt)
    p = orc.problem(1, 1, K, kb, fmt)
    assert p.gamma == np.float32(1 + 2.0 ** -7)
    c = float(orc.gemm(p, Aw, Bw)[0, 0])
    exact = K * (143.0 / 128.0) ** 2
    assert c == float(np.cumsum(np.full(K, np.float32((143.0 / 128.0) ** 2), np.float32), dtype=np.float32)[-1])
    assert c / exact > 1 + 2.0 ** -11 and c / exact < 1 + 2.0 ** -8
    ra, cb, _ = orc.rowcol_absmax(p, Aw, Bw)
    assert c > orc.threshold(K, ra[0], cb[0], 1 + 2.0 ** -11)        # the short-K slack would flag it
    assert c <= orc.threshold(K, ra[0], cb[0], orc.default_gamma(K))  # the default does not
    # and every mantissa of a same-sign, all-maximal row stays below the default bound
    for K in (8192, 65536):
        for m in range(128, 256, 5):
            v = np.float32((m / 128.0) ** 2)
            tot = float(np.cumsum(np.full(K, v, np.float32), dtype=np.float32)[-1])
            assert tot <= orc.threshold(K, m / 128.0, m / 128.0, orc.default_gamma(K)), (K, m)


def test_rowcol_absmax_and_threshold_rounding():
    M, N, K = 3, 2, 32
    a = np.zeros((M, K), np.float32); b = np.zeros((N, K), np.float32)
    a[0, 5] = -3.5; a[0, 6] = 2.0; a[1, 0] = 0.25; b[0, 31] = -7.0; b[1, 1] = 1.0 / 3.0
    Aw, Bw = wl.to_fp16_words(a), wl.to_fp16_words(b)
    p = orc.problem(M, N, K, 32, orc.FP16)
    ra, cb, finite = orc.rowcol_absmax(p, Aw, Bw)
    assert finite and list(ra) == [3.5, 0.25, 0.0] and cb[0] == 7.0
    assert cb[1] == np.float32(np.float16(1.0 / 3.0))
    # K=128, ra=cb=1: T = 128 * (1 + 2^-11) exactly
    assert orc.threshold(128, 1.0, 1.0) == 128.0625
    # each step rounds to binary32: compare with float32 scalar arithmetic
    g = np.float32(1 + 2.0 ** -11)
    for K_, r, c in [(768, 4.33, 0.0871), (4096, 0.99609375, 0.99609375), (576, 5.1, 0.23)]:
        want = np.float32(np.float32(np.float32(np.float32(K_) * np.float32(r)) * np.float32(c)) * g)
        assert orc.threshold(K_, r, c) == want
    # Inf / NaN operands are reported
    Aw2 = Aw.copy(); Aw2[2, 2] = 0x7C00
    assert not orc.rowcol_absmax(p, Aw2, Bw)[2]
    Bw2 = Bw.copy(); Bw2[1, 3] = 0x7E01
    assert not orc.rowcol_absmax(p, Aw, Bw2)[2]
