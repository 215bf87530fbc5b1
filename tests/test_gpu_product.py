"""GPU parity for the paper's product-term fault (Sec. III-E write-back, Eq. 1-2): HIP path
through the C ABI against the oracle, element by element."""
import dataclasses

import numpy as np
import pytest

import gpu_util as gu
from oracle import pyoracle as orc
from paper_2311_05782_amd import fi, workloads as wl
from test_gpu_parity import _campaign_parity

pytestmark = pytest.mark.gpu


def _safe_product_faults(Aw, Bw, fmt, n, seed):
    """Product-term faults that keep the exact regime exact: operands are even integers, so a
    non-zero product is an integer of magnitude >= 4 with few significant bits; flipping its
    sign, one of its two lowest exponent bits or one of its three highest mantissa bits gives a
    dyadic value whose sum with small integers is exactly representable in every order.  Zero
    products get the same masks in BF16 (the result is tiny and absorbed by any non-zero sum)
    and only sign or exponent masks in FP16 (still zero, or 2^-14 .. 2^-13 times a small integer
    would not be exact: those masks are left out)."""
    rng = np.random.default_rng(seed)
    (M, K), N = Aw.shape, Bw.shape[0]
    mant = 10 if fmt == orc.FP16 else 7
    masks = [0x8000, 1 << mant, 1 << (mant + 1), 1 << (mant - 1), 1 << (mant - 2), 1 << (mant - 3),
             (1 << mant) | 0x8000, 3 << (mant - 2)]
    A = orc.decode_array(Aw.ravel(), fmt).reshape(Aw.shape)
    B = orc.decode_array(Bw.ravel(), fmt).reshape(Bw.shape)
    rows = []
    while len(rows) < n:
        i, j, k = int(rng.integers(M)), int(rng.integers(N)), int(rng.integers(K))
        m = masks[int(rng.integers(len(masks)))]
        if A[i, k] * B[j, k] == 0 and fmt == orc.FP16 and m != 0x8000:
            continue
        rows.append((orc.SITE_PRODUCT, i, j, k, m))
    rows += [(orc.SITE_PRODUCT, M - 1, N - 1, K - 1, 0x8000), (orc.SITE_PRODUCT, 0, 0, 0, 0x8000),
             (orc.SITE_PRODUCT, M - 1, 0, 15, 1 << mant), (orc.SITE_PRODUCT, 0, N - 1, 16, 1 << mant),
             (orc.SITE_PRODUCT, M, 0, 0, 1), (orc.SITE_PRODUCT, 0, 0, K, 1), (orc.SITE_NONE, 0, 0, 0, 0)]
    return orc.make_faults(rows)


@pytest.mark.parametrize("fmt", [orc.FP16, orc.BF16])
@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4, 5, 6])
@pytest.mark.parametrize("shape", [(300, 200, 192, 32), (257, 65, 128, 64), (96, 40, 96, 48), (64, 64, 64, 16)])
def test_exact_regime_product_faults_bit_equal(fmt, cfg, shape):
    M, N, K, kb = shape
    Aw, Bw = wl.small_integers(M, N, K, fmt, seed=M + N + 1, lim=4, step=2)
    faults = _safe_product_faults(Aw, Bw, fmt, 30, seed=K + cfg)
    plan = gu.make_plan(Aw, Bw, kb, fmt, cfg=cfg, group=3)
    p = orc.problem(M, N, K, kb, fmt)
    for policy in (orc.CORRECT_NONE, orc.CORRECT_RECOMPUTE):
        recs, cout = gu.gpu_campaign(plan, faults, policy, want_c=True)
        ora = orc.campaign(p, Aw, Bw, faults, policy, orc.MODE_AFFECTED)
        for t in range(len(faults)):
            o, cf, cc = orc.trial(p, Aw, Bw, faults[t:t + 1], policy, orc.MODE_FULL, want_outputs=True)
            assert np.array_equal(cout[t].view(np.uint32), cc.view(np.uint32)), (t, faults[t])
            for name in ("n_flagged", "n_bitdiff", "n_dev_pre", "n_dev_post"):
                assert int(recs[t][name]) == int(o[name]), (name, t, faults[t])
        s = gu.compare_records(recs, ora, faults, exact_words=True)
        assert not s["mismatches"], s["mismatches"][:5]
        assert s["gpu_counts"] == s["oracle_counts"]
    plan.destroy()


@pytest.mark.parametrize("nbits", [1, 2, 4])
@pytest.mark.parametrize("fmt", [orc.FP16, orc.BF16])
def test_product_fault_campaign_random_operands(fmt, nbits):
    # ReLU-like activations (half zeros) as in the paper's CNNs (Sec. V-B scenario i), 1 / 2 / 4-bit
    # masks (Sec. IV-C), sites from the product sampler.
    base = wl.resnet_conv()
    A, B = wl.gaussian(384, 192, 256, fmt, seed=50 + nbits)
    Af = orc.decode_array(A.ravel(), fmt).reshape(A.shape)
    A = wl.to_words(np.maximum(Af, 0), fmt)
    w = dataclasses.replace(base, name="product_%d" % nbits, M=384, N=192, K=256, kb=32, fmt=fmt, A=A, B=B,
                            n_trials=3000, kind_mode=fi.KIND_ALL_PRODUCT, nbits=nbits,
                            policies=(wl.CORRECT_ZERO,), fault_seed=7 + nbits)
    s = _campaign_parity(w)[wl.CORRECT_ZERO]
    assert sum(s["gpu_counts"]) == 3000 and s["gpu_counts"][0] > 0 and s["gpu_counts"][2] > 0


def test_product_fault_campaign_one_trial_kernel_ragged_k():
    # K = 96 is not a multiple of the 64-wide k-tile: every trial takes the one-trial kernel.
    base = wl.tiny()
    A, B = wl.gaussian(130, 70, 96, orc.BF16, seed=61)
    w = dataclasses.replace(base, name="product_k96", M=130, N=70, K=96, kb=48, fmt=orc.BF16, A=A, B=B,
                            n_trials=1200, kind_mode=fi.KIND_ALL_PRODUCT, nbits=1,
                            policies=(wl.CORRECT_RECOMPUTE,), fault_seed=3)
    _campaign_parity(w)
    for cfg in (0, 1, 2):
        _campaign_parity(dataclasses.replace(w, n_trials=300), cfg=cfg)


def test_zero_difference_statistic_fp16_versus_bf16():
    # Table III's statistic: the share of trials whose destination register is unchanged by the
    # write-back.  On half-zero activations FP16 turns zeros into non-zeros far more often.
    share = {}
    for fmt in (orc.FP16, orc.BF16):
        A, B = wl.gaussian(256, 128, 256, fmt, seed=70)
        Af = orc.decode_array(A.ravel(), fmt).reshape(A.shape)
        A = wl.to_words(np.maximum(Af, 0), fmt)
        plan = gu.make_plan(A, B, 64, fmt)
        faults = fi.fi_sample_faults(5, 0, 4000, plan.desc, fi.KIND_ALL_PRODUCT, 1)
        recs = gu.gpu_campaign(plan, faults, fi.CORRECT_NONE)
        p = orc.problem(256, 128, 256, 64, fmt)
        ora = orc.campaign(p, A, B, gu.to_orc_faults(faults), orc.CORRECT_NONE, orc.MODE_AFFECTED)
        g = float(np.mean(recs["site_word_before"] == recs["site_word_after"]))
        o = float(np.mean(ora["site_word_before"] == ora["site_word_after"]))
        assert abs(g - o) < 0.02, (g, o)
        share[fmt] = g
        plan.destroy()
    assert share[orc.BF16] > share[orc.FP16] + 0.1


@pytest.mark.parametrize("fmt", [orc.FP16, orc.BF16])
@pytest.mark.parametrize("cfg", [0, 5])
@pytest.mark.parametrize("mode", [fi.PCHECK_BOUND, fi.PCHECK_RANGE_MAX, fi.PCHECK_RANGE_FLIP])
def test_exponent_only_checks_exact_regime(fmt, cfg, mode):
    # Sec. VI-A techniques applied to the erroneous product before the write-back.  Masks hit the
    # product's exponent bits: uncorrected values would leave the exact regime, corrected ones
    # (RangeCheck: at most 2^(e1+e2+1); BoundCheck: below 2^17) stay small dyadic numbers.
    M, N, K, kb = 200, 136, 128, 32
    Aw, Bw = wl.small_integers(M, N, K, fmt, seed=5, lim=4, step=2)
    A = orc.decode_array(Aw.ravel(), fmt).reshape(Aw.shape)
    B = orc.decode_array(Bw.ravel(), fmt).reshape(Bw.shape)
    rng = np.random.default_rng(mode * 10 + cfg)
    mant, ebits = (10, 5) if fmt == orc.FP16 else (7, 8)
    rows = []
    while len(rows) < 40:
        i, j, k = int(rng.integers(M)), int(rng.integers(N)), int(rng.integers(K))
        if A[i, k] * B[j, k] == 0:
            continue
        bit = mant + int(rng.integers(1, ebits))            # an exponent bit above the lowest
        w = orc.round16(float(A[i, k] * B[j, k]), fmt)
        if (w >> bit) & 1:                                     # flipping it down shrinks the value: fine too
            pass
        cw, fired = orc.product_check(w ^ (1 << bit), int(Aw[i, k]), int(Bw[j, k]), fmt, mode)
        if not fired and abs(orc.decode16(cw, fmt)) > 4096:    # uncorrected and huge: outside the exact regime
            continue
        rows.append((orc.SITE_PRODUCT, i, j, k, 1 << bit))
    faults = orc.make_faults(rows)
    plan = gu.make_plan(Aw, Bw, kb, fmt, cfg=cfg)
    plan.set_product_check(mode)
    p = orc.problem(M, N, K, kb, fmt, product_check=mode)
    recs, cout = gu.gpu_campaign(plan, faults, orc.CORRECT_NONE, want_c=True)
    ora = orc.campaign(p, Aw, Bw, faults, orc.CORRECT_NONE, orc.MODE_AFFECTED)
    assert np.array_equal(recs["product_flag"], ora["product_flag"])
    if not (fmt == orc.FP16 and mode == fi.PCHECK_BOUND):
        assert recs["product_flag"].sum() > 0
    for t in range(len(faults)):
        o, cf, cc = orc.trial(p, Aw, Bw, faults[t:t + 1], orc.CORRECT_NONE, orc.MODE_FULL, want_outputs=True)
        assert np.array_equal(cout[t].view(np.uint32), cc.view(np.uint32)), (t, faults[t])
    s = gu.compare_records(recs, ora, faults, exact_words=True)
    assert not s["mismatches"], s["mismatches"][:5]
    plan.set_product_check(fi.PCHECK_NONE)
    recs0 = gu.gpu_campaign(plan, faults, orc.CORRECT_NONE)
    assert recs0["product_flag"].sum() == 0
    with pytest.raises(fi.FiError):
        plan.set_product_check(7)
    plan.destroy()


def test_exponent_only_checks_confine_the_deviation_on_a_campaign():
    # Fig. 9's claim on synthetic operands: 4-bit faults in BF16 products; with a technique applied
    # the worst difference is bounded, and GPU and oracle agree trial by trial.
    fmt = orc.BF16
    A, B = wl.gaussian(256, 128, 256, fmt, seed=90)
    plan = gu.make_plan(A, B, 64, fmt)
    faults = fi.fi_sample_faults(9, 0, 3000, plan.desc, fi.KIND_ALL_PRODUCT, 4)
    ra, cb, _ = orc.rowcol_absmax(orc.problem(256, 128, 256, 64, fmt), A, B)
    site_tol = 2.0 ** -12 * 256 * float(ra.max()) * float(cb.max())
    worst = {}
    for mode in (fi.PCHECK_NONE, fi.PCHECK_BOUND, fi.PCHECK_RANGE_MAX, fi.PCHECK_RANGE_FLIP):
        plan.set_product_check(mode)
        recs = gu.gpu_campaign(plan, faults, fi.CORRECT_NONE)
        p = orc.problem(256, 128, 256, 64, fmt, product_check=mode)
        ora = orc.campaign(p, A, B, gu.to_orc_faults(faults), orc.CORRECT_NONE, orc.MODE_AFFECTED)
        assert np.array_equal(recs["product_flag"], ora["product_flag"])
        s = gu.compare_records(recs, ora, faults, site_tol=site_tol)
        assert not s["mismatches"], s["mismatches"][:5]
        worst[mode] = float(recs["max_dev_pre"].max())
        print("product check", mode, "fired", int(recs["product_flag"].sum()), "worst deviation", worst[mode],
              "classes", s["gpu_counts"])
    assert worst[fi.PCHECK_NONE] > 1e30
    assert worst[fi.PCHECK_BOUND] < 2.0 ** 18
    assert worst[fi.PCHECK_RANGE_MAX] < 1e3 and worst[fi.PCHECK_RANGE_FLIP] < 1e3
    plan.destroy()


def test_deviation_histogram_kernel():
    # Fig. 7 / Fig. 9 analogue: log2-binned per-trial differences.  The kernel must bin its own
    # records exactly as the definition says; against the oracle's campaign the histograms agree up
    # to trials that sit on a bin edge or whose low accumulator bits differ.
    import torch
    fmt = orc.BF16
    A, B = wl.gaussian(128, 128, 128, fmt, seed=95)
    plan = gu.make_plan(A, B, 64, fmt)
    n = 5000
    faults = fi.fi_sample_faults(2, 0, n, plan.desc, fi.KIND_ALL_PRODUCT, 2)
    faults[7]["row"] = 10 ** 6                                   # an invalid site: skipped
    d_f = fi.to_device(faults)
    d_r = fi.empty_results(n)
    plan.fi_gemm_inject_batch(d_f, n, fi.CORRECT_ZERO, d_r)
    recs = fi.results_to_host(d_r)
    p = orc.problem(128, 128, 128, 64, fmt)
    ofaults = gu.to_orc_faults(faults)
    ora = orc.campaign(p, A, B, ofaults, orc.CORRECT_ZERO, orc.MODE_AFFECTED)
    d_h = torch.zeros(256, dtype=torch.int64, device="cuda")
    for which in (fi.HIST_SITE, fi.HIST_DEV_PRE, fi.HIST_DEV_POST):
        plan.fi_deviation_histogram(d_f, d_r, n, which, d_h)
        h = d_h.cpu().numpy().astype(np.uint64)
        # the same records through the oracle's histogram (its record layout)
        mine = np.zeros(n, orc.RECORD_DTYPE)
        for k in ("site_word_before", "site_word_after", "max_dev_pre", "max_dev_post"):
            mine[k] = recs[k]
        mine["valid"] = (recs["status"] == 0)
        assert np.array_equal(h, orc.deviation_histogram(mine, ofaults, which)), which
        assert int(h.sum()) == n - 1
        ho = orc.deviation_histogram(ora, ofaults, which)
        assert int(np.abs(h.astype(np.int64) - ho.astype(np.int64)).sum()) <= 0.02 * n, which
        print("histogram", which, "zero bin", int(h[0]), "Inf/NaN bin", int(h[255]),
              "median bin", int(np.searchsorted(np.cumsum(h), h.sum() / 2)))
    with pytest.raises(fi.FiError):
        plan.fi_deviation_histogram(d_f, d_r, n, 3, d_h)
    plan.destroy()
