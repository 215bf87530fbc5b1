"""GPU tests of what include/fi.h promises about plans: handles, streams, scratch, the default
slack for long K and the guard of the affected-tiles-only campaign."""
import ctypes as C

import numpy as np
import pytest

from oracle import pyoracle as orc
from paper_2311_05782_amd import fi, workloads as wl
import gpu_util as gu

pytestmark = pytest.mark.gpu


def test_a_destroyed_plan_is_refused_not_read():
    Aw, Bw = wl.gaussian(64, 64, 64, orc.BF16, seed=1)
    plan = gu.make_plan(Aw, Bw, 32, orc.BF16)
    h = C.c_void_p(plan.handle.value)
    plan.destroy()
    L = fi.lib()
    assert L.fi_plan_destroy(h) == fi.STATE
    out = C.c_void_p()
    assert L.fi_plan_buffer(h, 0, C.byref(out)) == fi.STATE
    assert L.fi_plan_reserve(h, 8, None) == fi.STATE


def test_batches_of_one_plan_in_flight_on_two_streams_do_not_share_scratch():
    import torch
    w = wl.detector_stress()
    plan = gu.make_plan(w.A, w.B, w.kb, w.fmt)
    n = 2048
    fa = fi.fi_sample_faults(1, 0, n, plan.desc, fi.KIND_MIX_ACC_A, 1)
    fb = fi.fi_sample_faults(2, 0, n, plan.desc, fi.KIND_ALL_B, 2)
    d_fa, d_fb = fi.to_device(fa), fi.to_device(fb)
    want_a = gu.gpu_campaign(plan, fa, wl.CORRECT_ZERO)
    want_b = gu.gpu_campaign(plan, fb, wl.CORRECT_ZERO)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    plan.reserve(n, s1)
    plan.reserve(n, s2)
    r_a, r_b = fi.empty_results(n), fi.empty_results(n)
    torch.cuda.synchronize()
    for _ in range(3):
        # each batch runs for milliseconds: the second is enqueued while the first is running
        plan.fi_gemm_inject_batch(d_fa, n, wl.CORRECT_ZERO, r_a, stream=s1)
        plan.fi_gemm_inject_batch(d_fb, n, wl.CORRECT_ZERO, r_b, stream=s2)
        torch.cuda.synchronize()
        assert fi.results_to_host(r_a).tobytes() == want_a.tobytes()
        assert fi.results_to_host(r_b).tobytes() == want_b.tobytes()
    plan.destroy()


def test_reserve_then_capture_without_an_eager_call_first():
    import torch
    w = wl.tiny()
    plan = gu.make_plan(w.A, w.B, w.kb, w.fmt)
    n = 200
    faults = fi.fi_sample_faults(9, 0, n, plan.desc, fi.KIND_MIX_ACC_A, 1)
    d_f, d_r = fi.to_device(faults), fi.empty_results(n)
    side = torch.cuda.Stream()
    plan.reserve(n, side)                      # no batch has run on `side` yet
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            plan.fi_gemm_inject_batch(d_f, n, fi.CORRECT_ZERO, d_r, stream=torch.cuda.current_stream().cuda_stream)
    want = gu.gpu_campaign(plan, faults, fi.CORRECT_ZERO)
    for rep in range(3):
        d_r.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert fi.results_to_host(d_r).tobytes() == want.tobytes(), rep
    plan.destroy()


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4, 5, 6])
@pytest.mark.parametrize("fmt", [orc.FP16, orc.BF16])
def test_rows_of_all_maximal_same_sign_products_are_never_flagged(cfg, fmt):
    # The worst case for "a clean element is not flagged": every product of a row equals
    # ra_i * cb_j with one sign, so the exact sum IS K * ra_i * cb_j and only the slack factor
    # separates it from the bound.  K = 4096 with the default slack, every tile shape.
    M, N, K, kb = 160, 136, 4096, 64
    rng = np.random.default_rng(cfg)
    mant = rng.integers(128, 256, size=M) / 128.0            # 8 significant bits: exact in both formats
    a = np.repeat(mant[:, None], K, axis=1).astype(np.float32)
    a[::3] *= -1
    b = np.repeat((rng.integers(128, 256, size=N) / 128.0)[:, None], K, axis=1).astype(np.float32)
    Aw, Bw = wl.to_words(a, fmt), wl.to_words(b, fmt)
    plan = gu.make_plan(Aw, Bw, kb, fmt, cfg=cfg)
    faults = orc.make_faults([(orc.SITE_NONE, 0, 0, 0, 0)] * 3)
    recs = gu.gpu_campaign(plan, faults, wl.CORRECT_ZERO)
    assert not recs["n_flagged"].any() and not recs["n_bitdiff"].any() and not recs["n_dev_pre"].any()
    # and the fault-free result sits right under the bound (so the test has teeth)
    cs = np.abs(plan.buffer_to_host(fi.BUF_C_STAR))
    T = np.float32(K) * np.abs(a[:, :1]) * np.abs(b[:, 0])[None, :]
    assert np.all(cs <= T * np.float32(1 + 2.0 ** -11)) and np.all(cs >= T * np.float32(1 - 2.0 ** -11))
    plan.destroy()


def test_default_slack_for_long_K_matches_the_oracle_and_keeps_clean_trials_masked():
    M, N, K, kb, fmt = 40, 72, 8192, 64, orc.BF16
    a = np.full((M, K), 143.0 / 128.0, np.float32)           # sums that round upwards step after step
    b = np.full((N, K), 143.0 / 128.0, np.float32)
    a[5:9] = np.random.default_rng(0).standard_normal((4, K)).astype(np.float32)
    Aw, Bw = wl.to_words(a, fmt), wl.to_words(b, fmt)
    plan = gu.make_plan(Aw, Bw, kb, fmt)
    p = orc.problem(M, N, K, kb, fmt)
    assert p.gamma == np.float32(1 + 2.0 ** -10)
    faults = fi.fi_sample_faults(3, 0, 64, plan.desc, fi.KIND_ALL_ACC, 1)
    faults[:4]["kind"] = 0
    recs = gu.gpu_campaign(plan, faults, wl.CORRECT_ZERO)
    ora = orc.campaign(p, Aw, Bw, gu.to_orc_faults(faults), wl.CORRECT_ZERO, orc.MODE_AFFECTED)
    assert not recs["n_flagged"][:4].any()
    ra, cb, _ = orc.rowcol_absmax(p, Aw, Bw)
    s = gu.compare_records(recs, ora, faults, site_tol=2.0 ** -12 * K * float(ra.max()) * float(cb.max()))
    assert not s["mismatches"], s["mismatches"][:5]
    plan.destroy()


def test_affected_only_campaign_refuses_a_plan_whose_clean_result_is_flagged():
    # Under the exponent-only bound any |C*| >= 2^17 is flagged in every trial of a full campaign;
    # the affected-tiles-only campaign would never visit it, so it must refuse.
    M, N, K, kb, fmt = 64, 64, 64, 32, orc.BF16
    Aw, Bw = wl.small_integers(M, N, K, fmt, seed=3, lim=2, step=1)
    big = wl.to_words(np.full(K, 64.0, np.float32), fmt)
    Aw = Aw.copy(); Bw = Bw.copy()
    Aw[7, :] = big; Bw[9, :] = big                           # C*[7, 9] = 64 * 64 * 64 = 2^18
    plan = gu.make_plan(Aw, Bw, kb, fmt, bound_mode=fi.BOUND_EXPONENT)
    p = orc.problem(M, N, K, kb, fmt, bound_mode=orc.BOUND_EXPONENT)
    faults = orc.make_faults([(orc.SITE_NONE, 0, 0, 0, 0), (orc.SITE_ACC, 1, 1, 0, 1 << 22),
                              (orc.SITE_ACC, 7, 9, 1, 1 << 31)])
    recs = gu.gpu_campaign(plan, faults, wl.CORRECT_ZERO)
    for t in range(len(faults)):
        o = orc.trial(p, Aw, Bw, faults[t:t + 1], wl.CORRECT_ZERO, orc.MODE_FULL)
        assert int(recs["n_flagged"][t]) == int(o["n_flagged"]) >= 1, t
    d_r = fi.empty_results(len(faults))
    with pytest.raises(fi.FiError) as e:
        plan.fi_gemm_inject_batch_affected(fi.to_device(faults), len(faults), wl.CORRECT_ZERO, d_r)
    assert e.value.status == fi.UNSUPPORTED
    plan.destroy()
    # the same operands under the operand-derived bound: nothing clean is flagged, the call works
    plan = gu.make_plan(Aw, Bw, kb, fmt)
    plan.fi_gemm_inject_batch_affected(fi.to_device(faults), len(faults), wl.CORRECT_ZERO, d_r)
    assert fi.results_to_host(d_r).tobytes() == gu.gpu_campaign(plan, faults, wl.CORRECT_ZERO).tobytes()
    plan.destroy()


def test_operands_ending_at_the_end_of_their_allocation_short_K():
    # K = 16 and 48 with packed rows: the one-trial kernel's k-tile is 64 wide, so chunks past K
    # must be fetched from inside the row.  The operands sit at the very end of their buffers.
    import torch
    fmt = orc.BF16
    for (M, N, K, kb) in [(128, 128, 16, 16), (130, 70, 48, 16)]:
        Aw, Bw = wl.small_integers(M, N, K, fmt, seed=K, lim=2, step=1)
        pool_a = torch.zeros(M * K + 4096, dtype=torch.int16, device="cuda")
        pool_b = torch.zeros(N * K + 4096, dtype=torch.int16, device="cuda")
        d_A = pool_a[4096:].view(M, K); d_B = pool_b[4096:].view(N, K)
        d_A.copy_(fi.words_to_device(Aw)); d_B.copy_(fi.words_to_device(Bw))
        plan = fi.Plan(fi.plan_desc(M, N, K, kb, fmt), d_A, d_B)
        p = orc.problem(M, N, K, kb, fmt)
        assert np.array_equal(plan.buffer_to_host(fi.BUF_C_STAR).view(np.uint32), orc.gemm(p, Aw, Bw).view(np.uint32))
        faults = orc.make_faults([(orc.SITE_ACC, M - 1, N - 1, K // kb - 1, 1 << 30), (orc.SITE_A, M - 1, K - 1, 0, 0x8000),
                                  (orc.SITE_B, K - 1, N - 1, 0, 0x8000), (orc.SITE_PRODUCT, 1, 2, K - 1, 0x4000)])
        recs = gu.gpu_campaign(plan, faults, wl.CORRECT_RECOMPUTE)
        ora = orc.campaign(p, Aw, Bw, faults, wl.CORRECT_RECOMPUTE, orc.MODE_AFFECTED)
        s = gu.compare_records(recs, ora, faults, exact_words=True)
        assert not s["mismatches"], s["mismatches"]
        plan.destroy()
