"""GPU parity: the HIP path, called through the C-ABI binding, against the CPU oracle on the
same seeded inputs.  Integer results (sites, words, flags, counters, classes) must be equal;
where FP32 summation order can matter the rule is the guard-banded one in gpu_util."""
import os

import numpy as np
import pytest

from oracle import pyoracle as orc
from paper_2311_05782_amd import fi, workloads as wl
import gpu_util as gu

pytestmark = pytest.mark.gpu


def test_one_hip_runtime_and_native_library_loaded():
    import torch
    assert torch.cuda.is_available()
    fi.lib()
    maps = open("/proc/self/maps").read()
    hips = {ln.split()[-1] for ln in maps.splitlines() if "libamdhip64" in ln}
    assert len(hips) == 1, hips
    assert any("libfi_gfx950.so" in ln for ln in maps.splitlines())


def _mixed_faults(Aw, Bw, fmt, kb, n, seed):
    """Accumulator, A, B and fault-free trials for the exact regime, with sites forced into
    tile corners and ragged tails.  Operands are even integers, so accumulators are 0 or at
    least 4 in magnitude; accumulator bits 12..31 and operand masks that turn a word into
    another small integer, 64 or Inf keep every partial sum exactly representable, or send
    it so far up that the later terms vanish under every summation order.  Bit 30 sends a
    non-zero accumulator DOWN to about 2^-126: such a residue under later products is outside
    the exact regime (the oracle's sequential round-to-nearest adds absorb it; the matrix
    core aligns the incoming accumulator to the step's largest product and rounds it down:
    -2^-126 plus products that sum to 4 gave 4 - 2^-20), so those flips go to the last
    k-block, where nothing is added afterwards."""
    rng = np.random.default_rng(seed)
    (M, K), N = Aw.shape, Bw.shape[0]
    S = K // kb
    targets = wl.to_words(np.array([0, 2, -2, 4, -4, 64, np.inf, -np.inf], np.float32), fmt)

    def op_mask(word):
        return int(word) ^ int(targets[rng.integers(len(targets))])

    rows = []
    for t in range(n):
        kind = [orc.SITE_ACC, orc.SITE_ACC, orc.SITE_A, orc.SITE_B, orc.SITE_NONE][t % 5]
        if kind == orc.SITE_ACC:
            i, j, s, bit = rng.integers(M), rng.integers(N), rng.integers(S), int(rng.integers(12, 32))
            r = (kind, i, j, S - 1 if bit == 30 else s, 1 << bit)
        elif kind == orc.SITE_A:
            i, k = rng.integers(M), rng.integers(K)
            r = (kind, i, k, 0, op_mask(Aw[i, k]))
        elif kind == orc.SITE_B:
            k, j = rng.integers(K), rng.integers(N)
            r = (kind, k, j, 0, op_mask(Bw[j, k]))
        else:
            r = (kind, 0, 0, 0, 0)
        rows.append(r)
    # corners and last elements
    rows += [(orc.SITE_ACC, M - 1, N - 1, S - 1, 1 << 31), (orc.SITE_ACC, 0, 0, 0, 1 << 23),
             (orc.SITE_ACC, M - 1, 0, S - 1, 0x00C00000), (orc.SITE_ACC, 0, N - 1, 0, 1 << 31),
             (orc.SITE_ACC, 0, N - 1, S - 1, 1 << 30),
             (orc.SITE_A, M - 1, K - 1, 0, 0x8000), (orc.SITE_B, K - 1, N - 1, 0, 0x8000),
             (orc.SITE_A, 0, 0, 0, 0x18000 | op_mask(Aw[0, 0])), (orc.SITE_B, 0, 0, 0, op_mask(Bw[0, 0]))]
    return orc.make_faults(rows)


@pytest.mark.parametrize("fmt", [orc.FP16, orc.BF16])
@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4, 5, 6])
@pytest.mark.parametrize("shape", [(300, 200, 192, 32), (257, 65, 128, 64), (96, 40, 96, 48), (64, 64, 64, 16)])
def test_exact_regime_everything_bit_equal(fmt, cfg, shape):
    # Small-integer operands: every partial sum is exact, so summation order cannot matter and
    # outputs, words, flags and counters must all be identical.  Shapes span several tiles and
    # ragged tails in M, N and K (K = 96 is not a multiple of the 64-wide k-tile).
    M, N, K, kb = shape
    Aw, Bw = wl.small_integers(M, N, K, fmt, seed=M + N, lim=4, step=2)
    faults = _mixed_faults(Aw, Bw, fmt, kb, 25, seed=K + cfg)
    plan = gu.make_plan(Aw, Bw, kb, fmt, cfg=cfg, group=5)
    p = orc.problem(M, N, K, kb, fmt)
    gold = orc.gemm(p, Aw, Bw)
    assert np.array_equal(plan.buffer_to_host(fi.BUF_C_STAR).view(np.uint32), gold.view(np.uint32))
    for policy in (orc.CORRECT_NONE, orc.CORRECT_ZERO, orc.CORRECT_RECOMPUTE):
        recs, cout = gu.gpu_campaign(plan, faults, policy, want_c=True)
        for t in range(len(faults)):
            o, cf, cc = orc.trial(p, Aw, Bw, faults[t:t + 1], policy, orc.MODE_FULL, want_outputs=True)
            nan = np.isnan(cc)
            assert np.array_equal(np.isnan(cout[t]), nan), (t, faults[t])
            assert np.array_equal(cout[t][~nan].view(np.uint32), cc[~nan].view(np.uint32)), (t, faults[t])
            g = recs[t]
            for k in ("n_flagged", "n_dev_pre", "n_dev_post", "site_word_before", "site_word_after"):
                assert int(g[k]) == int(o[k]), (k, t, faults[t], int(g[k]), int(o[k]))
            if not nan.any():
                assert int(g["n_bitdiff"]) == int(o["n_bitdiff"]), (t, faults[t])
            assert np.float32(g["max_dev_pre"]) == np.float32(o["max_dev_pre"]), (t, faults[t])
            assert np.float32(g["max_dev_post"]) == np.float32(o["max_dev_post"]), (t, faults[t])
            assert int(g["status"]) == 0
    plan.destroy()


def test_exact_regime_random_shapes_formats_blocks_and_tile_shapes():
    # Sixty seeded draws of (format, M, N, K, k-block, tile configuration, trial group, batch size,
    # policy, outputs or not): shapes of one row or column up to several ragged tiles, K from one
    # 16-wide step up to 320, every k-block that divides K.  Everything bit for bit, as above.
    rng = np.random.default_rng(2311)
    for case in range(60):
        fmt = [orc.FP16, orc.BF16][int(rng.integers(2))]
        M, N = int(rng.integers(1, 420)), int(rng.integers(1, 330))
        steps = int(rng.integers(1, 21))
        K = 16 * steps
        divisors = [d for d in range(1, steps + 1) if steps % d == 0]
        kb = 16 * divisors[int(rng.integers(len(divisors)))]
        cfg, group = int(rng.integers(-1, 7)), int(rng.integers(1, 9))
        n, policy, want_c = int(rng.integers(1, 50)), int(rng.integers(3)), bool(rng.integers(2))
        what = (case, fmt, M, N, K, kb, cfg, group, n, policy, want_c)
        Aw, Bw = wl.small_integers(M, N, K, fmt, seed=case + 100, lim=4, step=2)
        faults = _mixed_faults(Aw, Bw, fmt, kb, n, seed=case)
        plan = gu.make_plan(Aw, Bw, kb, fmt, cfg=None if cfg < 0 else cfg, group=group)
        p = orc.problem(M, N, K, kb, fmt)
        got = gu.gpu_campaign(plan, faults, policy, want_c=want_c)
        recs, cout = got if want_c else (got, None)
        for t in range(len(faults)):
            o, cf, cc = orc.trial(p, Aw, Bw, faults[t:t + 1], policy, orc.MODE_FULL, want_outputs=True)
            nan = np.isnan(cc)
            g = recs[t]
            for k in ("n_flagged", "n_dev_pre", "n_dev_post", "site_word_before", "site_word_after"):
                assert int(g[k]) == int(o[k]), (k, t, faults[t], int(g[k]), int(o[k]), what)
            if not nan.any():
                assert int(g["n_bitdiff"]) == int(o["n_bitdiff"]), (t, faults[t], what)
            assert np.float32(g["max_dev_pre"]) == np.float32(o["max_dev_pre"]), (t, faults[t], what)
            assert np.float32(g["max_dev_post"]) == np.float32(o["max_dev_post"]), (t, faults[t], what)
            if want_c:
                assert np.array_equal(np.isnan(cout[t]), nan), (t, faults[t], what)
                assert np.array_equal(cout[t][~nan].view(np.uint32), cc[~nan].view(np.uint32)), (t, faults[t], what)
        plan.destroy()


def test_random_gaussian_campaigns_by_the_guard_band_rule():
    # 150 seeded draws of (format, shape, k-block, tile configuration, trial group, batch size,
    # policy, fault kinds, bits per fault, output-side detector, product check) on Gaussian
    # operands, one invalid site per batch: records against the oracle's by the parity rule.
    rng = np.random.default_rng(57820)
    for case in range(150):
        fmt = [orc.FP16, orc.BF16][int(rng.integers(2))]
        M, N = int(rng.integers(1, 300)), int(rng.integers(1, 260))
        steps = int(rng.integers(1, 25))
        K = 16 * steps
        divisors = [d for d in range(1, steps + 1) if steps % d == 0]
        kb = 16 * divisors[int(rng.integers(len(divisors)))]
        cfg, group = int(rng.integers(-1, 7)), int(rng.integers(1, 9))
        n, policy = int(rng.integers(1, 200)), int(rng.integers(3))
        kind_mode, nbits = int(rng.integers(5)), [1, 2, 4][int(rng.integers(3))]
        bound, pcheck = int(rng.integers(3)), int(rng.integers(4))
        what = (case, fmt, M, N, K, kb, cfg, group, n, policy, kind_mode, nbits, bound, pcheck)
        Aw, Bw = wl.gaussian(M, N, K, fmt, seed=case + 11)
        plan = gu.make_plan(Aw, Bw, kb, fmt, cfg=None if cfg < 0 else cfg, group=group, bound_mode=bound)
        plan.set_product_check(pcheck)
        faults = fi.fi_sample_faults(case, 0, n, plan.desc, kind_mode, nbits)
        if n > 3:
            faults[3]["row"] = 10 ** 7
        p = orc.problem(M, N, K, kb, fmt, bound_mode=bound, product_check=pcheck)
        recs = gu.gpu_campaign(plan, faults, policy)
        ora = orc.campaign(p, Aw, Bw, gu.to_orc_faults(faults), policy, orc.MODE_AFFECTED)
        ra, cb, _ = orc.rowcol_absmax(p, Aw, Bw)
        s = gu.compare_records(recs, ora, faults, site_tol=2.0 ** -12 * K * float(ra.max()) * float(cb.max()))
        assert not s["mismatches"], (s["mismatches"][:5], what)
        assert np.array_equal(recs["product_flag"], ora["product_flag"]), what
        plan.destroy()


def _check_unfaulted(plan, Aw, Bw, fmt, rows=None):
    A = orc.decode_array(Aw, fmt).astype(np.float64)
    Bt = orc.decode_array(Bw, fmt).astype(np.float64)
    if rows is not None:
        A = A[rows]
    R = A @ Bt.T
    S = np.abs(A) @ np.abs(Bt).T
    Cg = plan.buffer_to_host(fi.BUF_C_STAR)
    Sg = plan.buffer_to_host(fi.BUF_S_ABS)
    if rows is not None:
        Cg, Sg = Cg[rows], Sg[rows]
    # the stated tolerance for fault-free outputs
    assert np.all(np.abs(Cg.astype(np.float64) - R) <= 2.0 ** -12 * S)
    assert np.all(np.abs(Sg.astype(np.float64) - S) <= 2.0 ** -12 * S)
    return float(np.max(np.abs(Cg - R) / np.maximum(S, 1e-300)))


def _campaign_parity(w, n_trials=None, cfg=None, policies=None, rows_check=None):
    fmt = w.fmt
    n = n_trials or w.n_trials
    plan = gu.make_plan(w.A, w.B, w.kb, fmt, cfg=cfg)
    desc = plan.desc
    faults = fi.fi_sample_faults(w.fault_seed, 0, n, desc, w.kind_mode, w.nbits)
    p = orc.problem(w.M, w.N, w.K, w.kb, fmt)
    ofaults = orc.sample_faults(w.fault_seed, 0, n, p, w.kind_mode, w.nbits)
    assert faults.tobytes() == ofaults.tobytes()          # site selection is bit-exact
    _check_unfaulted(plan, w.A, w.B, fmt, rows_check)
    ra, cb, finite = orc.rowcol_absmax(p, w.A, w.B)
    assert finite
    kra = plan.buffer_to_host(fi.BUF_KRA)
    assert np.array_equal(kra, (np.float32(w.K) * ra).astype(np.float32))
    assert np.array_equal(plan.buffer_to_host(fi.BUF_CB), cb)
    operands = (orc.decode_array(w.A, fmt), orc.decode_array(w.B, fmt))   # the element's own 2^-12 * S_ij
    out = {}
    for policy in (policies or w.policies):
        recs = gu.gpu_campaign(plan, faults, policy)
        ora = orc.campaign(p, w.A, w.B, ofaults, policy, orc.MODE_AFFECTED)
        s = gu.compare_records(recs, ora, faults, operands=operands)
        assert not s["mismatches"], s["mismatches"][:10]
        assert s["certain"] >= n - s["borderline"]
        # classification kernel against the records it was given
        d_r = fi.to_device(recs)
        cls, cnt = gu.gpu_classify(plan, d_r, n)
        assert np.array_equal(cls, gu.cls_of(recs)) and cnt.tolist() == s["gpu_counts"]
        ocls, ocnt = orc.classify(ora)
        # totals agree up to the borderline trials
        assert sum(abs(int(a) - int(b)) for a, b in zip(cnt, ocnt)) <= 2 * s["borderline"]
        out[policy] = s
        print(w.name, "policy", policy, s["gpu_counts"], s["oracle_counts"], "borderline", s["borderline"],
              "class compared on", s["certain"], "of", n)
    plan.destroy()
    return out


def test_tiny_campaign():
    s = _campaign_parity(wl.tiny())[wl.CORRECT_ZERO]
    assert sum(s["gpu_counts"]) == 64 and min(s["gpu_counts"]) > 0


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4, 5, 6])
def test_tiny_campaign_every_tile_shape_many_trials(cfg):
    w = wl.tiny()
    _campaign_parity(w, n_trials=1500, cfg=cfg, policies=(wl.CORRECT_ZERO, wl.CORRECT_RECOMPUTE, wl.CORRECT_NONE))


def test_bert_linear_campaign_full_size():
    _campaign_parity(wl.bert_linear())


def test_resnet_conv_campaign_full_size():
    _campaign_parity(wl.resnet_conv())


def test_detector_stress_campaign_full_size_both_policies():
    out = _campaign_parity(wl.detector_stress())
    z, r = out[wl.CORRECT_ZERO], out[wl.CORRECT_RECOMPUTE]
    assert z["gpu_counts"] == r["gpu_counts"]     # the class does not depend on the corrector


def test_square4096_campaign_full_size_launch_configuration_of_the_benchmark():
    # 1024 trials of 4096^3 in one launch; every trial is checked against the oracle, which
    # can compute each faulted element on its own.  Unfaulted outputs: every row of C* and S.
    _campaign_parity(wl.square4096())


def test_zero_fault_trials_are_masked_on_every_workload():
    for make in (wl.tiny, wl.bert_linear, wl.resnet_conv, wl.detector_stress):
        w = make()
        plan = gu.make_plan(w.A, w.B, w.kb, w.fmt)
        faults = orc.make_faults([(orc.SITE_NONE, 0, 0, 0, 0), (orc.SITE_ACC, 1, 1, 0, 0),
                                  (orc.SITE_A, 2, 3, 0, 0), (orc.SITE_NONE, 5, 5, 5, 5)])
        recs = gu.gpu_campaign(plan, faults, wl.CORRECT_ZERO)
        for k in ("n_flagged", "n_bitdiff", "n_dev_pre", "n_dev_post", "status"):
            assert not recs[k].any(), (w.name, k)
        assert not recs["max_dev_pre"].any() and (gu.cls_of(recs) == fi.MASKED).all()
        # the fault-free result does not depend on the workgroup tile: a clean trial run with any
        # other tile shape is still bit-identical to the plan's C*
        for cfg in (0, 1, 2, 3, 4, 5, 6):
            plan.tune(cfg, 3)
            recs = gu.gpu_campaign(plan, faults, wl.CORRECT_ZERO)
            assert not recs["n_bitdiff"].any() and not recs["n_flagged"].any(), (w.name, cfg)
        plan.destroy()


def test_out_of_range_sites_run_fault_free_and_say_so():
    w = wl.tiny()
    plan = gu.make_plan(w.A, w.B, w.kb, w.fmt)
    faults = orc.make_faults([(orc.SITE_ACC, 128, 0, 0, 1), (orc.SITE_ACC, 0, 128, 0, 1),
                              (orc.SITE_ACC, 0, 0, 4, 1), (orc.SITE_A, 0, 128, 0, 1),
                              (orc.SITE_B, 128, 0, 0, 1), (9, 0, 0, 0, 1), (orc.SITE_ACC, 5, 5, 1, 1 << 30)])
    recs = gu.gpu_campaign(plan, faults, wl.CORRECT_ZERO)
    assert recs["status"].tolist() == [1, 1, 1, 1, 1, 1, 0]
    assert not recs["n_bitdiff"][:6].any() and recs["n_bitdiff"][6] == 1
    plan.destroy()


def test_layouts_leading_dimensions_and_global_bound():
    M, N, K, kb, fmt = 200, 136, 128, 32, orc.FP16
    Aw, Bw = wl.gaussian(M, N, K, fmt, seed=12)
    p = orc.problem(M, N, K, kb, fmt)
    faults = fi.fi_sample_faults(5, 0, 200, fi.plan_desc(M, N, K, kb, fmt), fi.KIND_MIX_ACC_A, 1)
    of = gu.to_orc_faults(faults)
    base = gu.make_plan(Aw, Bw, kb, fmt)
    cbase = base.buffer_to_host(fi.BUF_C_STAR)
    rbase = gu.gpu_campaign(base, faults, wl.CORRECT_ZERO)
    # B given as K rows of N
    alt = gu.make_plan(Aw, np.ascontiguousarray(Bw.T), kb, fmt, b_layout=1)
    assert np.array_equal(alt.buffer_to_host(fi.BUF_C_STAR).view(np.uint32), cbase.view(np.uint32))
    assert gu.gpu_campaign(alt, faults, wl.CORRECT_ZERO).tobytes() == rbase.tobytes()
    # padded leading dimensions
    Ap = np.zeros((M, K + 8), np.uint16); Ap[:, :K] = Aw
    Bp = np.zeros((N, K + 16), np.uint16); Bp[:, :K] = Bw
    import torch
    dA, dB = fi.words_to_device(Ap), fi.words_to_device(Bp)
    pad = fi.Plan(fi.plan_desc(M, N, K, kb, fmt, lda=K + 8, ldb=K + 16), dA, dB)
    assert np.array_equal(pad.buffer_to_host(fi.BUF_C_STAR).view(np.uint32), cbase.view(np.uint32))
    assert gu.gpu_campaign(pad, faults, wl.CORRECT_ZERO).tobytes() == rbase.tobytes()
    # global bound against the oracle
    ops = (orc.decode_array(Aw, fmt), orc.decode_array(Bw, fmt))
    glob = gu.make_plan(Aw, Bw, kb, fmt, bound_mode=fi.BOUND_GLOBAL)
    pg = orc.problem(M, N, K, kb, fmt, bound_mode=orc.BOUND_GLOBAL)
    s = gu.compare_records(gu.gpu_campaign(glob, faults, wl.CORRECT_ZERO),
                           orc.campaign(pg, Aw, Bw, of, wl.CORRECT_ZERO), faults, operands=ops)
    assert not s["mismatches"], s["mismatches"][:5]
    s = gu.compare_records(rbase, orc.campaign(p, Aw, Bw, of, wl.CORRECT_ZERO), faults, operands=ops)
    assert not s["mismatches"], s["mismatches"][:5]
    for pl in (base, alt, pad, glob):
        pl.destroy()


def test_nonfinite_operands_are_a_plan_error():
    Aw, Bw = wl.gaussian(64, 64, 64, orc.BF16, seed=1)
    Aw = Aw.copy(); Aw[3, 9] = 0x7F80
    with pytest.raises(fi.FiError) as e:
        gu.make_plan(Aw, Bw, 32, orc.BF16)
    assert e.value.status == fi.INVALID_ARG


def test_plan_describe_names_the_kernels_in_use():
    Aw, Bw = wl.gaussian(128, 128, 128, orc.BF16, seed=2)
    plan = gu.make_plan(Aw, Bw, 64, orc.BF16)
    assert "gemm_fi_multi_kernel<bf16, R=8, 64x64" in plan.describe()      # a small problem
    plan.tune(5)
    assert "gemm_fi_multi_kernel<bf16, R=8, 128x64" in plan.describe()
    plan.tune(1)
    assert "one trial per item, 128x128, 256 threads, persistent x2 per CU" in plan.describe()
    plan.tune(2)
    assert plan.describe() == "gemm_fi_kernel<bf16, 256x64, 256 threads>"
    plan.tune(3)
    assert "R=4, 128x128" in plan.describe()
    plan.destroy()
    Aw, Bw = wl.gaussian(64, 64, 96, orc.FP16, seed=2)        # K % 64 != 0: front-padded operand copies
    plan = gu.make_plan(Aw, Bw, 32, orc.FP16)
    assert "gemm_fi_multi_kernel<fp16, R=8, 64x64" in plan.describe()
    plan.tune(5)
    assert "R=8, 128x64" in plan.describe()
    plan.destroy()


@pytest.mark.parametrize("N", [136, 130])
def test_standalone_detector_equals_fused_epilogue_and_oracle(N):
    import torch
    M, K, kb, fmt = 150, 128, 32, orc.FP16
    Aw, Bw = wl.gaussian(M, N, K, fmt, seed=3)
    p = orc.problem(M, N, K, kb, fmt)
    plan = gu.make_plan(Aw, Bw, kb, fmt)
    faults = fi.fi_sample_faults(8, 0, 64, plan.desc, fi.KIND_MIX_ACC_A, 2)
    faults["xor_mask"][::3] = 1 << 30            # plenty of exponent-MSB flips
    faults["xor_mask"][1::8] = 1 << 14           # FP16 operand exponent MSB: Inf / NaN rows
    raw_recs, raw = gu.gpu_campaign(plan, faults, wl.CORRECT_NONE, want_c=True)
    ra, cb, _ = orc.rowcol_absmax(p, Aw, Bw)
    cstar = plan.buffer_to_host(fi.BUF_C_STAR)
    for policy in (wl.CORRECT_ZERO, wl.CORRECT_RECOMPUTE, wl.CORRECT_NONE):
        fused_recs, fused = gu.gpu_campaign(plan, faults, policy, want_c=True)
        d_c = torch.from_numpy(raw.copy()).cuda()
        d_fl = torch.empty(raw.shape, dtype=torch.uint8, device="cuda")
        d_n = torch.empty(len(faults), dtype=torch.int32, device="cuda")
        plan.fi_detect_correct(d_c, len(faults), policy, d_fl, d_n)
        torch.cuda.synchronize()
        alone, flags, nfl = d_c.cpu().numpy(), d_fl.cpu().numpy(), d_n.cpu().numpy().astype(np.uint32)
        assert np.array_equal(nfl, fused_recs["n_flagged"]) and np.array_equal(nfl, raw_recs["n_flagged"])
        assert np.array_equal(alone.view(np.uint32), fused.view(np.uint32))
        oc, oflags, on = orc.detect_correct(p, ra, cb, raw, policy, c_star=cstar)
        assert np.array_equal(flags, oflags) and np.array_equal(nfl, on)
        assert np.array_equal(alone.view(np.uint32), oc.view(np.uint32))
        assert nfl.sum() > 50
    # counters and flags are optional
    d_c = torch.from_numpy(raw.copy()).cuda()
    plan.fi_detect_correct(d_c, len(faults), wl.CORRECT_ZERO)
    torch.cuda.synchronize()
    plan.destroy()


@pytest.mark.parametrize("cfg", [0, 5])
def test_exponent_bound_detector_campaign_and_standalone(cfg):
    import torch
    M, N, K, kb, fmt = 200, 136, 128, 64, orc.BF16
    Aw, Bw = wl.gaussian(M, N, K, fmt, seed=21)
    p = orc.problem(M, N, K, kb, fmt, bound_mode=orc.BOUND_EXPONENT)
    plan = gu.make_plan(Aw, Bw, kb, fmt, cfg=cfg, bound_mode=fi.BOUND_EXPONENT)
    faults = fi.fi_sample_faults(5, 0, 512, plan.desc, fi.KIND_MIX_ACC_A, 1)
    faults["xor_mask"][::2] = 1 << np.random.default_rng(0).integers(23, 31, size=256).astype(np.uint32)
    recs, raw = gu.gpu_campaign(plan, faults, wl.CORRECT_NONE, want_c=True)
    s = gu.compare_records(recs, orc.campaign(p, Aw, Bw, gu.to_orc_faults(faults), wl.CORRECT_NONE), faults,
                           operands=(orc.decode_array(Aw, fmt), orc.decode_array(Bw, fmt)))
    assert not s["mismatches"], s["mismatches"][:5]
    assert (recs["n_flagged"] > 0).sum() > 20
    # the flag is a function of the output word alone: exponent 1eeexxxx with a 1 among eee
    e = (raw.view(np.uint32) >> 23) & 0xFF
    want = ((e & 0x80) != 0) & ((e & 0x70) != 0)
    assert np.array_equal(recs["n_flagged"], want.reshape(len(faults), -1).sum(axis=1).astype(np.uint32))
    d_c = torch.from_numpy(raw.copy()).cuda()
    d_fl = torch.empty(raw.shape, dtype=torch.uint8, device="cuda")
    d_n = torch.empty(len(faults), dtype=torch.int32, device="cuda")
    plan.fi_detect_correct(d_c, len(faults), wl.CORRECT_ZERO, d_fl, d_n)
    torch.cuda.synchronize()
    assert np.array_equal(d_fl.cpu().numpy().astype(bool), want)
    assert np.array_equal(d_c.cpu().numpy().view(np.uint32), np.where(want, 0, raw.view(np.uint32)))
    plan.destroy()


def test_campaign_calls_replay_correctly_from_a_hip_graph():
    # The library clears records and counters with kernels, not memsets, so its calls can be
    # captured.  Replays are interleaved with eager work and synchronisations and every replay is
    # checked against the eager result.
    import torch
    w = wl.tiny()
    plan = gu.make_plan(w.A, w.B, w.kb, w.fmt)
    n = 256
    faults = fi.fi_sample_faults(5, 0, n, plan.desc, fi.KIND_ALL_ACC, 1)
    d_f = fi.to_device(faults)
    d_r = fi.empty_results(n)
    d_cls = torch.empty(n, dtype=torch.uint8, device="cuda")
    d_cnt = torch.empty(3, dtype=torch.int64, device="cuda")
    plan.fi_gemm_inject_batch(d_f, n, fi.CORRECT_ZERO, d_r)
    plan.fi_classify(d_r, n, d_cls, d_cnt)
    torch.cuda.synchronize()
    want_r = fi.results_to_host(d_r).copy()
    want_cnt = d_cnt.cpu().numpy().copy()
    side = torch.cuda.Stream()
    plan.reserve(n, side)               # each stream has its own batch scratch: size it outside the capture
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            s = torch.cuda.current_stream().cuda_stream
            plan.fi_gemm_inject_batch(d_f, n, fi.CORRECT_ZERO, d_r, stream=s)
            plan.fi_classify(d_r, n, d_cls, d_cnt, stream=s)
    for rep in range(4):
        d_r.zero_(); d_cnt.fill_(-1)                                   # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = fi.results_to_host(d_r)
        assert got.tobytes() == want_r.tobytes(), rep
        assert np.array_equal(d_cnt.cpu().numpy(), want_cnt), rep
        # a different fault list through the same graph (the list lives in device memory)
        if rep == 1:
            faults2 = fi.fi_sample_faults(6, 0, n, plan.desc, fi.KIND_ALL_ACC, 1)
            d_f.copy_(fi.to_device(faults2))
            plan.fi_gemm_inject_batch(d_f, n, fi.CORRECT_ZERO, d_r)
            plan.fi_classify(d_r, n, d_cls, d_cnt)
            torch.cuda.synchronize()
            want_r = fi.results_to_host(d_r).copy()
            want_cnt = d_cnt.cpu().numpy().copy()
    plan.destroy()


@pytest.mark.parametrize("shape", [(1, 1, 64, 64), (1, 70, 128, 32), (33, 1, 64, 16), (5, 3, 16, 16), (129, 65, 4096, 64)])
def test_degenerate_and_extreme_shapes(shape):
    # One row, one column, a single 16-wide k-step, a long K; batches of 1, 7 and 9 trials (less
    # than, and one more than, a group of 8), every fault kind; exact regime, bit for bit.
    M, N, K, kb = shape
    fmt = orc.BF16
    Aw, Bw = wl.small_integers(M, N, K, fmt, seed=K + M, lim=2, step=2)
    p = orc.problem(M, N, K, kb, fmt)
    rng = np.random.default_rng(M * 7 + N)
    rows = []
    for t in range(9):
        kind = [orc.SITE_ACC, orc.SITE_PRODUCT, orc.SITE_A, orc.SITE_B, orc.SITE_NONE][t % 5]
        i, j, k = int(rng.integers(M)), int(rng.integers(N)), int(rng.integers(K))
        if kind == orc.SITE_ACC:
            rows.append((kind, i, j, int(rng.integers(K // kb)), 1 << int(rng.integers(20, 32))))
        elif kind == orc.SITE_PRODUCT:
            rows.append((kind, i, j, k, 0x8000))
        elif kind == orc.SITE_A:
            rows.append((kind, i, k, 0, 0x8000))
        elif kind == orc.SITE_B:
            rows.append((kind, k, j, 0, 0x8000))
        else:
            rows.append((kind, 0, 0, 0, 0))
    faults = orc.make_faults(rows)
    plan = gu.make_plan(Aw, Bw, kb, fmt)
    gold = orc.gemm(p, Aw, Bw)
    assert np.array_equal(plan.buffer_to_host(fi.BUF_C_STAR).view(np.uint32), gold.view(np.uint32))
    for n in (1, 7, 9):
        recs, cout = gu.gpu_campaign(plan, faults[:n], orc.CORRECT_RECOMPUTE, want_c=True)
        ora = orc.campaign(p, Aw, Bw, faults[:n], orc.CORRECT_RECOMPUTE, orc.MODE_AFFECTED)
        for t in range(n):
            o, cf, cc = orc.trial(p, Aw, Bw, faults[t:t + 1], orc.CORRECT_RECOMPUTE, orc.MODE_FULL, want_outputs=True)
            nan = np.isnan(cc)
            assert np.array_equal(np.isnan(cout[t]), nan)
            assert np.array_equal(cout[t][~nan].view(np.uint32), cc[~nan].view(np.uint32)), (t, faults[t])
        s = gu.compare_records(recs, ora, faults[:n], exact_words=True)
        assert not s["mismatches"], s["mismatches"][:5]
    plan.destroy()


@pytest.mark.parametrize("name", ["tiny128", "bert_linear", "resnet_conv", "detector_stress"])
def test_affected_tiles_only_campaign_gives_the_same_records(name):
    # Computing only what a fault can reach must reproduce the full campaign's records exactly
    # (same kernels, same accumulation order); it is timed as trials per second only.
    import time
    import torch
    w = wl.ALL[name]()
    n = min(w.n_trials, 4096)
    for cfg in ((None,) if name != "tiny128" else (None, 0, 1, 2)):
        plan = gu.make_plan(w.A, w.B, w.kb, w.fmt)
        faults = fi.fi_sample_faults(w.fault_seed, 0, n, plan.desc, w.kind_mode if name != "resnet_conv" else fi.KIND_ALL_B,
                                     w.nbits)
        faults[3]["row"] = 10 ** 7                                  # an invalid site
        d_f = fi.to_device(faults)
        full = gu.gpu_campaign(plan, faults, w.policies[0])
        if cfg is not None:
            plan.tune(cfg)
        d_r = fi.empty_results(n)
        plan.fi_gemm_inject_batch_affected(d_f, n, w.policies[0], d_r)
        part = fi.results_to_host(d_r)
        assert part.tobytes() == full.tobytes(), [t for t in range(n) if part[t] != full[t]][:5]
        torch.cuda.synchronize(); t0 = time.perf_counter()
        for _ in range(3):
            plan.fi_gemm_inject_batch_affected(d_f, n, w.policies[0], d_r)
        torch.cuda.synchronize()
        print(name, "affected-only: %.0f trials/s" % (3 * n / (time.perf_counter() - t0)))
        plan.destroy()
