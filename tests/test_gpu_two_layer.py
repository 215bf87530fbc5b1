"""GPU parity for the two-layer workload: the hand-over kernel (ReLU + rounding to the operand
format) and the next layer's GEMM on per-trial operands, through the C ABI, against the oracle."""
import numpy as np
import pytest

from oracle import pyoracle as orc
from paper_2311_05782_amd import fi, workloads as wl
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _activation_gpu(c, fmt):
    import torch
    d_c = torch.from_numpy(np.ascontiguousarray(c, np.float32)).cuda()
    d_h = torch.empty(d_c.numel(), dtype=torch.int16, device="cuda")
    fi.fi_activation_round(fmt, d_c, d_c.numel(), d_h)
    torch.cuda.synchronize()
    return d_h.cpu().numpy().view(np.uint16).reshape(c.shape)


@pytest.mark.parametrize("fmt", [orc.FP16, orc.BF16])
def test_activation_round_bit_equal_including_specials_and_a_ragged_tail(fmt):
    rng = np.random.default_rng(7)
    special = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, -np.nan, 65504.0, 65519.9, 65520.0, 2.0 ** -24,
                        2.0 ** -25, 1.5 * 2.0 ** -25, 2.0 ** -14, 3.3e38, 3.4e38, 1e-40, -1e-40], np.float32)
    c = np.concatenate([special, rng.normal(0, 1, 300001), rng.normal(0, 1e4, 100000), rng.normal(0, 1e-6, 100000),
                        rng.uniform(0, 2.0 ** -13, 50000)]).astype(np.float32)
    assert c.size % 4 != 0
    # every bit pattern of the upper half too: all exponents, both signs
    hi = (np.arange(65536, dtype=np.uint32) << 16 | 0x8000).view(np.float32)
    # the rounding boundaries of both formats on every exponent and leading mantissa: just below a
    # tie, the tie (odd and even neighbours), just above - BF16 drops 16 bits, FP16 drops 13 and
    # moves to a fixed grid below 2^-14
    up16 = np.arange(65536, dtype=np.uint32) << 16
    up19 = np.arange(1 << 19, dtype=np.uint32) << 13
    edges = np.concatenate([up16 | lo for lo in (0x7FFF, 0x8001, 0x0001, 0xFFFF)] +
                           [up19 | lo for lo in (0x0FFF, 0x1000, 0x1001, 0x1FFF)]).view(np.float32)
    # FP16's subnormal grid: every binary32 value from below 2^-25 up to 2^-14, every 97th word
    sub = np.arange(0x32000000, 0x38900000, 97, dtype=np.uint32).view(np.float32)
    for x in (c, hi, c[:3], edges, sub):
        got, want = _activation_gpu(x, fmt), orc.activation_round(x, fmt)
        nan = np.isnan(x)
        assert np.array_equal(got[~nan], want[~nan])
        assert np.array_equal(got[nan] & 0x7FFF, want[nan] & 0x7FFF)


def _stack_gpu(plan, stack, policy, want_c=False):
    import torch
    n = stack.shape[0]
    d = plan.desc
    d_s = fi.words_to_device(stack)
    d_r = fi.empty_results(n)
    d_c = torch.empty((n, d.M, d.N), dtype=torch.float32, device="cuda") if want_c else None
    plan.fi_gemm_propagate_batch(d_s, stack.shape[1] * stack.shape[2], n, policy, d_r, d_c)
    recs = fi.results_to_host(d_r)
    return (recs, d_c.cpu().numpy()) if want_c else recs


@pytest.mark.parametrize("fmt", [orc.FP16, orc.BF16])
@pytest.mark.parametrize("cfg", [0, 1, 2])
@pytest.mark.parametrize("shape", [(300, 200, 192, 32), (130, 65, 96, 48), (64, 64, 64, 16)])
def test_next_layer_exact_regime_bit_equal(fmt, cfg, shape):
    # small-integer operands in every trial: sums are exact, so outputs and every counter agree
    M, N, K, kb = shape
    Aw, Bw = wl.small_integers(M, N, K, fmt, seed=M + K, lim=4, step=2)
    rng = np.random.default_rng(cfg + N)
    n = 7
    stack = np.stack([Aw.copy() for _ in range(n)])
    for t in range(1, n):                                        # trial 0 keeps the golden operand
        rows = rng.choice(M, size=int(rng.integers(1, 6)), replace=False)
        other = wl.small_integers(M, N, K, fmt, seed=100 + t, lim=4, step=2)[0]
        stack[t, rows] = other[rows]
    stack[n - 1] = wl.small_integers(M, N, K, fmt, seed=999, lim=4, step=2)[0]   # every row differs
    plan = gu.make_plan(Aw, Bw, kb, fmt, cfg=cfg, group=3)
    p = orc.problem(M, N, K, kb, fmt)
    for policy in (orc.CORRECT_NONE, orc.CORRECT_ZERO, orc.CORRECT_RECOMPUTE):
        recs, cout = _stack_gpu(plan, stack, policy, want_c=True)
        orecs, occ = orc.propagate(p, Aw, Bw, stack, policy, want_outputs=True)
        assert np.array_equal(cout.view(np.uint32), occ.view(np.uint32))
        for k in ("n_flagged", "n_bitdiff", "n_dev_pre", "n_dev_post"):
            assert np.array_equal(recs[k], orecs[k]), (k, recs[k], orecs[k])
        assert np.array_equal(recs["max_dev_pre"], orecs["max_dev_pre"].astype(np.float32))
        assert np.array_equal(recs["max_dev_post"], orecs["max_dev_post"].astype(np.float32))
        assert recs["n_bitdiff"][0] == 0 and recs["n_bitdiff"][n - 1] > M * N // 2
        assert not recs["status"].any() and not recs["site_word_after"].any()
    plan.destroy()


@pytest.mark.parametrize("fmt,cfg", [(orc.FP16, 0), (orc.BF16, 1), (orc.BF16, 2)])
def test_next_layer_on_perturbed_gaussian_operands_guard_band_rule(fmt, cfg):
    M, N, K, kb = 260, 136, 256, 32
    Aw, Bw = wl.gaussian(M, N, K, fmt, seed=31)
    rng = np.random.default_rng(32)
    n = 48
    stack = np.stack([Aw.copy() for _ in range(n)])
    for t in range(n):
        for i in rng.choice(M, size=int(rng.integers(0, 4)), replace=False):
            bit = int(rng.integers(0, 15))                       # any mantissa or exponent bit
            stack[t, i, rng.integers(K)] ^= np.uint16(1 << bit)
    stack[5, 7, 3] = 0x7C00 if fmt == orc.FP16 else 0x7F80       # an Inf and a NaN handed on
    stack[6, 9, 200] = 0x7E00 if fmt == orc.FP16 else 0x7FC0
    plan = gu.make_plan(Aw, Bw, kb, fmt, cfg=cfg)
    p = orc.problem(M, N, K, kb, fmt)
    none = np.zeros(n, fi.FAULT_DTYPE)
    for policy in (orc.CORRECT_ZERO, orc.CORRECT_RECOMPUTE):
        recs = _stack_gpu(plan, stack, policy)
        orecs = orc.propagate(p, Aw, Bw, stack, policy, mode=orc.MODE_AFFECTED)
        s = gu.compare_records(recs, orecs, none, site_tol=1.0)
        assert not s["mismatches"], s["mismatches"][:5]
        assert s["gpu_counts"][1] > 0 and s["gpu_counts"][2] > 0 and n - s["borderline"] >= 12
        assert recs["n_flagged"][5] >= N and recs["n_flagged"][6] >= N     # a whole non-finite row each
    # stride 0: every trial reads the same operand
    import torch
    d_r = fi.empty_results(3)
    plan.fi_gemm_propagate_batch(fi.words_to_device(stack[5]), 0, 3, orc.CORRECT_ZERO, d_r)
    r = fi.results_to_host(d_r)
    assert r[0].tobytes() == r[1].tobytes() == r[2].tobytes() and r[0]["n_flagged"] >= N
    with pytest.raises(fi.FiError):
        plan.fi_gemm_propagate_batch(fi.words_to_device(stack), 8, 3, orc.CORRECT_ZERO, d_r)
    plan.destroy()


@pytest.mark.parametrize("fmt", [orc.FP16, orc.BF16])
def test_two_layers_end_to_end_against_the_oracle_chain(fmt):
    # layer 1: campaign with materialised corrected outputs -> ReLU + rounding -> layer 2 on the
    # stack.  Small-integer inputs make layer 1 exact, so both sides hand on the same words.
    import torch
    M, D, H, P, kb = 70, 64, 144, 40, 32
    lim = 2 if fmt == orc.FP16 else 1
    Xw, W1w = wl.small_integers(M, H, D, fmt, seed=41, lim=lim)
    W2w = wl.small_integers(P, P, H, fmt, seed=42, lim=lim)[0][:, :H]          # [P][H]
    p1 = orc.problem(M, H, D, kb, fmt)
    plan1 = gu.make_plan(Xw, W1w, kb, fmt)
    n = 96
    faults = fi.fi_sample_faults(9, 0, n, plan1.desc, fi.KIND_ALL_ACC, 1)
    faults["xor_mask"][::4] = 1 << 31                            # sign flips: ReLU decides
    recs1, c1 = gu.gpu_campaign(plan1, faults, orc.CORRECT_ZERO, want_c=True)
    h_gpu = _activation_gpu(c1, fmt)
    hstar_gpu = _activation_gpu(plan1.buffer_to_host(fi.BUF_C_STAR), fmt)
    # the fused form of the same two calls hands on the same words and the same records
    d_hf = torch.empty((n, M, H), dtype=torch.int16, device="cuda")
    d_rf = fi.empty_results(n)
    plan1.fi_gemm_inject_batch_act(fi.to_device(faults), n, orc.CORRECT_ZERO, d_rf, d_hf)
    torch.cuda.synchronize()
    assert np.array_equal(d_hf.cpu().numpy().view(np.uint16), h_gpu)
    assert fi.results_to_host(d_rf).tobytes() == recs1.tobytes()
    # the oracle's chain
    of = gu.to_orc_faults(faults)
    occ = np.stack([orc.trial(p1, Xw, W1w, of[t:t + 1], orc.CORRECT_ZERO, want_outputs=True)[2] for t in range(n)])
    h_orc = orc.activation_round(occ, fmt)
    hstar_orc = orc.activation_round(orc.gemm(p1, Xw, W1w), fmt)
    assert np.array_equal(h_gpu, h_orc) and np.array_equal(hstar_gpu, hstar_orc)
    assert (hstar_orc == 0).mean() > 0.3
    p2 = orc.problem(M, P, H, 48, fmt)
    plan2 = gu.make_plan(hstar_gpu, W2w, 48, fmt)
    recs2 = _stack_gpu(plan2, h_gpu, orc.CORRECT_NONE)
    orecs2 = orc.propagate(p2, hstar_orc, W2w, h_orc, orc.CORRECT_NONE, mode=orc.MODE_AFFECTED)
    s = gu.compare_records(recs2, orecs2, np.zeros(n, fi.FAULT_DTYPE), site_tol=1.0)
    assert not s["mismatches"], s["mismatches"][:5]
    # layer-to-output masking: trials that layer 1 does not call masked but whose final output is
    sdc1 = gu.cls_of(recs1) != 0
    masked2 = gu.cls_of(recs2) == 0
    assert np.array_equal(masked2, orecs2["cls"] == 0) or s["borderline"] > 0
    assert (sdc1 & masked2).sum() > 5 and (sdc1 & ~masked2).sum() > 5
    assert not (~sdc1 & ~masked2 & (recs1["n_bitdiff"] == 0)).any()
    plan1.destroy(); plan2.destroy()


@pytest.mark.parametrize("fmt", [orc.FP16, orc.BF16])
@pytest.mark.parametrize("cfg", [None, 0, 1, 3, 4, 5, 6])
@pytest.mark.parametrize("shape", [(300, 200, 192, 32), (257, 65, 128, 64), (64, 64, 64, 16), (96, 40, 96, 48)])
def test_fused_hand_over_equals_campaign_then_activation_round(fmt, cfg, shape):
    # fi_gemm_inject_batch_act against fi_gemm_inject_batch + fi_activation_round: same words (NaN
    # payloads included: both round the same corrected value with the same integer code), same
    # records; Gaussian operands, every fault kind, flips that make Inf / NaN / negative values.
    import torch
    M, N, K, kb = shape
    Aw, Bw = wl.gaussian(M, N, K, fmt, seed=M + N)
    plan = gu.make_plan(Aw, Bw, kb, fmt, cfg=cfg, group=3)
    n = 61
    rows = []
    rng = np.random.default_rng(K + (cfg or 0))
    for t in range(n):
        kind = [orc.SITE_ACC, orc.SITE_A, orc.SITE_B, orc.SITE_PRODUCT, orc.SITE_NONE][t % 5]
        i, j, k = int(rng.integers(M)), int(rng.integers(N)), int(rng.integers(K))
        if kind == orc.SITE_ACC:
            rows.append((kind, i, j, int(rng.integers(K // kb)), 1 << [30, 31, 23, 22, 29][t // 5 % 5]))
        elif kind == orc.SITE_A:
            rows.append((kind, i, k, 0, [0x4000, 0x8000, 0x0200][t // 5 % 3]))
        elif kind == orc.SITE_B:
            rows.append((kind, k, j, 0, [0x4000, 0x8000, 0x0200][t // 5 % 3]))
        elif kind == orc.SITE_PRODUCT:
            rows.append((kind, i, j, k, 0x4000))
        else:
            rows.append((kind, 0, 0, 0, 0))
    faults = orc.make_faults(rows)
    d_f = fi.to_device(faults)
    for policy in (orc.CORRECT_NONE, orc.CORRECT_ZERO, orc.CORRECT_RECOMPUTE):
        d_c = torch.empty((n, M, N), dtype=torch.float32, device="cuda")
        d_h2 = torch.empty((n, M, N), dtype=torch.int16, device="cuda")
        d_h1 = torch.full((n, M, N), 0x5555, dtype=torch.int16, device="cuda")
        r1, r2 = fi.empty_results(n), fi.empty_results(n)
        plan.fi_gemm_inject_batch(d_f, n, policy, r2, d_c)
        fi.fi_activation_round(fmt, d_c, n * M * N, d_h2)
        plan.fi_gemm_inject_batch_act(d_f, n, policy, r1, d_h1)
        torch.cuda.synchronize()
        assert torch.equal(d_h1, d_h2), (policy, int((d_h1 != d_h2).sum()))
        assert fi.results_to_host(r1).tobytes() == fi.results_to_host(r2).tobytes()
        c = d_c.cpu().numpy()
        if policy == orc.CORRECT_NONE:
            assert np.isnan(c).any() or np.isinf(c).any()        # the specials were really there
    plan.destroy()


def test_fused_hand_over_is_refused_where_the_one_trial_kernel_runs():
    Aw, Bw = wl.gaussian(64, 64, 96, orc.BF16, seed=5)
    plan = gu.make_plan(Aw, Bw, 32, orc.BF16, cfg=2)             # 256 x 64 tiles: the one-trial kernel
    import torch
    d_h = torch.empty((2, 64, 64), dtype=torch.int16, device="cuda")
    with pytest.raises(fi.FiError):
        plan.fi_gemm_inject_batch_act(fi.to_device(orc.make_faults([(orc.SITE_NONE, 0, 0, 0, 0)] * 2)), 2, 0,
                                      fi.empty_results(2), d_h)
    plan.destroy()


def test_the_chain_replays_correctly_from_a_hip_graph():
    # The three calls clear their records with kernels and, once the stream's batch scratch is
    # reserved, allocate nothing, so the whole chain can be captured; replays alternate with eager work and are compared with the eager result.
    import torch
    fmt, kb = orc.BF16, 32
    Xw, W1w, W2w = wl.two_layer_mlp(M=128, D=64, H=192, fmt=fmt, seed=3)
    M, D, H = 128, 64, 192
    plan1 = gu.make_plan(Xw, W1w, kb, fmt)
    d_hstar = torch.empty((M, H), dtype=torch.int16, device="cuda")
    fi.fi_activation_round(fmt, plan1.buffer_ptr(fi.BUF_C_STAR), M * H, d_hstar)
    torch.cuda.synchronize()
    plan2 = fi.Plan(fi.plan_desc(M, D, H, kb, fmt), d_hstar, fi.words_to_device(W2w))
    n = 40
    lists = [fi.fi_sample_faults(s, 0, n, plan1.desc, fi.KIND_MIX_ACC_A, 2) for s in (1, 2, 3)]
    d_f = fi.to_device(lists[0])
    d_c1 = torch.empty((n, M, H), dtype=torch.float32, device="cuda")
    d_h = torch.empty((n, M, H), dtype=torch.int16, device="cuda")
    r1, r2 = fi.empty_results(n), fi.empty_results(n)

    def chain(stream=None):
        plan1.fi_gemm_inject_batch(d_f, n, orc.CORRECT_ZERO, r1, d_c1, stream=stream)
        fi.fi_activation_round(fmt, d_c1, n * M * H, d_h, stream=stream)
        plan2.fi_gemm_propagate_batch(d_h, M * H, n, orc.CORRECT_NONE, r2, stream=stream)

    eager = []
    for f in lists:
        d_f.copy_(fi.to_device(f))
        chain()
        eager.append((fi.results_to_host(r1).tobytes(), fi.results_to_host(r2).tobytes()))
    assert eager[0] != eager[1]
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    d_f.copy_(fi.to_device(lists[0]))
    torch.cuda.synchronize()
    plan1.reserve(n, side)              # the capturing stream's batch scratch, sized outside the capture
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            chain(stream=torch.cuda.current_stream().cuda_stream)
    for rep in range(2):
        for k, f in enumerate(lists):
            d_f.copy_(fi.to_device(f))
            r1.zero_(); r2.fill_(0xFF)                              # eager work between replays
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert (fi.results_to_host(r1).tobytes(), fi.results_to_host(r2).tobytes()) == eager[k], (rep, k)
    # the two-call form (hand-over fused into the campaign) captured the same way
    def fused(stream=None):
        plan1.fi_gemm_inject_batch_act(d_f, n, orc.CORRECT_ZERO, r1, d_h, stream=stream)
        plan2.fi_gemm_propagate_batch(d_h, M * H, n, orc.CORRECT_NONE, r2, stream=stream)
    g2 = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g2, stream=side):
            fused(stream=torch.cuda.current_stream().cuda_stream)
    for k, f in enumerate(lists):
        d_f.copy_(fi.to_device(f))
        r1.zero_(); r2.fill_(0xFF); d_h.fill_(0x1234)
        torch.cuda.synchronize()
        g2.replay()
        torch.cuda.synchronize()
        assert (fi.results_to_host(r1).tobytes(), fi.results_to_host(r2).tobytes()) == eager[k], ("fused", k)
    plan1.destroy(); plan2.destroy()
