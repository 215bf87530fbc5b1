"""Pins for the hand-over between two layers (ReLU, rounding to the operand format) and for the
next layer's GEMM on per-trial operands (Sec. I: the gap between the resilience of one matrix
multiplication and of what is computed from it; Sec. V-B (i): zeros are common in activations)."""
import numpy as np
import pytest

from oracle import pyoracle as orc
from paper_2311_05782_amd import workloads as wl
import np_reference as ref

FIELDS = ["n_flagged", "n_bitdiff", "n_dev_pre", "n_dev_post", "cls"]


# ---- activation + rounding ------------------------------------------------------------------

def test_activation_special_values():
    c = np.array([-0.0, -1.0, 0.0, 1.0, np.inf, -np.inf, 65519.9, 65520.0, 1e-9, 2.0 ** -24, 2.0 ** -25,
                  3.0e38, 3.4e38], np.float32)
    h16 = orc.activation_round(c, orc.FP16).tolist()
    assert h16 == [0, 0, 0, 0x3C00, 0x7C00, 0, 0x7BFF, 0x7C00, 0, 0x0001, 0, 0x7C00, 0x7C00]
    hb = orc.activation_round(c, orc.BF16).tolist()
    # 3.4e38 lies above the midpoint between the largest BF16 and 2^128: rounds to Inf
    assert hb[:6] == [0, 0, 0, 0x3F80, 0x7F80, 0] and hb[11] == 0x7F62 and hb[12] == 0x7F80
    for fmt, qnan in ((orc.FP16, 0x7E00), (orc.BF16, 0x7FC0)):
        n = orc.activation_round(np.array([np.nan, -np.nan], np.float32), fmt)
        assert [int(x) & 0x7FFF for x in n] == [qnan, qnan]      # a NaN is handed on as a NaN


def test_activation_equals_numpy_conversion_after_a_numpy_relu():
    rng = np.random.default_rng(3)
    c = np.concatenate([rng.normal(0, 1, 20000), rng.normal(0, 300, 20000), rng.normal(0, 1e-6, 20000),
                        rng.uniform(-70000, 70000, 20000)]).astype(np.float32)
    relu = np.where(c > 0, c, np.float32(0))
    with np.errstate(over="ignore"):
        want16 = relu.astype(np.float16).view(np.uint16)
    assert np.array_equal(orc.activation_round(c, orc.FP16), want16)
    bits = relu.view(np.uint32).astype(np.uint64)
    wantb = ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16).astype(np.uint16)
    assert np.array_equal(orc.activation_round(c, orc.BF16), wantb)
    assert (want16 == 0).mean() > 0.4                           # about half the activations are zero


# ---- next layer on per-trial operands --------------------------------------------------------

def _problem(M=6, N=5, K=64, kb=32, fmt=orc.FP16, seed=4):
    Aw, Bw = wl.gaussian(M, N, K, fmt, seed=seed)
    return orc.problem(M, N, K, kb, fmt), Aw, Bw


def test_identical_operands_reproduce_the_fault_free_result():
    p, Aw, Bw = _problem()
    stack = np.stack([Aw, Aw])
    for mode in (orc.MODE_FULL, orc.MODE_AFFECTED):
        recs, cc = orc.propagate(p, Aw, Bw, stack, orc.CORRECT_ZERO, mode=mode, want_outputs=True)
        cstar = orc.gemm(p, Aw, Bw)
        assert np.array_equal(cc.view(np.uint32), np.stack([cstar, cstar]).view(np.uint32))
        for k in FIELDS:
            assert recs[k].tolist() == [0, 0]
        assert recs["max_dev_pre"].tolist() == [0.0, 0.0]


@pytest.mark.parametrize("fmt", [orc.FP16, orc.BF16])
def test_one_changed_word_is_the_operand_fault_of_a_single_layer_trial(fmt):
    # replacing A by "A with one word XORed" must give the records of the A-operand fault trial,
    # which is pinned on its own against the NumPy reference
    p, Aw, Bw = _problem(fmt=fmt, seed=8)
    rng = np.random.default_rng(1)
    for policy in (orc.CORRECT_ZERO, orc.CORRECT_RECOMPUTE, orc.CORRECT_NONE):
        faults, stack = [], []
        for t in range(24):
            i, k, bit = int(rng.integers(p.M)), int(rng.integers(p.K)), int(rng.integers(16))
            At = Aw.copy(); At[i, k] ^= np.uint16(1 << bit)
            faults.append((orc.SITE_A, i, k, 0, 1 << bit)); stack.append(At)
        recs = orc.propagate(p, Aw, Bw, np.stack(stack), policy)
        for t, f in enumerate(faults):
            want = orc.trial(p, Aw, Bw, f, policy)
            for k in FIELDS + ["max_dev_pre", "max_dev_post", "n_border_T", "n_border_tau"]:
                a, b = recs[t][k], want[k]
                assert a == b or (np.isnan(a) and np.isnan(b)), (t, f, k, a, b)
        assert (recs["n_bitdiff"] > 0).sum() > 12


def test_outputs_against_numpy_scalar_accumulation_and_counters_by_hand():
    M, N, K, kb, fmt = 4, 3, 32, 16, orc.FP16
    p, Aw, Bw = _problem(M, N, K, kb, fmt, seed=9)
    rng = np.random.default_rng(2)
    stack = np.stack([wl.to_words(rng.normal(0, s, (M, K)).astype(np.float32), fmt) for s in (1.0, 30.0, 3000.0)])
    stack[0, 1:] = Aw[1:]                                        # trial 0: only row 0 differs
    recs, cc = orc.propagate(p, Aw, Bw, stack, orc.CORRECT_NONE, want_outputs=True)
    A, B = ref.decode(Aw, fmt), ref.decode(Bw, fmt)
    ra, cb = np.abs(A).max(axis=1), np.abs(B).max(axis=1)
    T = ((np.float32(K) * ra).astype(np.float32)[:, None] * cb[None, :]).astype(np.float32)
    T = (T * np.float32(1 + 2.0 ** -11)).astype(np.float32)
    S = np.abs(A.astype(np.float64)) @ np.abs(B.astype(np.float64)).T
    cstar = np.array([[ref.dot(A[i], B[j], kb)[0] for j in range(N)] for i in range(M)], np.float32)
    for t in range(3):
        At = ref.decode(stack[t], fmt)
        y = np.array([[ref.dot(At[i], B[j], kb)[0] for j in range(N)] for i in range(M)], np.float32)
        assert np.array_equal(cc[t].view(np.uint32), y.view(np.uint32))
        dev = np.abs(y.astype(np.float64) - cstar.astype(np.float64))
        assert int(recs[t]["n_flagged"]) == int((~(np.abs(y) <= T)).sum())
        assert int(recs[t]["n_bitdiff"]) == int((y.view(np.uint32) != cstar.view(np.uint32)).sum())
        assert int(recs[t]["n_dev_pre"]) == int((~(dev <= S * 2.0 ** -12)).sum())
        assert float(recs[t]["max_dev_pre"]) == float(dev.max())
    assert int(recs[0]["n_bitdiff"]) <= N and int(recs[2]["n_flagged"]) > 0


def test_full_and_affected_modes_agree_and_policies_correct_only_flagged_elements():
    p, Aw, Bw = _problem(M=12, N=9, K=64, kb=32, fmt=orc.BF16, seed=10)
    rng = np.random.default_rng(5)
    stack = np.stack([Aw.copy() for _ in range(16)])
    for t in range(16):
        rows = rng.choice(p.M, size=int(rng.integers(0, 4)), replace=False)
        for i in rows:
            stack[t, i, rng.integers(p.K)] ^= np.uint16(1 << int(rng.integers(7, 15)))   # exponent bits
    cstar = orc.gemm(p, Aw, Bw)
    raw = orc.propagate(p, Aw, Bw, stack, orc.CORRECT_NONE, want_outputs=True)[1]
    for policy in (orc.CORRECT_ZERO, orc.CORRECT_RECOMPUTE):
        full, cf = orc.propagate(p, Aw, Bw, stack, policy, mode=orc.MODE_FULL, want_outputs=True)
        aff, ca = orc.propagate(p, Aw, Bw, stack, policy, mode=orc.MODE_AFFECTED, want_outputs=True)
        assert full.tobytes() == aff.tobytes() and cf.tobytes() == ca.tobytes()
        ra, cb, _ = orc.rowcol_absmax(p, Aw, Bw)
        _, flags, n = orc.detect_correct(p, ra, cb, raw, policy, c_star=cstar)
        assert np.array_equal(n, full["n_flagged"]) and n.sum() > 0
        fl = flags.astype(bool)
        want = np.where(fl, np.float32(0) if policy == orc.CORRECT_ZERO else np.broadcast_to(cstar, raw.shape), raw)
        assert np.array_equal(cf.view(np.uint32), want.view(np.uint32))
        if policy == orc.CORRECT_RECOMPUTE:
            assert np.all(full["n_dev_post"] <= full["n_dev_pre"])


# ---- two layers, worked by hand ----------------------------------------------------------------

def _two_layer(fmt, a_value, fault, policy=orc.CORRECT_NONE, K=128, kb=32, N1=4, P=2):
    """X = one row of a_value, W1 = N1 columns of ones, W2 = P x N1 ones."""
    X = wl.to_words(np.full((1, K), a_value, np.float32), fmt)
    W1 = wl.to_words(np.ones((N1, K), np.float32), fmt)
    W2 = wl.to_words(np.ones((P, 16), np.float32), fmt)          # layer-2 K padded to one 16-wide k-block
    p1 = orc.problem(1, N1, K, kb, fmt)
    rec1, cf, cc = orc.trial(p1, X, W1, fault, policy, want_outputs=True)
    hstar = np.zeros((1, 16), np.uint16); hstar[:, :N1] = orc.activation_round(orc.gemm(p1, X, W1), fmt)
    h = np.zeros((1, 16), np.uint16); h[:, :N1] = orc.activation_round(cc, fmt)
    p2 = orc.problem(1, P, 16, 16, fmt)
    rec2, y = orc.propagate(p2, hstar, W2, h[None], orc.CORRECT_NONE, want_outputs=True)
    return rec1, rec2[0], y[0], orc.gemm(p2, hstar, W2)


@pytest.mark.parametrize("fmt", [orc.FP16, orc.BF16])
def test_two_layers_worked_examples(fmt):
    # c1 = 128 in each of 4 columns, h = 128, y* = 512.  After block 0 the accumulator is 32.
    r1, r2, y, ystar = _two_layer(fmt, 1.0, (orc.SITE_ACC, 0, 1, 0, 1 << 23))      # 32 -> 64: c = 160
    assert ystar.tolist() == [[512.0, 512.0]] and y.tolist() == [[544.0, 544.0]]
    # 160 exceeds layer 1's bound 128 * (1 + 2^-11): detected there, handed on uncorrected here
    assert (int(r1["cls"]), int(r2["cls"]), int(r2["n_dev_pre"])) == (orc.DETECTED, orc.SDC, 2)
    r1, r2, y, _ = _two_layer(fmt, 1.0, (orc.SITE_ACC, 0, 1, 0, 1 << 23), policy=orc.CORRECT_RECOMPUTE)
    assert int(r2["cls"]) == orc.MASKED and y.tolist() == [[512.0, 512.0]]         # corrected before the hand-over
    r1, r2, y, _ = _two_layer(fmt, 1.0, (orc.SITE_ACC, 0, 1, 3, 1 << 31))          # 128 -> -128: ReLU -> 0
    assert y.tolist() == [[384.0, 384.0]] and float(r2["max_dev_pre"]) == 128.0
    r1, r2, y, _ = _two_layer(fmt, 1.0, (orc.SITE_ACC, 0, 1, 0, 1 << 30), policy=orc.CORRECT_ZERO)
    assert int(r1["cls"]) == orc.SDC and y.tolist() == [[480.0, 480.0]]           # 32 -> 2^-123: c = 96
    # a low mantissa flip that layer 1 still sees (c = 128 + 2^-16 after a last-block flip of bit 0)
    # disappears when the activation is rounded to the operand format
    r1, r2, y, ystar = _two_layer(fmt, 1.0, (orc.SITE_ACC, 0, 1, 3, 1))
    assert int(r1["n_bitdiff"]) == 1 and int(r2["n_bitdiff"]) == 0 and np.array_equal(y, ystar)


@pytest.mark.parametrize("fmt", [orc.FP16, orc.BF16])
def test_relu_masks_every_fault_that_leaves_a_negative_pre_activation_negative(fmt):
    # c1 = -128: h* = 0.  Whatever happens to the magnitude, a result that stays <= 0 is handed on
    # as 0 and the next layer's output is bit-identical; only the sign flip gets through.
    for bit in range(31):
        r1, r2, y, ystar = _two_layer(fmt, -1.0, (orc.SITE_ACC, 0, 2, 1, 1 << bit))
        assert int(r2["n_bitdiff"]) == 0 and int(r2["cls"]) == orc.MASKED, bit
        assert np.array_equal(y.view(np.uint32), ystar.view(np.uint32))
    assert sum(int(_two_layer(fmt, -1.0, (orc.SITE_ACC, 0, 2, 1, 1 << b))[0]["cls"]) != orc.MASKED
               for b in range(31)) >= 8                          # layer 1 alone calls many of them SDC
    r1, r2, y, _ = _two_layer(fmt, -1.0, (orc.SITE_ACC, 0, 2, 3, 1 << 31))         # -128 -> +128
    assert y.tolist() == [[128.0, 128.0]] and int(r2["n_dev_pre"]) == 2
