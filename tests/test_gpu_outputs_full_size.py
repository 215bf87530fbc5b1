"""Outputs of full-size campaigns, in the launch configuration the benchmark times (default
tiles and trial grouping): every element a fault cannot reach equals the fault-free result bit
for bit - so no tile of any trial was skipped, duplicated or mixed up - and every element it can
reach meets the oracle within the element's own tolerance."""
import numpy as np
import pytest

from oracle import pyoracle as orc
from paper_2311_05782_amd import fi, workloads as wl
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _oracle_reached(w, f):
    """The oracle's raw faulty values of what fault f can reach, from a full-mode trial of the
    sub-problem that holds them (an output element depends on its row of A and its column of B
    only): returns (rows, cols, values, tolerance per element)."""
    kind, r, c, kb, mask = int(f["kind"]), int(f["row"]), int(f["col"]), int(f["kblock"]), int(f["xor_mask"])
    Af = orc.decode_array(w.A, w.fmt).astype(np.float64)
    Bf = orc.decode_array(w.B, w.fmt).astype(np.float64)
    if kind in (orc.SITE_ACC, orc.SITE_PRODUCT):
        p = orc.problem(1, 1, w.K, w.kb, w.fmt)
        sub = orc.make_faults([(kind, 0, 0, kb, mask)])
        _, cf, _ = orc.trial(p, w.A[r:r + 1], w.B[c:c + 1], sub, orc.CORRECT_NONE, orc.MODE_FULL, want_outputs=True)
        tol = 2.0 ** -12 * (np.abs(Af[r]) @ np.abs(Bf[c]))
        return np.array([r]), np.array([c]), cf.reshape(-1), np.array([tol])
    if kind == orc.SITE_A:
        p = orc.problem(1, w.N, w.K, w.kb, w.fmt)
        sub = orc.make_faults([(kind, 0, c, 0, mask)])
        _, cf, _ = orc.trial(p, w.A[r:r + 1], w.B, sub, orc.CORRECT_NONE, orc.MODE_FULL, want_outputs=True)
        a = Af[r].copy()
        a[c] = float(orc.decode16(int(w.A[r, c]) ^ (mask & 0xFFFF), w.fmt))
        tol = 2.0 ** -12 * (np.abs(Bf) @ np.abs(a))
        return np.full(w.N, r), np.arange(w.N), cf.reshape(-1), tol
    raise AssertionError(kind)


@pytest.mark.parametrize("name", ["bert_linear", "resnet_conv", "detector_stress"])
def test_clean_elements_equal_the_fault_free_result_and_reached_ones_meet_the_oracle(name):
    import torch
    w = wl.ALL[name]()
    n = 64
    plan = gu.make_plan(w.A, w.B, w.kb, w.fmt)                 # default tiles, default trial grouping
    faults = fi.fi_sample_faults(w.fault_seed + 17, 0, n, plan.desc, w.kind_mode, w.nbits)
    faults[5]["kind"] = 0                                      # one fault-free trial
    d_f, d_r = fi.to_device(faults), fi.empty_results(n)
    d_c = torch.empty((n, w.M, w.N), dtype=torch.float32, device="cuda")
    d_c.fill_(float("nan"))
    plan.fi_gemm_inject_batch(d_f, n, fi.CORRECT_NONE, d_r, d_c)      # raw faulty outputs
    torch.cuda.synchronize()
    cstar = torch.from_numpy(plan.buffer_to_host(fi.BUF_C_STAR)).cuda()
    differs = d_c.view(torch.int32) != cstar.view(torch.int32).unsqueeze(0)          # [n][M][N]
    per_trial = differs.flatten(1).sum(dim=1).cpu().numpy()
    recs = fi.results_to_host(d_r)
    assert np.array_equal(per_trial, recs["n_bitdiff"])       # the records count what the outputs show
    n_checked = 0
    for t in range(n):
        f = faults[t]
        pos = torch.nonzero(differs[t]).cpu().numpy()          # [k][2] = (row, col) of every differing word
        if int(f["kind"]) == 0:
            assert len(pos) == 0
            continue
        rows, cols, want, tol = _oracle_reached(w, f)
        reach = set(zip(rows.tolist(), cols.tolist()))
        assert all((int(i), int(j)) in reach for i, j in pos), (t, f, pos[:5])
        got = d_c[t][torch.from_numpy(rows).cuda(), torch.from_numpy(cols).cuda()].cpu().numpy().astype(np.float64)
        want64 = want.astype(np.float64)
        both_bad = ~np.isfinite(got) & ~np.isfinite(want64)
        ok = both_bad | (np.abs(got - want64) <= tol)
        if int(f["kind"]) in (orc.SITE_ACC, orc.SITE_PRODUCT) and not ok.all():
            # a flipped exponent bit scales the (tolerated) difference of the two accumulators at
            # the site by what it scales the accumulator by
            ora = orc.campaign(orc.problem(w.M, w.N, w.K, w.kb, w.fmt), w.A, w.B, gu.to_orc_faults(faults[t:t + 1]),
                               orc.CORRECT_NONE, orc.MODE_AFFECTED)[0]
            before, after = abs(gu._f32(ora["site_word_before"])), abs(gu._f32(ora["site_word_after"]))
            scale = after / before if before > tol[0] else np.inf
            ok = np.abs(got - want64) <= tol * (2.0 + scale)
        assert ok.all(), (t, f, got[~ok][:4], want64[~ok][:4], tol[~ok][:4])
        n_checked += len(rows)
    assert n_checked >= n - 1
    plan.destroy()
