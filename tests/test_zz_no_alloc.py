"""The entry point that allocates nothing (fi_gemm_inject_batch_noalloc) against
fi_gemm_inject_batch: same records and outputs, bit for bit, on two calls in a row, the second
with a smaller batch (the static scratch keeps the first call's contents)."""
import numpy as np
import pytest

from oracle import pyoracle as orc
from paper_2311_05782_amd import fi, workloads as wl
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _mixed(plan, n, seed):
    f = fi.fi_sample_faults(seed, 0, n, plan.desc, fi.KIND_MIX_ACC_A, 1)
    g = fi.fi_sample_faults(seed + 1, 0, n, plan.desc, fi.KIND_ALL_B, 2)
    h = fi.fi_sample_faults(seed + 2, 0, n, plan.desc, fi.KIND_ALL_PRODUCT, 4)
    f[2::5] = g[2::5]
    f[3::5] = h[3::5]
    f[4::25]["kind"] = 0
    f[7]["row"] = 10 ** 7                       # an invalid site
    return f


@pytest.mark.parametrize("cfg", [None, 3, 0])
def test_noalloc_entry_point_equals_the_allocating_one_on_two_calls_in_a_row(cfg):
    import torch
    M, N, K, kb, fmt = 300, 200, 192, 32, orc.FP16
    Aw, Bw = wl.gaussian(M, N, K, fmt, seed=31)
    plan = gu.make_plan(Aw, Bw, kb, fmt, cfg=cfg)
    for n, seed, policy, want_c in ((777, 5, wl.CORRECT_RECOMPUTE, False), (61, 9, wl.CORRECT_ZERO, True)):
        faults = _mixed(plan, n, seed)
        d_f = fi.to_device(faults)
        ref = gu.gpu_campaign(plan, faults, policy, want_c=want_c)
        d_r = fi.empty_results(n)
        d_r.fill_(0xAB)
        d_c = torch.full((n, M, N), 7.0, dtype=torch.float32, device="cuda") if want_c else None
        plan.fi_gemm_inject_batch_noalloc(d_f, n, policy, d_r, d_c)
        got = fi.results_to_host(d_r)
        if want_c:
            ref, ref_c = ref
            assert np.array_equal(d_c.cpu().numpy().view(np.uint32), ref_c.view(np.uint32))
        assert got.tobytes() == ref.tobytes(), [t for t in range(n) if got[t] != ref[t]][:5]
        # and against the oracle, by the guard-banded rule
        p = orc.problem(M, N, K, kb, fmt)
        ora = orc.campaign(p, Aw, Bw, gu.to_orc_faults(faults), policy, orc.MODE_AFFECTED)
        ra, cb, _ = orc.rowcol_absmax(p, Aw, Bw)
        s = gu.compare_records(got, ora, faults, site_tol=2.0 ** -12 * K * float(ra.max()) * float(cb.max()))
        assert not s["mismatches"], s["mismatches"][:5]
    plan.destroy()


def test_noalloc_entry_point_rejects_batches_beyond_its_scratch():
    Aw, Bw = wl.gaussian(64, 64, 64, orc.BF16, seed=1)
    plan = gu.make_plan(Aw, Bw, 32, orc.BF16)
    n = 16385
    d_f = fi.to_device(np.zeros(n, fi.FAULT_DTYPE))
    d_r = fi.empty_results(n)
    with pytest.raises(fi.FiError) as e:
        plan.fi_gemm_inject_batch_noalloc(d_f, n, wl.CORRECT_ZERO, d_r)
    assert e.value.status == fi.UNSUPPORTED and "16384" in str(e.value)
    plan.fi_gemm_inject_batch_noalloc(d_f, 16384, wl.CORRECT_ZERO, d_r)      # the largest batch it takes
    recs = fi.results_to_host(d_r)[:16384]
    assert not recs["n_flagged"].any() and not recs["n_bitdiff"].any() and not recs["status"].any()
    plan.destroy()
