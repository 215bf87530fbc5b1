"""Pins for site selection (Sec. IV-A: uniform target, random bit(s), one fault per trial)."""
import os

import numpy as np

from oracle import pyoracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_splitmix64_published_vectors():
    with open(os.path.join(GOLDEN, "splitmix64_vectors.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    for row in rows:
        seed, want = int(row[0]), [int(x) for x in row[1:]]
        assert orc.splitmix64_stream(seed, len(want)) == want


def test_draw_order_and_ranges():
    p = orc.problem(10, 7, 96, 32, orc.FP16)
    seed, t = 12345, 5
    u = orc.splitmix64_stream((seed + (t << 32)) % 2 ** 64, 4)
    unif = lambda n, x: ((x >> 32) * n) >> 32
    f = orc.sample_faults(seed, t, 1, p, orc.KIND_ALL_ACC, 1)[0]
    assert (f["kind"], f["row"], f["col"], f["kblock"]) == (orc.SITE_ACC, unif(10, u[0]), unif(7, u[1]), unif(3, u[2]))
    assert f["xor_mask"] == 1 << unif(32, u[3])
    f = orc.sample_faults(seed, t, 1, p, orc.KIND_ALL_A, 2)[0]
    s, kk = unif(3, u[1]), unif(32, u[2])
    assert (f["kind"], f["row"], f["col"], f["kblock"]) == (orc.SITE_A, unif(10, u[0]), s * 32 + kk, s)
    assert f["xor_mask"] == 3 << unif(15, u[3])
    f = orc.sample_faults(seed, t, 1, p, orc.KIND_ALL_B, 4)[0]
    assert (f["kind"], f["row"], f["col"]) == (orc.SITE_B, s * 32 + kk, unif(7, u[0]))
    assert f["xor_mask"] == 15 << unif(13, u[3])
    # counter-keyed: any slice of a campaign can be regenerated alone
    whole = orc.sample_faults(9, 0, 100, p, orc.KIND_MIX_ACC_A, 1)
    part = orc.sample_faults(9, 40, 20, p, orc.KIND_MIX_ACC_A, 1)
    assert whole[40:60].tobytes() == part.tobytes()
    assert np.all(whole["kind"][0::2] == orc.SITE_ACC) and np.all(whole["kind"][1::2] == orc.SITE_A)


def _chi2(counts):
    e = counts.sum() / len(counts)
    return float(((counts - e) ** 2 / e).sum())


def test_uniformity_and_mask_shape():
    p = orc.problem(16, 8, 128, 32, orc.BF16)
    n = 64000
    f = orc.sample_faults(3, 0, n, p, orc.KIND_ALL_ACC, 2)
    assert f["row"].max() == 15 and f["col"].max() == 7 and f["kblock"].max() == 3
    pos = np.log2((f["xor_mask"] & -f["xor_mask"].astype(np.int64)).astype(np.float64)).astype(int)
    assert np.all(f["xor_mask"] == (3 << pos).astype(np.uint32)) and pos.min() == 0 and pos.max() == 30
    # chi-square against uniform; 99.9% quantiles for 15, 7, 3 and 30 degrees of freedom
    assert _chi2(np.bincount(f["row"], minlength=16)) < 37.7
    assert _chi2(np.bincount(f["col"], minlength=8)) < 24.3
    assert _chi2(np.bincount(f["kblock"], minlength=4)) < 16.3
    assert _chi2(np.bincount(pos, minlength=31)) < 59.7
    # rows and columns are not the same draw
    assert np.corrcoef(f["row"], f["col"])[0, 1] ** 2 < 1e-3
    fa = orc.sample_faults(3, 0, n, p, orc.KIND_ALL_A, 1)
    assert fa["col"].max() == 127 and np.all(fa["kblock"] == fa["col"] // 32)
    assert np.all(fa["xor_mask"] < 65536) and _chi2(np.bincount(fa["col"], minlength=128)) < 181.0
