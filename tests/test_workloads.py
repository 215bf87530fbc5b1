"""The synthetic input recipe: shapes, distributions and structure of the five campaigns."""
import numpy as np

from oracle import pyoracle as orc
from paper_2311_05782_amd import workloads as wl


def test_tiny_and_determinism():
    w = wl.tiny()
    assert (w.M, w.N, w.K, w.kb, w.fmt, w.n_trials, w.nbits) == (128, 128, 128, 32, wl.FP16, 64, 1)
    assert w.A.shape == (128, 128) and w.A.dtype == np.uint16 and w.B.shape == (128, 128)
    w2 = wl.tiny()
    assert w.A.tobytes() == w2.A.tobytes() and w.B.tobytes() == w2.B.tobytes()
    a = orc.decode_array(w.A, orc.FP16)
    assert abs(a.mean()) < 0.05 and abs(a.std() - 1) < 0.05


def test_bert_and_resnet_statistics():
    w = wl.bert_linear()
    assert (w.M, w.K, w.N) == (512, 768, 3072) and w.kind_mode == wl.KIND_MIX_ACC_A
    b = orc.decode_array(w.B, orc.FP16)
    assert abs(b.std() - 0.02) < 0.001
    sub = (np.abs(b) < 2.0 ** -14) & (b != 0)
    assert 0.001 < sub.mean() < 0.005          # FP16 subnormal weights do occur
    r = wl.resnet_conv()
    assert (r.M, r.K, r.N, r.fmt) == (3136, 576, 64, wl.BF16)
    a = orc.decode_array(r.A, orc.BF16)
    assert a.min() == 0 and 0.48 < (a == 0).mean() < 0.52
    assert abs(orc.decode_array(r.B, orc.BF16).std() - np.sqrt(2 / 576)) < 0.003


def test_detector_stress_rows():
    w = wl.detector_stress()
    a = orc.decode_array(w.A, orc.FP16)
    heavy = np.abs(a).max(axis=1) > 50
    assert heavy.sum() == 205 and np.isfinite(a).all()
    assert w.policies == (wl.CORRECT_ZERO, wl.CORRECT_RECOMPUTE) and w.nbits == 2
