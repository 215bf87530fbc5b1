"""Seeded synthetic inputs for fault-injection campaigns on DNN-shaped GEMMs.

This module only *draws inputs*: operand bit patterns with the shapes, value
distributions and sparsity of the workloads, plus the campaign parameters that
go with them.  It holds none of the method's arithmetic (no GEMM, no fault
application, no detector) and is the one module that both the GPU path's
callers and the CPU checker's callers may import.  NumPy only.

The paper evaluates on trained models (Table I); neither their datasets nor
their weights are available offline, so these synthetic operands stand in for
one GEMM of such a model: a linear layer of a transformer encoder, an im2col'd
3x3 convolution after a ReLU, and square stress shapes.
"""
from dataclasses import dataclass, field

import numpy as np

FP16, BF16 = 0, 1
KIND_ALL_ACC, KIND_ALL_A, KIND_ALL_B, KIND_MIX_ACC_A = 0, 1, 2, 3
CORRECT_NONE, CORRECT_ZERO, CORRECT_RECOMPUTE = 0, 1, 2


def to_fp16_words(x):
    """float32 array -> IEEE binary16 bit patterns, round-to-nearest-even."""
    return np.asarray(x, np.float32).astype(np.float16).view(np.uint16)


def to_bf16_words(x):
    """float32 array -> bfloat16 bit patterns, round-to-nearest-even (finite inputs)."""
    bits = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    return ((bits + 0x7FFF + lsb) >> 16).astype(np.uint16)


def to_words(x, fmt):
    return to_fp16_words(x) if fmt == FP16 else to_bf16_words(x)


@dataclass
class Workload:
    name: str
    M: int
    N: int
    K: int
    kb: int
    fmt: int
    n_trials: int
    kind_mode: int
    nbits: int
    policies: tuple
    input_seed: int = 0
    fault_seed: int = 0
    A: np.ndarray = field(default=None, repr=False)   # [M, K] uint16
    B: np.ndarray = field(default=None, repr=False)   # [N, K] uint16 (column j of B is row j)

    @property
    def flops_per_trial(self):
        return 2.0 * self.M * self.N * self.K


def _finish(w, a32, b32):
    w.A = np.ascontiguousarray(to_words(a32, w.fmt))
    w.B = np.ascontiguousarray(to_words(b32, w.fmt))
    return w


def tiny(seed=0):
    """128^3 FP16, N(0,1) operands, k-block 32, 64 single-bit accumulator faults."""
    w = Workload("tiny128", 128, 128, 128, 32, FP16, 64, KIND_ALL_ACC, 1, (CORRECT_ZERO,), seed, 0)
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((w.M, w.K), dtype=np.float32)
    b = rng.standard_normal((w.N, w.K), dtype=np.float32)
    return _finish(w, a, b)


def bert_linear(seed=1):
    """512x768 activations ~N(0,1) times 768x3072 weights ~N(0,0.02), FP16."""
    w = Workload("bert_linear", 512, 3072, 768, 32, FP16, 4096, KIND_MIX_ACC_A, 1,
                 (CORRECT_RECOMPUTE,), seed, 1)
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((w.M, w.K), dtype=np.float32)
    b = rng.standard_normal((w.N, w.K), dtype=np.float32) * np.float32(0.02)
    return _finish(w, a, b)


def resnet_conv(seed=2):
    """56x56 output pixels x (3x3x64) patches x 64 filters, BF16, ReLU'd activations.

    Patches are drawn iid (a real im2col repeats each pixel in up to 9 rows)."""
    w = Workload("resnet_conv", 3136, 64, 576, 32, BF16, 8192, KIND_ALL_ACC, 1,
                 (CORRECT_ZERO,), seed, 2)
    rng = np.random.default_rng(seed)
    a = np.maximum(rng.standard_normal((w.M, w.K), dtype=np.float32), np.float32(0))
    b = rng.standard_normal((w.N, w.K), dtype=np.float32) * np.float32(np.sqrt(2.0 / 576.0))
    return _finish(w, a, b)


def square4096(seed=3):
    """4096^3 BF16, U(-1,1) operands, k-block 64, 1024 accumulator faults per batch."""
    w = Workload("square4096", 4096, 4096, 4096, 64, BF16, 1024, KIND_ALL_ACC, 1,
                 (CORRECT_ZERO,), seed, 3)
    rng = np.random.default_rng(seed)
    a = rng.random((w.M, w.K), dtype=np.float32) * np.float32(2) - np.float32(1)
    b = rng.random((w.N, w.K), dtype=np.float32) * np.float32(2) - np.float32(1)
    return _finish(w, a, b)


def detector_stress(seed=4):
    """1024^3 FP16 N(0,1) with round(0.2*M) seeded rows of A scaled by 100; 2-bit bursts."""
    w = Workload("detector_stress", 1024, 1024, 1024, 32, FP16, 16384, KIND_ALL_ACC, 2,
                 (CORRECT_ZERO, CORRECT_RECOMPUTE), seed, 4)
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((w.M, w.K), dtype=np.float32)
    b = rng.standard_normal((w.N, w.K), dtype=np.float32)
    heavy = rng.permutation(w.M)[: int(round(0.2 * w.M))]
    a[heavy, :] *= np.float32(100)
    return _finish(w, a, b)


def small_integers(M, N, K, fmt, seed=0, lim=4, step=1):
    """Operands are multiples of `step` in [-lim, lim]: every product and partial sum is an
    exactly representable integer, so any summation order gives the same bits."""
    rng = np.random.default_rng(seed)
    n = lim // step
    a = (rng.integers(-n, n + 1, size=(M, K)) * step).astype(np.float32)
    b = (rng.integers(-n, n + 1, size=(N, K)) * step).astype(np.float32)
    return to_words(a, fmt), to_words(b, fmt)


def gaussian(M, N, K, fmt, seed=0, scale_a=1.0, scale_b=1.0):
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((M, K), dtype=np.float32) * np.float32(scale_a)
    b = rng.standard_normal((N, K), dtype=np.float32) * np.float32(scale_b)
    return to_words(a, fmt), to_words(b, fmt)


def two_layer_mlp(M=512, D=768, H=3072, fmt=BF16, seed=5):
    """Inputs of a two-layer feed-forward block Y = relu(X W1) W2 with the shapes of a
    transformer encoder's (D -> H -> D): X [M][D] ~ N(0,1), W1 [H][D] and W2 [D][H] ~ N(0, 0.02),
    both weight matrices stored with the contraction index contiguous.  Returns the three word
    arrays; seeded, synthetic (no trained weights)."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, D), dtype=np.float32)
    w1 = rng.standard_normal((H, D), dtype=np.float32) * np.float32(0.02)
    w2 = rng.standard_normal((D, H), dtype=np.float32) * np.float32(0.02)
    return to_words(x, fmt), to_words(w1, fmt), to_words(w2, fmt)


ALL = {"tiny128": tiny, "bert_linear": bert_linear, "resnet_conv": resnet_conv,
       "square4096": square4096, "detector_stress": detector_stress}
