"""ctypes loader for the CPU oracle (test infrastructure, never used by the product path).

Only tests, the smoke check and the benchmark's cpu_baseline leg import this.
The record / fault dtypes below mirror oracle/fi_oracle.h and nothing else.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fi_oracle.c")
_LIB = os.path.join(_HERE, "libfi_oracle.so")

FP16, BF16 = 0, 1
SITE_NONE, SITE_ACC, SITE_A, SITE_B, SITE_PRODUCT = 0, 1, 2, 3, 4
CORRECT_NONE, CORRECT_ZERO, CORRECT_RECOMPUTE = 0, 1, 2
BOUND_ROWCOL, BOUND_GLOBAL, BOUND_EXPONENT = 0, 1, 2
MASKED, SDC, DETECTED = 0, 1, 2
MODE_FULL, MODE_AFFECTED = 0, 1
KIND_ALL_ACC, KIND_ALL_A, KIND_ALL_B, KIND_MIX_ACC_A, KIND_ALL_PRODUCT = 0, 1, 2, 3, 4


class Problem(C.Structure):
    _fields_ = [("M", C.c_int), ("N", C.c_int), ("K", C.c_int), ("kb", C.c_int),
                ("fmt", C.c_int), ("b_layout", C.c_int), ("bound_mode", C.c_int),
                ("gamma", C.c_float), ("lda", C.c_long), ("ldb", C.c_long), ("product_check", C.c_int)]


FAULT_DTYPE = np.dtype([("kind", "<u4"), ("row", "<u4"), ("col", "<u4"),
                        ("kblock", "<u4"), ("xor_mask", "<u4")])

RECORD_DTYPE = np.dtype([("max_dev_pre", "<f8"), ("max_dev_post", "<f8"),
                         ("n_flagged", "<u4"), ("n_bitdiff", "<u4"),
                         ("n_dev_pre", "<u4"), ("n_dev_post", "<u4"),
                         ("site_word_before", "<u4"), ("site_word_after", "<u4"),
                         ("n_border_T", "<u4"), ("n_border_tau", "<u4"),
                         ("valid", "<u4"), ("cls", "<u4"), ("product_flag", "<u4"), ("reserved", "<u4")])
PCHECK_NONE, PCHECK_BOUND, PCHECK_RANGE_MAX, PCHECK_RANGE_FLIP = 0, 1, 2, 3

DEFAULT_GAMMA = 1.0 + 2.0 ** -11


# FI_ORACLE_SANITIZE=1 builds and loads an AddressSanitizer + UndefinedBehaviorSanitizer build of
# the oracle instead (CPU only; run the interpreter with libasan preloaded).
_SANITIZE = bool(os.environ.get("FI_ORACLE_SANITIZE"))
if _SANITIZE:
    _LIB = os.path.join(_HERE, "libfi_oracle_san.so")


def build(force=False):
    """Compile the oracle with gcc.  -ffp-contract=off keeps a*b+c as two roundings."""
    if os.path.exists(_LIB) and not force and os.path.getmtime(_LIB) >= max(
            os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "fi_oracle.h"))):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-Wall", "-Wextra", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"]
    if _SANITIZE:
        cmd[1:1] = ["-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        vp, u16p, f32p, f64p = C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p
        PP = C.POINTER(Problem)
        L.orc_decode16.restype = C.c_float
        L.orc_decode16.argtypes = [C.c_uint16, C.c_int]
        L.orc_round16.restype = C.c_uint16
        L.orc_round16.argtypes = [C.c_float, C.c_int]
        L.orc_product_check.restype = C.c_uint16
        L.orc_product_check.argtypes = [C.c_uint16, C.c_uint16, C.c_uint16, C.c_int, C.c_int, C.POINTER(C.c_int)]
        L.orc_decode_array.restype = None
        L.orc_decode_array.argtypes = [u16p, C.c_size_t, C.c_int, f32p]
        L.orc_dot.restype = C.c_float
        L.orc_dot.argtypes = [PP, u16p, u16p, C.c_int, C.c_int]
        L.orc_gemm.restype = C.c_int
        L.orc_gemm.argtypes = [PP, u16p, u16p, f32p, f64p, f64p]
        L.orc_rowcol_absmax.restype = C.c_int
        L.orc_rowcol_absmax.argtypes = [PP, u16p, u16p, f32p, f32p]
        L.orc_default_gamma.restype = C.c_float
        L.orc_default_gamma.argtypes = [C.c_int]
        L.orc_threshold.restype = C.c_float
        L.orc_threshold.argtypes = [C.c_int, C.c_float, C.c_float, C.c_float]
        L.orc_detect_correct.restype = C.c_int
        L.orc_detect_correct.argtypes = [PP, f32p, f32p, f32p, C.c_int, C.c_int, f32p, vp, vp]
        L.orc_trial.restype = C.c_int
        L.orc_trial.argtypes = [PP, u16p, u16p, vp, C.c_int, C.c_int, f32p, f32p, vp]
        L.orc_campaign.restype = C.c_int
        L.orc_campaign.argtypes = [PP, u16p, u16p, vp, C.c_int, C.c_int, C.c_int, vp]
        L.orc_deviation_histogram.restype = None
        L.orc_deviation_histogram.argtypes = [vp, vp, C.c_int, C.c_int, vp]
        L.orc_activation_round.restype = None
        L.orc_activation_round.argtypes = [f32p, C.c_size_t, C.c_int, u16p]
        L.orc_propagate.restype = C.c_int
        L.orc_propagate.argtypes = [PP, u16p, u16p, u16p, C.c_size_t, C.c_int, C.c_int, C.c_int, f32p, vp]
        L.orc_classify.restype = None
        L.orc_classify.argtypes = [vp, C.c_int, vp, vp]
        L.orc_splitmix64_next.restype = C.c_uint64
        L.orc_splitmix64_next.argtypes = [C.POINTER(C.c_uint64)]
        L.orc_sample_faults.restype = C.c_int
        L.orc_sample_faults.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, PP, C.c_int, C.c_int, vp]
        L.orc_threads.restype = C.c_int
        L.orc_threads.argtypes = []
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def default_gamma(K):
    return float(lib().orc_default_gamma(int(K)))


def problem(M, N, K, kb, fmt, b_layout=0, bound_mode=BOUND_ROWCOL, gamma=None,
            lda=None, ldb=None, product_check=0):
    if gamma is None:
        gamma = default_gamma(K)
    if lda is None:
        lda = K
    if ldb is None:
        ldb = K if b_layout == 0 else N
    return Problem(M, N, K, kb, fmt, b_layout, bound_mode, gamma, lda, ldb, product_check)


def decode16(w, fmt):
    return float(np.float32(lib().orc_decode16(int(w), fmt)))


def round16(x, fmt):
    """binary32 value -> FP16 / BF16 word, round to nearest even."""
    return int(lib().orc_round16(float(np.float32(x)), fmt))


def product_check(w_err, w_a, w_b, fmt, mode):
    """(corrected word, fired) of the exponent-only check of Sec. VI-A."""
    fired = C.c_int(0)
    w = lib().orc_product_check(int(w_err), int(w_a), int(w_b), fmt, mode, C.byref(fired))
    return int(w), int(fired.value)


def decode_array(words, fmt):
    words = _u16(words)
    out = np.empty(words.shape, np.float32)
    lib().orc_decode_array(_ptr(words), words.size, fmt, _ptr(out))
    return out


def dot(p, A, B, i, j):
    A, B = _u16(A), _u16(B)
    return np.float32(lib().orc_dot(C.byref(p), _ptr(A), _ptr(B), i, j))


def gemm(p, A, B, want_double=False):
    A, B = _u16(A), _u16(B)
    Cm = np.empty((p.M, p.N), np.float32)
    R = np.empty((p.M, p.N), np.float64) if want_double else None
    S = np.empty((p.M, p.N), np.float64) if want_double else None
    rc = lib().orc_gemm(C.byref(p), _ptr(A), _ptr(B), _ptr(Cm), _ptr(R), _ptr(S))
    if rc:
        raise ValueError("orc_gemm failed: %d" % rc)
    return (Cm, R, S) if want_double else Cm


def rowcol_absmax(p, A, B):
    A, B = _u16(A), _u16(B)
    ra = np.empty(p.M, np.float32)
    cb = np.empty(p.N, np.float32)
    rc = lib().orc_rowcol_absmax(C.byref(p), _ptr(A), _ptr(B), _ptr(ra), _ptr(cb))
    if rc == 1:
        raise ValueError("orc_rowcol_absmax: bad arguments")
    return ra, cb, rc == 0


def threshold(K, ra, cb, gamma=DEFAULT_GAMMA):
    return np.float32(lib().orc_threshold(int(K), float(ra), float(cb), float(gamma)))


def detect_correct(p, ra, cb, Cb, policy, c_star=None, want_flags=True):
    """Returns (corrected copy, flags or None, n_flagged[batch])."""
    Cb = np.array(Cb, dtype=np.float32, copy=True).reshape(-1, p.M, p.N)
    batch = Cb.shape[0]
    flags = np.empty(Cb.shape, np.uint8) if want_flags else None
    nfl = np.zeros(batch, np.uint32)
    ra = np.ascontiguousarray(ra, np.float32)
    cb = np.ascontiguousarray(cb, np.float32)
    cs = None if c_star is None else np.ascontiguousarray(c_star, np.float32)
    rc = lib().orc_detect_correct(C.byref(p), _ptr(ra), _ptr(cb), _ptr(Cb), batch, policy,
                                  _ptr(cs), _ptr(flags), _ptr(nfl))
    if rc:
        raise ValueError("orc_detect_correct failed: %d" % rc)
    return Cb, flags, nfl


def make_faults(rows):
    """rows: iterable of (kind, row, col, kblock, xor_mask)."""
    rows = list(rows)
    out = np.zeros(len(rows), FAULT_DTYPE)
    for t, r in enumerate(rows):
        out[t] = tuple(int(x) for x in r)
    return out


def trial(p, A, B, fault, policy, mode=MODE_FULL, want_outputs=False):
    A, B = _u16(A), _u16(B)
    f = make_faults([fault]) if not isinstance(fault, np.ndarray) else fault
    rec = np.zeros(1, RECORD_DTYPE)
    cf = np.empty((p.M, p.N), np.float32) if want_outputs else None
    cc = np.empty((p.M, p.N), np.float32) if want_outputs else None
    rc = lib().orc_trial(C.byref(p), _ptr(A), _ptr(B), _ptr(f), policy, mode,
                         _ptr(cf), _ptr(cc), _ptr(rec))
    if rc:
        raise ValueError("orc_trial failed: %d" % rc)
    return (rec[0], cf, cc) if want_outputs else rec[0]


def campaign(p, A, B, faults, policy, mode=MODE_AFFECTED):
    A, B = _u16(A), _u16(B)
    faults = np.ascontiguousarray(faults)
    assert faults.dtype == FAULT_DTYPE
    recs = np.zeros(len(faults), RECORD_DTYPE)
    rc = lib().orc_campaign(C.byref(p), _ptr(A), _ptr(B), _ptr(faults), len(faults), policy,
                            mode, _ptr(recs))
    if rc:
        raise ValueError("orc_campaign failed: %d" % rc)
    return recs


def activation_round(c, fmt):
    """h = RNE_fmt(relu(c)) as 16-bit words, same shape as c."""
    c = np.ascontiguousarray(c, np.float32)
    h = np.empty(c.shape, np.uint16)
    lib().orc_activation_round(_ptr(c), c.size, fmt, _ptr(h))
    return h


def propagate(p, A, B, A_stack, policy, mode=MODE_FULL, want_outputs=False):
    """A_stack: [n_trials, M, lda] words, trial t's own A operand.  Returns records (and the
    corrected outputs [n_trials, M, N])."""
    A, B = _u16(A), _u16(B)
    A_stack = _u16(A_stack)
    assert A_stack.ndim == 3 and A_stack.shape[1] == p.M and A_stack.shape[2] == p.lda
    n = A_stack.shape[0]
    recs = np.zeros(n, RECORD_DTYPE)
    cc = np.empty((n, p.M, p.N), np.float32) if want_outputs else None
    rc = lib().orc_propagate(C.byref(p), _ptr(A), _ptr(B), _ptr(A_stack), p.M * p.lda, n, policy, mode,
                             _ptr(cc), _ptr(recs))
    if rc:
        raise ValueError("orc_propagate failed: %d" % rc)
    return (recs, cc) if want_outputs else recs


HIST_SITE, HIST_DEV_PRE, HIST_DEV_POST = 0, 1, 2


def deviation_histogram(recs, faults, which):
    """256 log2 bins (binary32 exponent field) of a per-trial deviation; see fi_oracle.h."""
    recs = np.ascontiguousarray(recs)
    faults = np.ascontiguousarray(faults)
    assert recs.dtype == RECORD_DTYPE and faults.dtype == FAULT_DTYPE and len(recs) == len(faults)
    hist = np.zeros(256, np.uint64)
    lib().orc_deviation_histogram(_ptr(recs), _ptr(faults), len(recs), which, _ptr(hist))
    return hist


def classify(recs):
    recs = np.ascontiguousarray(recs)
    cls = np.empty(len(recs), np.uint8)
    counts = np.zeros(3, np.uint64)
    lib().orc_classify(_ptr(recs), len(recs), _ptr(cls), _ptr(counts))
    return cls, counts


def splitmix64_stream(state, n):
    st = C.c_uint64(state)
    return [int(lib().orc_splitmix64_next(C.byref(st))) for _ in range(n)]


def sample_faults(seed, first_trial, n_trials, p, kind_mode, nbits):
    out = np.zeros(n_trials, FAULT_DTYPE)
    rc = lib().orc_sample_faults(seed, first_trial, n_trials, C.byref(p), kind_mode, nbits, _ptr(out))
    if rc:
        raise ValueError("orc_sample_faults failed: %d" % rc)
    return out


def threads():
    return int(lib().orc_threads())
