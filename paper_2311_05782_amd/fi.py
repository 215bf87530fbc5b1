"""Thin binding over the C-ABI library libfi_gfx950.so (see include/fi.h).

Argument marshalling only: every step of a campaign runs in the library's HIP
kernels.  PyTorch provides device memory and streams, nothing else.  There is
no fallback: if the library is missing or no gfx950 device is present, the
calls raise.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# FI_LIBRARY selects another build of the same ABI (e.g. a tuning experiment).
LIB_PATH = os.environ.get("FI_LIBRARY") or os.path.join(_HERE, "libfi_gfx950.so")

OK, INVALID_ARG, UNSUPPORTED, OOM, DEVICE, STATE = range(6)
FP16, BF16 = 0, 1
SITE_NONE, SITE_ACC, SITE_A, SITE_B, SITE_PRODUCT = 0, 1, 2, 3, 4
CORRECT_NONE, CORRECT_ZERO, CORRECT_RECOMPUTE = 0, 1, 2
BOUND_ROWCOL, BOUND_GLOBAL, BOUND_EXPONENT = 0, 1, 2
MASKED, SDC, DETECTED = 0, 1, 2
PCHECK_NONE, PCHECK_BOUND, PCHECK_RANGE_MAX, PCHECK_RANGE_FLIP = 0, 1, 2, 3
HIST_SITE, HIST_DEV_PRE, HIST_DEV_POST = 0, 1, 2
KIND_ALL_ACC, KIND_ALL_A, KIND_ALL_B, KIND_MIX_ACC_A, KIND_ALL_PRODUCT = 0, 1, 2, 3, 4
BUF_C_STAR, BUF_S_ABS, BUF_KRA, BUF_CB = 0, 1, 2, 3

# Symbols include/fi.h declares; the loader checks every one.
EXPORTS = ["fi_plan_create", "fi_plan_destroy", "fi_plan_buffer", "fi_plan_tune", "fi_plan_describe",
           "fi_plan_set_product_check", "fi_plan_reserve", "fi_plan_set_clock_sink", "fi_probe_mfma_loop", "fi_deviation_histogram",
           "fi_gemm_inject_batch", "fi_gemm_inject_batch_act", "fi_gemm_inject_batch_noalloc", "fi_gemm_inject_batch_affected", "fi_detect_correct", "fi_classify", "fi_sample_faults",
           "fi_activation_round", "fi_gemm_propagate_batch", "fi_last_error", "fi_build_info"]

FAULT_DTYPE = np.dtype([("kind", "<u4"), ("row", "<u4"), ("col", "<u4"), ("kblock", "<u4"),
                        ("xor_mask", "<u4")])
RESULT_DTYPE = np.dtype([("n_flagged", "<u4"), ("n_bitdiff", "<u4"), ("n_dev_pre", "<u4"),
                         ("n_dev_post", "<u4"), ("max_dev_pre", "<f4"), ("max_dev_post", "<f4"),
                         ("site_word_before", "<u4"), ("site_word_after", "<u4"),
                         ("n_border_T", "<u4"), ("n_border_tau", "<u4"), ("status", "<u4"),
                         ("product_flag", "<u4")])
assert FAULT_DTYPE.itemsize == 20 and RESULT_DTYPE.itemsize == 48


class PlanDesc(C.Structure):
    _fields_ = [("M", C.c_uint32), ("N", C.c_uint32), ("K", C.c_uint32), ("k_block", C.c_uint32),
                ("dtype", C.c_uint32), ("b_layout", C.c_uint32), ("bound_mode", C.c_uint32),
                ("gamma", C.c_float), ("lda", C.c_int64), ("ldb", C.c_int64)]


class FiError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("fi status %d: %s" % (status, message))
        self.status = status


_lib = None


def lib():
    """Load the built library; build it first only if nothing is built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build(force=True)
    # PyTorch ships its own HIP runtime with the same soname the library asks for; importing
    # torch first makes the loader bind the library to that one runtime, so torch's streams
    # and allocations are valid inside the library.
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    for name in EXPORTS:
        if not hasattr(L, name):
            raise ImportError("%s does not export %s" % (LIB_PATH, name))
    vp = C.c_void_p
    L.fi_last_error.restype = C.c_char_p
    L.fi_last_error.argtypes = []
    L.fi_build_info.restype = C.c_char_p
    L.fi_build_info.argtypes = []
    # A binary older than the sources beside it is refused, not silently used.
    if not os.environ.get("FI_LIBRARY"):
        from . import build as _build
        built, now = L.fi_build_info().decode(), _build.sources_digest()
        if built != now:
            raise ImportError("%s was built from other sources (%s..., now %s...): run "
                              "python paper_2311_05782_amd/build.py" % (LIB_PATH, built[:12], now[:12]))
    L.fi_plan_create.argtypes = [C.POINTER(PlanDesc), vp, vp, vp, C.POINTER(vp)]
    L.fi_plan_destroy.argtypes = [vp]
    L.fi_plan_buffer.argtypes = [vp, C.c_uint32, C.POINTER(vp)]
    L.fi_plan_tune.argtypes = [vp, C.c_int32, C.c_int32, vp]
    L.fi_plan_describe.argtypes = [vp, C.c_char_p, C.c_uint64]
    L.fi_plan_set_product_check.argtypes = [vp, C.c_uint32]
    L.fi_plan_reserve.argtypes = [vp, C.c_uint32, vp]
    L.fi_plan_set_clock_sink.argtypes = [vp, vp]
    L.fi_probe_mfma_loop.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, vp, vp, vp]
    L.fi_gemm_inject_batch.argtypes = [vp, vp, C.c_uint32, C.c_uint32, vp, vp, vp]
    L.fi_gemm_inject_batch_noalloc.argtypes = [vp, vp, C.c_uint32, C.c_uint32, vp, vp, vp]
    L.fi_gemm_inject_batch_act.argtypes = [vp, vp, C.c_uint32, C.c_uint32, vp, vp, vp]
    L.fi_gemm_inject_batch_affected.argtypes = [vp, vp, C.c_uint32, C.c_uint32, vp, vp]
    L.fi_detect_correct.argtypes = [vp, vp, C.c_uint32, C.c_uint32, vp, vp, vp]
    L.fi_activation_round.argtypes = [C.c_uint32, vp, C.c_uint64, vp, vp]
    L.fi_gemm_propagate_batch.argtypes = [vp, vp, C.c_uint64, C.c_uint32, C.c_uint32, vp, vp, vp]
    L.fi_classify.argtypes = [vp, vp, C.c_uint32, vp, vp, vp]
    L.fi_deviation_histogram.argtypes = [vp, vp, vp, C.c_uint32, C.c_uint32, vp, vp]
    L.fi_sample_faults.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.POINTER(PlanDesc), C.c_uint32,
                                   C.c_uint32, vp]
    for name in EXPORTS:
        if name not in ("fi_last_error", "fi_build_info"):
            getattr(L, name).restype = C.c_int32
    _lib = L
    return L


def _check(status):
    if status != OK:
        raise FiError(status, lib().fi_last_error().decode("utf-8", "replace"))


def _dptr(t):
    """Device pointer of a torch tensor (or a raw int / None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return C.c_void_p(stream)
    return C.c_void_p(stream.cuda_stream)


def plan_desc(M, N, K, k_block, dtype, b_layout=0, bound_mode=BOUND_ROWCOL, gamma=0.0, lda=None, ldb=None):
    if lda is None:
        lda = K
    if ldb is None:
        ldb = K if b_layout == 0 else N
    return PlanDesc(M, N, K, k_block, dtype, b_layout, bound_mode, gamma, lda, ldb)


def fi_sample_faults(seed, first_trial, n_trials, desc, kind_mode, nbits):
    """Host-side fault list as a NumPy structured array (FAULT_DTYPE)."""
    out = np.zeros(n_trials, FAULT_DTYPE)
    _check(lib().fi_sample_faults(seed, first_trial, n_trials, C.byref(desc), kind_mode, nbits,
                                  out.ctypes.data_as(C.c_void_p)))
    return out


def fi_probe_mfma_loop(dtype, random_data, iters, n_workgroups, d_sink, d_clocks=None, stream=None):
    _check(lib().fi_probe_mfma_loop(dtype, random_data, iters, n_workgroups, _dptr(d_sink), _dptr(d_clocks),
                                    _stream(stream)))


def fi_activation_round(dtype, d_c, n, d_h, stream=None):
    _check(lib().fi_activation_round(dtype, _dptr(d_c), n, _dptr(d_h), _stream(stream)))


class Plan:
    """Owns one fi_plan.  d_A / d_B are torch uint16-sized device tensors kept alive here."""

    def __init__(self, desc, d_A, d_B, stream=None):
        self.desc = desc
        self._keep = (d_A, d_B)
        self._h = C.c_void_p()
        _check(lib().fi_plan_create(C.byref(desc), _dptr(d_A), _dptr(d_B), _stream(stream), C.byref(self._h)))

    @property
    def handle(self):
        return self._h

    def buffer_ptr(self, which):
        p = C.c_void_p()
        _check(lib().fi_plan_buffer(self._h, which, C.byref(p)))
        return p.value

    def buffer_to_host(self, which):
        """Copy a plan-owned array to the host (tests and reports)."""
        import torch
        d = self.desc
        shape = {BUF_C_STAR: (d.M, d.N), BUF_S_ABS: (d.M, d.N), BUF_KRA: (d.M,), BUF_CB: (d.N,)}[which]
        n = int(np.prod(shape))
        out = torch.empty(n, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        hip = _hip()
        rc = hip.hipMemcpy(C.c_void_p(out.data_ptr()), C.c_void_p(self.buffer_ptr(which)), C.c_size_t(n * 4), 3)
        if rc != 0:
            raise RuntimeError("hipMemcpy failed: %d" % rc)
        return out.cpu().numpy().reshape(shape)

    def tune(self, tile_config=-1, trial_group=-1, stream=None):
        _check(lib().fi_plan_tune(self._h, tile_config, trial_group, _stream(stream)))

    def reserve(self, max_trials, stream=None):
        _check(lib().fi_plan_reserve(self._h, max_trials, _stream(stream)))

    def set_clock_sink(self, d_clocks):
        self._clock_keep = d_clocks
        _check(lib().fi_plan_set_clock_sink(self._h, _dptr(d_clocks)))

    def set_product_check(self, mode):
        _check(lib().fi_plan_set_product_check(self._h, mode))

    def describe(self):
        buf = C.create_string_buffer(512)
        _check(lib().fi_plan_describe(self._h, buf, len(buf)))
        return buf.value.decode()

    def fi_gemm_inject_batch(self, d_faults, n_trials, policy, d_results, d_c_out=None, stream=None):
        _check(lib().fi_gemm_inject_batch(self._h, _dptr(d_faults), n_trials, policy, _dptr(d_results),
                                          _dptr(d_c_out), _stream(stream)))

    def fi_gemm_inject_batch_act(self, d_faults, n_trials, policy, d_results, d_h_out, stream=None):
        _check(lib().fi_gemm_inject_batch_act(self._h, _dptr(d_faults), n_trials, policy, _dptr(d_results),
                                              _dptr(d_h_out), _stream(stream)))

    def fi_gemm_inject_batch_noalloc(self, d_faults, n_trials, policy, d_results, d_c_out=None, stream=None):
        _check(lib().fi_gemm_inject_batch_noalloc(self._h, _dptr(d_faults), n_trials, policy, _dptr(d_results),
                                                  _dptr(d_c_out), _stream(stream)))

    def fi_deviation_histogram(self, d_faults, d_results, n_trials, which, d_hist, stream=None):
        _check(lib().fi_deviation_histogram(self._h, _dptr(d_faults), _dptr(d_results), n_trials, which,
                                            _dptr(d_hist), _stream(stream)))

    def fi_gemm_inject_batch_affected(self, d_faults, n_trials, policy, d_results, stream=None):
        _check(lib().fi_gemm_inject_batch_affected(self._h, _dptr(d_faults), n_trials, policy, _dptr(d_results),
                                                   _stream(stream)))

    def fi_gemm_propagate_batch(self, d_a_stack, trial_stride, n_trials, policy, d_results, d_c_out=None, stream=None):
        _check(lib().fi_gemm_propagate_batch(self._h, _dptr(d_a_stack), trial_stride, n_trials, policy,
                                             _dptr(d_results), _dptr(d_c_out), _stream(stream)))

    def fi_detect_correct(self, d_c, batch, policy, d_flags=None, d_n_flagged=None, stream=None):
        _check(lib().fi_detect_correct(self._h, _dptr(d_c), batch, policy, _dptr(d_flags),
                                       _dptr(d_n_flagged), _stream(stream)))

    def fi_classify(self, d_results, n_trials, d_class, d_counts, stream=None):
        _check(lib().fi_classify(self._h, _dptr(d_results), n_trials, _dptr(d_class), _dptr(d_counts),
                                 _stream(stream)))

    def destroy(self):
        if self._h:
            _check(lib().fi_plan_destroy(self._h))
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


_hip_lib = None


def _hip():
    global _hip_lib
    if _hip_lib is None:
        _hip_lib = C.CDLL("libamdhip64.so.7")   # the runtime torch already loaded
        _hip_lib.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        _hip_lib.hipMemcpy.restype = C.c_int
    return _hip_lib


# ---- marshalling helpers: NumPy structured arrays <-> device byte tensors -----------------

def to_device(arr):
    """Host NumPy array (any dtype, structured included) -> torch uint8 device tensor."""
    import torch
    raw = np.ascontiguousarray(arr).view(np.uint8).reshape(-1)
    return torch.from_numpy(raw.copy()).to("cuda")


def words_to_device(words):
    """uint16 operand bit patterns -> device tensor of the same shape (int16 storage)."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(words).view(np.int16).copy()).to("cuda")


def empty_results(n_trials):
    import torch
    return torch.empty(n_trials * RESULT_DTYPE.itemsize, dtype=torch.uint8, device="cuda")


def results_to_host(d_results):
    import torch
    torch.cuda.synchronize()
    return d_results.cpu().numpy().view(RESULT_DTYPE).copy()
