"""Host-side checks of the C-ABI library: it loads, exports what include/fi.h declares,
rejects bad arguments before touching a device, and its sampler equals the oracle's."""
import ctypes as C
import os
import re
import subprocess

import numpy as np
import pytest

from oracle import pyoracle as orc
from paper_2311_05782_amd import fi

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "fi.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fi_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = fi.lib()
    declared = _declared()
    assert sorted(fi.EXPORTS) == declared
    nm = subprocess.run(["nm", "-D", "--defined-only", fi.LIB_PATH], stdout=subprocess.PIPE, text=True).stdout
    exported = set(re.findall(r" T (fi_[a-z_]+)", nm))
    assert set(declared) <= exported
    for name in declared:
        assert getattr(L, name) is not None


def test_struct_layouts_match_header():
    text = open(os.path.join(ROOT, "include", "fi.h")).read()
    m = re.search(r"typedef struct \{([^}]*)\} fi_trial_result;", text, flags=re.S)
    body = re.sub(r"/\*.*?\*/", "", m.group(1), flags=re.S)
    names = re.findall(r"(\w+)\s*[;,]", body)
    assert names == list(fi.RESULT_DTYPE.names)
    m = re.search(r"typedef struct \{([^}]*)\} fi_fault;", text, flags=re.S)
    assert re.findall(r"(\w+)\s*[;,]", m.group(1)) == list(fi.FAULT_DTYPE.names)
    assert C.sizeof(fi.PlanDesc) == 48


@pytest.mark.parametrize("kind_mode,nbits", [(0, 1), (0, 2), (1, 1), (2, 4), (3, 1), (4, 1), (4, 2), (4, 4)])
def test_sampler_equals_oracle(kind_mode, nbits):
    for (M, N, K, kb, seed, first) in [(128, 128, 128, 32, 0, 0), (512, 3072, 768, 32, 1, 100),
                                       (3136, 64, 576, 32, 2 ** 63 + 5, 7), (4096, 4096, 4096, 64, 3, 0)]:
        mine = fi.fi_sample_faults(seed, first, 300, fi.plan_desc(M, N, K, kb, fi.BF16), kind_mode, nbits)
        theirs = orc.sample_faults(seed, first, 300, orc.problem(M, N, K, kb, orc.BF16), kind_mode, nbits)
        assert mine.tobytes() == theirs.tobytes()


def _status(call):
    with pytest.raises(fi.FiError) as e:
        call()
    return e.value.status, str(e.value)


def test_argument_errors_need_no_device():
    good = fi.plan_desc(128, 128, 128, 32, fi.FP16)
    out = C.c_void_p()
    L = fi.lib()
    A = C.c_void_p(0x1000)
    B = C.c_void_p(0x2000)

    def create(desc, a=A, b=B, o=C.byref(out)):
        return lambda: fi._check(L.fi_plan_create(C.byref(desc) if desc else None, a, b, None, o))

    assert _status(create(None))[0] == fi.INVALID_ARG
    assert _status(create(fi.plan_desc(0, 128, 128, 32, fi.FP16)))[0] == fi.INVALID_ARG
    assert _status(create(fi.plan_desc(128, 128, 100, 32, fi.FP16)))[0] == fi.INVALID_ARG   # K % kb
    assert _status(create(fi.plan_desc(128, 128, 120, 24, fi.FP16)))[0] == fi.INVALID_ARG   # kb % 16
    assert _status(create(fi.plan_desc(128, 128, 128, 32, 2)))[0] == fi.UNSUPPORTED          # TF32 etc.
    assert _status(create(fi.plan_desc(128, 128, 128, 32, fi.FP16, gamma=0.5)))[0] == fi.INVALID_ARG
    assert _status(create(good, a=None))[0] == fi.INVALID_ARG
    assert _status(create(good, o=None))[0] == fi.INVALID_ARG
    assert _status(create(fi.plan_desc(128, 128, 128, 32, fi.FP16, lda=64)))[0] == fi.INVALID_ARG
    assert _status(create(good, a=C.c_void_p(0x1002)))[0] == fi.UNSUPPORTED                  # alignment
    assert _status(create(fi.plan_desc(128, 128, 128, 32, fi.FP16, lda=132)))[0] == fi.UNSUPPORTED
    assert out.value is None
    # NULL plans
    assert _status(lambda: fi._check(L.fi_plan_destroy(None)))[0] == fi.INVALID_ARG
    assert _status(lambda: fi._check(L.fi_gemm_inject_batch(None, A, 1, 0, B, None, None)))[0] == fi.INVALID_ARG
    assert _status(lambda: fi._check(L.fi_detect_correct(None, A, 1, 0, None, None, None)))[0] == fi.INVALID_ARG
    assert _status(lambda: fi._check(L.fi_classify(None, A, 1, None, B, None)))[0] == fi.INVALID_ARG
    assert _status(lambda: fi._check(L.fi_gemm_propagate_batch(None, A, 0, 1, 0, B, None, None)))[0] == fi.INVALID_ARG
    assert _status(lambda: fi._check(L.fi_gemm_inject_batch_affected(None, A, 1, 0, B, None)))[0] == fi.INVALID_ARG
    assert _status(lambda: fi._check(L.fi_plan_reserve(None, 16, None)))[0] == fi.INVALID_ARG
    assert _status(lambda: fi._check(L.fi_gemm_inject_batch_act(None, A, 1, 0, B, A, None)))[0] == fi.INVALID_ARG
    assert _status(lambda: fi._check(L.fi_gemm_inject_batch_noalloc(None, A, 1, 0, B, None, None)))[0] == fi.INVALID_ARG
    # a handle that is not a live plan (never created, or destroyed) is looked up, not dereferenced
    bogus = C.c_void_p(0x1000)
    assert _status(lambda: fi._check(L.fi_plan_destroy(bogus)))[0] == fi.STATE
    assert _status(lambda: fi._check(L.fi_plan_reserve(bogus, 16, None)))[0] == fi.STATE
    assert _status(lambda: fi._check(L.fi_gemm_inject_batch(bogus, A, 1, 0, B, None, None)))[0] == fi.STATE
    assert _status(lambda: fi._check(L.fi_classify(bogus, A, 1, None, B, None)))[0] == fi.STATE
    assert _status(lambda: fi._check(L.fi_gemm_inject_batch_act(bogus, A, 1, 0, B, A, None)))[0] == fi.STATE
    assert _status(lambda: fi._check(L.fi_gemm_inject_batch_noalloc(bogus, A, 1, 0, B, None, None)))[0] == fi.STATE
    # the hand-over kernel's arguments
    assert _status(lambda: fi._check(L.fi_activation_round(2, A, 16, B, None)))[0] == fi.UNSUPPORTED
    assert _status(lambda: fi._check(L.fi_activation_round(fi.BF16, None, 16, B, None)))[0] == fi.INVALID_ARG
    assert _status(lambda: fi._check(L.fi_activation_round(fi.BF16, A, 0, B, None)))[0] == fi.INVALID_ARG
    assert _status(lambda: fi._check(L.fi_activation_round(fi.BF16, A, 16, C.c_void_p(0x2008), None)))[0] == fi.UNSUPPORTED
    # sampler argument checks
    assert _status(lambda: fi.fi_sample_faults(0, 0, 4, good, 9, 1))[0] == fi.INVALID_ARG
    assert _status(lambda: fi.fi_sample_faults(0, 0, 4, good, 0, 0))[0] == fi.INVALID_ARG
    st, msg = _status(lambda: fi.fi_sample_faults(0, 0, 4, good, 0, 17))
    assert st == fi.INVALID_ARG and "nbits" in msg


def test_no_device_is_reported_not_hidden():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a device is present")
    out = C.c_void_p()
    good = fi.plan_desc(128, 128, 128, 32, fi.FP16)
    st, msg = _status(lambda: fi._check(fi.lib().fi_plan_create(C.byref(good), C.c_void_p(0x1000),
                                                              C.c_void_p(0x2000), None, C.byref(out))))
    assert st == fi.STATE and out.value is None


def test_library_reports_the_sources_it_was_built_from():
    from paper_2311_05782_amd import build
    L = fi.lib()
    assert L.fi_build_info().decode() == build.sources_digest()


def _one_trial_kernel_fetch_offsets(M, K, lda, BM, n_waves, kshift, m0):
    """Element offsets of every 16-byte chunk the one-trial kernel's staging fetches for one
    operand and one workgroup (the address arithmetic of its issue_tile, restated): row groups
    of 8 rows per wave instruction, lane = 8 * row-in-group + slot, fetched chunk = slot ^ g(row),
    rows past the end clamped to the last, chunks outside [0, K) fetched from the row's start."""
    out = []
    nkt = (K + kshift + 63) // 64
    groups = BM // 8 // n_waves
    for kt in range(nkt):
        k0 = kt * 64 - kshift
        inside = k0 >= 0 and k0 + 64 <= K
        for wave in range(n_waves):
            for c in range(groups):
                for lane in range(64):
                    row = (wave * groups + c) * 8 + (lane >> 3)
                    ch = ((lane & 7) ^ ((row & 7) ^ ((row >> 3) & 1))) * 8
                    goff = min(m0 + row, M - 1) * lda + ch
                    kin = 0 <= k0 + ch < K
                    out.append(goff + (k0 if (inside or kin) else -ch))
    return out


def test_one_trial_kernel_never_fetches_outside_its_operands():
    # Every chunk is 8 elements; it must lie inside [0, (M-1)*lda + K) for packed and padded rows,
    # K shorter than a k-tile, ragged tiles and every k-shift an accumulator fault can ask for.
    for (M, K, lda) in [(5, 16, 16), (128, 16, 16), (33, 48, 48), (300, 96, 96), (257, 128, 136), (64, 64, 64)]:
        for (BM, nw) in [(256, 8), (128, 4), (256, 4)]:
            for kshift in (0, 16, 32, 48):
                for m0 in range(0, M, BM):
                    offs = _one_trial_kernel_fetch_offsets(M, K, lda, BM, nw, kshift, m0)
                    assert min(offs) >= 0 and max(offs) + 8 <= (M - 1) * lda + K, (M, K, lda, BM, kshift, m0)
