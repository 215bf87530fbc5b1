"""Builds libfi_gfx950.so (the C-ABI library) in-tree with hipcc for gfx950.

The GEMM kernels are instantiated in one translation unit per (kernel family, operand format,
tile configuration) - csrc/gemm_inst.hip compiled with three -D switches - so the objects build
in parallel; csrc/fi_api.hip holds the C ABI and the small kernels.  Objects go to _build/
(not committed); the digest of the sources is compiled into the library (fi_build_info) so
that a loader can tell a stale binary from a current one.
"""
import hashlib
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libfi_gfx950.so")
HEADERS = ["gemm_fi.hpp", "gemm_fi_multi.hpp", "aux_kernels.hpp", "tile_cfg.hpp"]
SOURCES = ["fi_api.hip", "gemm_inst.hip"]
# (family, dtype, cfg): family 0 = one trial per work item, 1 = R trials per work item
INSTANCES = ([(1, dt, cfg) for dt in (0, 1) for cfg in (0, 1, 2, 3, 4, 5)] +
             [(0, dt, cfg) for dt in (0, 1) for cfg in (0, 1, 2)])


def source_files():
    return [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.join(ROOT, "include", "fi.h")]


def sources_digest():
    """SHA-256 over the kernel and ABI sources, in a fixed order."""
    h = hashlib.sha256()
    for f in sorted(source_files()):
        h.update(os.path.basename(f).encode() + b"\0")
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(d) > t for d in source_files())


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(ln for ln in r.stdout.splitlines()
                    if "packed-fp32-ops" not in ln)       # the host pass does not know the feature
    if r.returncode != 0:
        raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
    if verbose and out.strip():
        print(out)


def build(force=True, verbose=False, jobs=None):
    """Compile every HIP source for gfx950.  hipcc cross-compiles without a GPU."""
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    digest = sources_digest()
    common = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              "-Wno-unused-command-line-argument",
              "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    if os.environ.get("FI_SAVE_TEMPS"):
        common += ["-save-temps=obj"]
    # FI_SANITIZE_HOST=1: AddressSanitizer + UndefinedBehaviorSanitizer on the HOST side of the
    # ABI file only (argument checks, plan bookkeeping), into libfi_gfx950_san.so; load it through
    # FI_LIBRARY with clang's libclang_rt.asan-x86_64.so preloaded.  Device code is never sanitized.
    sanitize = bool(os.environ.get("FI_SANITIZE_HOST"))
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-g"] if sanitize else []
    lib = os.path.join(HERE, "libfi_gfx950_san.so") if sanitize else LIB
    cmds, objs = [], []
    api_o = os.path.join(OBJ, "fi_api.o")
    if sanitize:
        api_o = os.path.join(OBJ, "fi_api_san.o")
    cmds.append(common + san + ['-DFI_SOURCES_SHA256="%s"' % digest, "-c", os.path.join(CSRC, "fi_api.hip"), "-o", api_o])
    objs.append(api_o)
    for fam, dt, cfg in INSTANCES:
        o = os.path.join(OBJ, "gemm_f%d_d%d_c%d.o" % (fam, dt, cfg))
        cmds.append(common + ["-DFI_INST_FAMILY=%d" % fam, "-DFI_INST_DT=%d" % dt, "-DFI_INST_CFG=%d" % cfg,
                              "-c", os.path.join(CSRC, "gemm_inst.hip"), "-o", o])
        objs.append(o)
    jobs = jobs or int(os.environ.get("MAX_JOBS", 0)) or min(16, os.cpu_count() or 4)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        list(pool.map(lambda c: _run(c, verbose), cmds))
    # the sanitized build links clang's shared sanitizer runtime (to be preloaded by the loader)
    link_san = ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan", "-fno-gpu-sanitize"] if sanitize else []
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + link_san + objs + ["-o", lib], verbose)
    # A kernel whose host-side instantiation was dropped shows up only at load time, as an
    # undefined launch stub: refuse such a library here.
    nm = subprocess.run(["nm", "-D", "--undefined-only", lib], stdout=subprocess.PIPE, text=True).stdout
    missing = [ln.split()[-1] for ln in nm.splitlines() if "__device_stub__" in ln or " _ZN2fi" in ln]
    if missing:
        os.remove(lib)
        raise RuntimeError("libfi_gfx950.so would have undefined symbols: " + ", ".join(missing[:4]))
    return lib


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
