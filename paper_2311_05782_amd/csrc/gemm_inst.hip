// One translation unit per (kernel family, operand format, tile configuration): compiled with
//   -DFI_INST_FAMILY=0|1   0: gemm_fi_kernel (one trial per work item), 1: gemm_fi_multi_kernel
//   -DFI_INST_DT=0|1       FI_FP16 / FI_BF16
//   -DFI_INST_CFG=0..2     index into kCfg / kMulti
// and exporting the launcher tile_cfg.hpp declares for that triple.
#include <hip/hip_runtime.h>

#include "tile_cfg.hpp"
#include "gemm_fi.hpp"
#include "gemm_fi_multi.hpp"

#define FI_CAT3(a, b, c, d) a##b##c##d
#define FI_NAME(prefix, dt, cfg) FI_CAT3(prefix, dt, _c, cfg)

namespace fi {

#if FI_INST_FAMILY == 0

template <int MODE>
static hipError_t launch_mode(const GemmArgs& a, int n_blocks, hipStream_t s) {
  constexpr TileCfg c = kCfg[FI_INST_CFG];
  hipLaunchKernelGGL((gemm_fi_kernel<FI_INST_DT, c.bm, c.bn, c.wm, c.wn, MODE>), dim3(n_blocks),
                     dim3(c.wm * c.wn * 64), 0, s, a);
  return hipGetLastError();
}

hipError_t FI_NAME(launch_single_d, FI_INST_DT, FI_INST_CFG)(int mode, const GemmArgs& a, int n_blocks,
                                                             hipStream_t s) {
  switch (mode) {
    case MODE_CAMPAIGN: return launch_mode<MODE_CAMPAIGN>(a, n_blocks, s);
    case MODE_GOLDEN: return launch_mode<MODE_GOLDEN>(a, n_blocks, s);
    case MODE_AFFECTED: return launch_mode<MODE_AFFECTED>(a, n_blocks, s);
    case MODE_PROPAGATE: return launch_mode<MODE_PROPAGATE>(a, n_blocks, s);
  }
  return hipErrorInvalidValue;
}

#else

// Two launches: the plain instantiation on the first part of the batch (no fault, accumulator
// flips, product-term faults), the operand-patching one on the second part (operand faults).
// Each finds its trial count on the device and exits at once if it is zero.
hipError_t FI_NAME(launch_multi_d, FI_INST_DT, FI_INST_CFG)(const GemmArgs& a, int n_blocks, hipStream_t s) {
  constexpr MultiCfg c = kMulti[FI_INST_CFG];
  hipLaunchKernelGGL((gemm_fi_multi_kernel<FI_INST_DT, c.r, c.bm, c.bn, c.wm, c.wn, VAR_PLAIN>), dim3(n_blocks),
                     dim3(c.wm * c.wn * 64), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((gemm_fi_multi_kernel<FI_INST_DT, c.r, c.bm, c.bn, c.wm, c.wn, VAR_OPERAND>), dim3(n_blocks),
                     dim3(c.wm * c.wn * 64), 0, s, a);
  return hipGetLastError();
}

#if FI_INST_CFG >= 4
// The next layer of a two-layer workload: one launch, every trial with its own A operand.
hipError_t FI_NAME(launch_prop_d, FI_INST_DT, FI_INST_CFG)(const GemmArgs& a, int n_blocks, hipStream_t s) {
  constexpr MultiCfg c = kMulti[FI_INST_CFG];
  static_assert(c.r == 1, "one trial per item");
  hipLaunchKernelGGL((gemm_fi_multi_kernel<FI_INST_DT, c.r, c.bm, c.bn, c.wm, c.wn, VAR_PROPAGATE>), dim3(n_blocks),
                     dim3(c.wm * c.wn * 64), 0, s, a);
  return hipGetLastError();
}
#endif

#endif

}  // namespace fi
