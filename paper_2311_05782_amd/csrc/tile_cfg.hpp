// Tile configurations of the two GEMM kernel families and the host-side launchers, one per
// (operand format, configuration).  Each launcher lives in its own translation unit
// (gemm_inst.hip compiled once per pair), so the library builds in parallel.
#pragma once

#include <hip/hip_runtime.h>

#include "fi.h"

namespace fi {

struct GemmArgs;

// One trial per work item: workgroup tile BM x BN computed by WM x WN waves.
struct TileCfg { int bm, bn, wm, wn; };
constexpr TileCfg kCfg[] = {
    {256, 256, 4, 2},   // 8 waves, each 64 x 128: large square-ish problems
    {128, 128, 2, 2},   // 4 waves, each 64 x 64
    {256, 64, 4, 1},    // 4 waves, each 64 x 64: narrow outputs (N <= 64)
};
constexpr int kNumCfg = sizeof(kCfg) / sizeof(kCfg[0]);

// R trials share one staged BM x BN tile (see gemm_fi_multi.hpp); `wgs` persistent workgroups
// per compute unit (two workgroups of four waves put one wave of each on every SIMD, so the
// barriers and the epilogue of one run under the MFMAs of the other).
struct MultiCfg { int r, bm, bn, wm, wn, wgs; };
constexpr MultiCfg kMulti[] = {
    {4, 128, 128, 4, 2, 1},   // each wave 32 x 64 for 4 trials
    {2, 128, 128, 4, 2, 1},   // each wave 32 x 64 for 2 trials
    {8, 128, 64, 4, 2, 1},    // each wave 32 x 32 for 8 trials
    {8, 64, 64, 2, 2, 2},     // each wave 32 x 32 for 8 trials, two workgroups per compute unit
    {1, 256, 256, 4, 2, 1},   // one trial per item, each wave 64 x 128
    {1, 128, 128, 2, 2, 2},   // one trial per item, each wave 64 x 64, two workgroups per compute unit
};
// The one-trial configurations also exist in a third instantiation for the next layer of a
// two-layer workload (every trial with its own A operand).
constexpr int kMultiOneTrial[2] = {4, 5};
constexpr int kNumMulti = sizeof(kMulti) / sizeof(kMulti[0]);

// mode: MODE_CAMPAIGN .. MODE_PROPAGATE of gemm_fi.hpp.
#define FI_DECLARE_SINGLE(DT, CFG) \
  hipError_t launch_single_d##DT##_c##CFG(int mode, const GemmArgs& a, int n_blocks, hipStream_t s);
// Both instantiations of the multi-trial kernel, one after the other (see gemm_fi_multi.hpp).
#define FI_DECLARE_MULTI(DT, MC) \
  hipError_t launch_multi_d##DT##_c##MC(const GemmArgs& a, int n_blocks, hipStream_t s);
FI_DECLARE_SINGLE(0, 0) FI_DECLARE_SINGLE(0, 1) FI_DECLARE_SINGLE(0, 2)
FI_DECLARE_SINGLE(1, 0) FI_DECLARE_SINGLE(1, 1) FI_DECLARE_SINGLE(1, 2)
#define FI_DECLARE_PROP(DT, MC) \
  hipError_t launch_prop_d##DT##_c##MC(const GemmArgs& a, int n_blocks, hipStream_t s);
FI_DECLARE_MULTI(0, 0) FI_DECLARE_MULTI(0, 1) FI_DECLARE_MULTI(0, 2) FI_DECLARE_MULTI(0, 3) FI_DECLARE_MULTI(0, 4) FI_DECLARE_MULTI(0, 5)
FI_DECLARE_MULTI(1, 0) FI_DECLARE_MULTI(1, 1) FI_DECLARE_MULTI(1, 2) FI_DECLARE_MULTI(1, 3) FI_DECLARE_MULTI(1, 4) FI_DECLARE_MULTI(1, 5)
FI_DECLARE_PROP(0, 4) FI_DECLARE_PROP(0, 5) FI_DECLARE_PROP(1, 4) FI_DECLARE_PROP(1, 5)
#undef FI_DECLARE_PROP
#undef FI_DECLARE_SINGLE
#undef FI_DECLARE_MULTI

}  // namespace fi
