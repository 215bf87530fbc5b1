// C ABI of the fault-injection campaign engine (see include/fi.h): argument
// checking, plan construction and kernel launches.  No device work happens
// anywhere else.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <unordered_set>
#include <vector>

#include "aux_kernels.hpp"
#include "fi.h"
#include "gemm_fi.hpp"
#include "gemm_fi_multi.hpp"
#include "tile_cfg.hpp"

namespace {

thread_local char g_err[512] = "";

fi_status fail(fi_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define FI_HIP(call)                                                                        \
  do {                                                                                      \
    hipError_t e_ = (call);                                                                 \
    if (e_ != hipSuccess)                                                                   \
      return fail(e_ == hipErrorOutOfMemory ? FI_OOM : FI_DEVICE, "%s failed: %s", #call,   \
                  hipGetErrorString(e_));                                                   \
  } while (0)

constexpr int PAD = 512;                       // row/column vectors are zero padded to this multiple
size_t padded(uint32_t n) { return ((size_t)n + PAD - 1) / PAD * PAD; }
// elements of the fault-free result's allocation: whole tiles of rows plus one tile width
size_t golden_elems(const fi_plan_desc& d) { return padded((uint32_t)d.M) * (size_t)d.N + PAD; }

using fi::kCfg;
using fi::kMulti;
using fi::kNumCfg;
using fi::kNumMulti;
using fi::TileCfg;
using fi::MultiCfg;

}  // namespace

// Trial order and descriptors of one batch of the multi-trial kernel.  One set per stream a
// plan's batches have been enqueued on: batches on the same stream follow each other, batches
// on different streams may be in flight together and must not share this state.
struct BatchScratch {
  hipStream_t stream = nullptr;
  uint32_t* perm = nullptr;   // [cap] trial order + 2 counters behind it
  uint32_t* desc = nullptr;   // [(cap + 16) * kMultiDescWords]
  uint32_t cap = 0;
};

struct fi_plan {
  fi_plan_desc d = {};
  const uint16_t* A = nullptr;
  const uint16_t* B = nullptr;       // effective [N][ldb] K-contiguous matrix
  uint32_t ldb = 0;
  uint16_t* Bt = nullptr;            // plan-owned transposed copy (b_layout 1) or NULL
  // K not a multiple of 64: copies of A and B ([M][K + kshift], [N][K + kshift]) with kshift zeros
  // in front of every row, for the kernels that want whole 64-wide k-tiles; else NULL and 0
  uint16_t* Apad = nullptr;
  uint16_t* Bpad = nullptr;
  uint32_t kshift = 0;
  float* c_star = nullptr;           // [M][N]
  float* s_abs = nullptr;            // [M][N]
  float* kra = nullptr;              // [pad(M)]
  float* cb = nullptr;               // [pad(N)]
  float* scratch = nullptr;          // 4 floats + 4 words: maxima, "operand not finite", clean flags
  float t_global = 0.0f;
  uint32_t n_clean_flagged = 0;      // elements of C* the plan's own detector flags
  int cfg = 0;                       // index into kCfg
  int cfg_affected = 0;              // index into kCfg for the affected-tiles-only campaign
  int mcfg = -1;                     // index into kMulti, or -1: every trial through the single-trial kernel
  int prop_cfg = -1;                 // index into kMulti for the next-layer batch, or -1: single-trial kernel
  int group = 32;                    // trials sharing a tile back to back
  int device = 0;
  std::vector<BatchScratch> batch;   // per stream, see BatchScratch
  int n_cus = 8;                     // compute units of the device: grid of the persistent kernel
  int product_check = FI_PCHECK_NONE;
  unsigned long long* clocks = nullptr;   // caller's [12] counter sink, or NULL (fi_plan_set_clock_sink)
};

namespace {

using fi::GemmArgs;

// Each (format, configuration) pair has its launcher in a translation unit of its own.
hipError_t launch_gemm(int mode, int dtype, int cfg, const GemmArgs& a, int n_blocks, hipStream_t s) {
#define FI_CASE(DT, CFG) \
  if (dtype == DT && cfg == CFG) return fi::launch_single_d##DT##_c##CFG(mode, a, n_blocks, s)
  FI_CASE(0, 0); FI_CASE(0, 1); FI_CASE(0, 2);
  FI_CASE(1, 0); FI_CASE(1, 1); FI_CASE(1, 2);
#undef FI_CASE
  return hipErrorInvalidValue;
}

hipError_t launch_multi(int dtype, int mcfg, const GemmArgs& a, int n_blocks, hipStream_t s) {
#define FI_CASE(DT, MC) \
  if (dtype == DT && mcfg == MC) return fi::launch_multi_d##DT##_c##MC(a, n_blocks, s)
  FI_CASE(0, 0); FI_CASE(0, 1); FI_CASE(0, 2); FI_CASE(0, 3); FI_CASE(0, 4); FI_CASE(0, 5);
  FI_CASE(1, 0); FI_CASE(1, 1); FI_CASE(1, 2); FI_CASE(1, 3); FI_CASE(1, 4); FI_CASE(1, 5);
#undef FI_CASE
  return hipErrorInvalidValue;
}

hipError_t launch_prop(int dtype, int mcfg, const GemmArgs& a, int n_blocks, hipStream_t s) {
#define FI_CASE(DT, MC) \
  if (dtype == DT && mcfg == MC) return fi::launch_prop_d##DT##_c##MC(a, n_blocks, s)
  FI_CASE(0, 4); FI_CASE(0, 5); FI_CASE(1, 4); FI_CASE(1, 5);
#undef FI_CASE
  return hipErrorInvalidValue;
}

// Eight trials per tile carry the least operand traffic per flop.  On the largest problems one eight-wave workgroup per CU on a
// 128 x 64 tile measured fastest (less traffic into LDS per flop); below that two four-wave
// workgroups on 64 x 64 tiles win, because the barriers and the per-item epilogue of one run
// under the MFMAs of the other (+2 .. 16 % on 1024^3, 512 x 3072 x 768 and 3136 x 64 x 576).
int pick_multi(const fi_plan_desc& d) {
  const double work = (double)d.M * (double)d.N * (double)d.K;
  return work >= 34359738368.0 /* 2^35 */ ? 2 : 3;
}

int pick_cfg(const fi_plan_desc& d) {
  if (d.N <= 64) return 2;
  if (d.M >= 512 && d.N >= 512) return 0;
  return 1;
}

GemmArgs base_args(const fi_plan* p, int cfg = -1) {
  GemmArgs a;
  memset(&a, 0, sizeof(a));
  const TileCfg c = kCfg[cfg >= 0 ? cfg : p->cfg];
  a.A = p->A; a.B = p->B; a.lda = (uint32_t)p->d.lda; a.ldb = p->ldb;
  a.M = (int)p->d.M; a.N = (int)p->d.N; a.K = (int)p->d.K; a.kb = (int)p->d.k_block;
  a.tiles_m = (a.M + c.bm - 1) / c.bm;
  a.tiles_n = (a.N + c.bn - 1) / c.bn;
  a.kra = p->kra; a.cb = p->cb; a.gamma = p->d.gamma;
  a.bound_global = p->d.bound_mode != FI_BOUND_ROWCOL;
  a.t_global = p->t_global;
  a.c_star = p->c_star; a.s_abs = p->s_abs;
  const size_t gold_bytes = golden_elems(p->d) * sizeof(float);
  a.c_star_bytes = gold_bytes < (1ull << 32) ? (uint32_t)gold_bytes : 0u;
  a.clocks = p->clocks;
  return a;
}

// C* with the same kernel family the campaign uses (so that a fault-free tile of a trial is
// bit-identical to it), and S = |A| x |B| on sign-cleared copies of the operands.
fi_status compute_golden(fi_plan* p, hipStream_t s, const uint16_t* absA, const uint16_t* absB) {
  GemmArgs a = base_args(p);
  a.n_trials = 1; a.group = 1;
  a.c_out = p->c_star;
  FI_HIP(launch_gemm(fi::MODE_GOLDEN, (int)p->d.dtype, p->cfg, a, a.tiles_m * a.tiles_n, s));
  a.A = absA; a.B = absB;
  a.lda = a.ldb = (uint32_t)p->d.K;     // the copies are packed
  a.c_out = p->s_abs;
  FI_HIP(launch_gemm(fi::MODE_GOLDEN, (int)p->d.dtype, p->cfg, a, a.tiles_m * a.tiles_n, s));
  return FI_OK;
}

fi_status check_device() {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(FI_STATE, "no HIP device: %s", hipGetErrorString(e));
  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, dev);
  if (e != hipSuccess) return fail(FI_STATE, "hipGetDeviceProperties: %s", hipGetErrorString(e));
  if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
    return fail(FI_STATE, "device %d is %s; this library is built for gfx950 only", dev, prop.gcnArchName);
  return FI_OK;
}

fi_status check_desc(const fi_plan_desc* d, float* gamma_out) {
  if (!d) return fail(FI_INVALID_ARG, "desc is NULL");
  if (d->M == 0 || d->N == 0 || d->K == 0) return fail(FI_INVALID_ARG, "M, N, K must be non-zero");
  if (d->k_block == 0 || d->k_block % 16 != 0)
    return fail(FI_INVALID_ARG, "k_block must be a non-zero multiple of 16 (got %u)", d->k_block);
  if (d->K % d->k_block != 0)
    return fail(FI_INVALID_ARG, "K (%u) must be a multiple of k_block (%u)", d->K, d->k_block);
  if (d->dtype != FI_FP16 && d->dtype != FI_BF16)
    return fail(FI_UNSUPPORTED, "dtype %u: only FP16 (0) and BF16 (1) operands", d->dtype);
  if (d->b_layout > 1) return fail(FI_INVALID_ARG, "b_layout must be 0 or 1");
  if (d->bound_mode > FI_BOUND_EXPONENT) return fail(FI_INVALID_ARG, "bound_mode must be 0, 1 or 2");
  // Default slack: 1 + 2^-11 for K <= 4096, growing in proportion beyond (a K-term FP32
  // accumulation inflates a sum by at most (1 + 2^-24)^(K-1); twice that, in units of 4096 terms).
  float g = d->gamma == 0.0f ? 1.0f + (float)((d->K + 4095u) / 4096u) / 2048.0f : d->gamma;
  if (!(g >= 1.0f) || !(g <= 3.0e38f)) return fail(FI_INVALID_ARG, "gamma must be finite and >= 1");
  if (d->K > 65536u) return fail(FI_UNSUPPORTED, "K > 65536");
  if (d->M > (1u << 24) || d->N > (1u << 24)) return fail(FI_UNSUPPORTED, "M or N > 2^24");
  if (gamma_out) *gamma_out = g;
  return FI_OK;
}

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

// Live plans.  A handle is looked up here before it is dereferenced, so a destroyed (or
// never created) plan is an error and not a read of freed memory.
std::mutex g_live_mu;
std::unordered_set<const fi_plan*> g_live;

fi_status check_plan(const fi_plan* p) {
  if (!p) return fail(FI_INVALID_ARG, "plan is NULL");
  std::lock_guard<std::mutex> lock(g_live_mu);
  if (g_live.find(p) == g_live.end()) return fail(FI_STATE, "plan is not live (destroyed or never created)");
  return FI_OK;
}

void free_plan_buffers(fi_plan* p) {
  if (p->Bt) (void)hipFree(p->Bt);
  if (p->Apad) (void)hipFree(p->Apad);
  if (p->Bpad) (void)hipFree(p->Bpad);
  if (p->c_star) (void)hipFree(p->c_star);
  if (p->s_abs) (void)hipFree(p->s_abs);
  if (p->kra) (void)hipFree(p->kra);
  if (p->cb) (void)hipFree(p->cb);
  if (p->scratch) (void)hipFree(p->scratch);
  for (BatchScratch& b : p->batch) {
    if (b.perm) (void)hipFree(b.perm);
    if (b.desc) (void)hipFree(b.desc);
  }
  p->batch.clear();
}

// The batch scratch of `stream`, holding at least n trials.  Allocates on the first batch of a
// stream and when a batch is larger than any before on it (the replaced buffers are freed,
// which waits for device work that may still read them).
fi_status batch_scratch(fi_plan* p, hipStream_t stream, uint32_t n, BatchScratch** out) {
  BatchScratch* b = nullptr;
  for (BatchScratch& x : p->batch)
    if (x.stream == stream) b = &x;
  if (!b) {
    if (p->batch.size() >= 64) return fail(FI_STATE, "a plan serves at most 64 distinct streams");
    p->batch.emplace_back();
    b = &p->batch.back();
    b->stream = stream;
  }
  if (b->cap < n) {
    if (b->perm) (void)hipFree(b->perm);
    if (b->desc) (void)hipFree(b->desc);
    b->perm = nullptr; b->desc = nullptr; b->cap = 0;
    FI_HIP(hipMalloc(&b->perm, ((size_t)n + 2) * sizeof(uint32_t)));
    FI_HIP(hipMalloc(&b->desc, ((size_t)n + 16) * fi::kMultiDescWords * sizeof(uint32_t)));
    b->cap = n;
  }
  *out = b;
  return FI_OK;
}


fi_status build_plan(fi_plan* p, const void* d_A, const void* d_B, hipStream_t s) {
  const fi_plan_desc& d = p->d;
  const size_t mn = (size_t)d.M * d.N;
  // C* is padded to whole 256-row tiles plus one tile width (zeros): the next layer's kernel
  // reads the tile-shaped neighbourhood of its outputs without clamping rows or columns.
  const size_t mn_pad = golden_elems(d);
  FI_HIP(hipMalloc(&p->c_star, mn_pad * sizeof(float)));
  FI_HIP(hipMemsetAsync(p->c_star + mn, 0, (mn_pad - mn) * sizeof(float), s));
  FI_HIP(hipMalloc(&p->s_abs, mn * sizeof(float)));
  FI_HIP(hipMalloc(&p->kra, padded(d.M) * sizeof(float)));
  FI_HIP(hipMalloc(&p->cb, padded(d.N) * sizeof(float)));
  FI_HIP(hipMalloc(&p->scratch, 8 * sizeof(float)));
  p->A = static_cast<const uint16_t*>(d_A);
  if (d.b_layout == 0) {
    p->B = static_cast<const uint16_t*>(d_B);
    p->ldb = (uint32_t)d.ldb;
  } else {
    FI_HIP(hipMalloc(&p->Bt, (size_t)d.N * d.K * sizeof(uint16_t)));
    dim3 grid((d.N + 31) / 32, (d.K + 31) / 32);
    hipLaunchKernelGGL(fi::transpose16_kernel, grid, dim3(256), 0, s,
                       static_cast<const uint16_t*>(d_B), (uint32_t)d.ldb, p->Bt, d.K, (int)d.K, (int)d.N);
    FI_HIP(hipGetLastError());
    p->B = p->Bt;
    p->ldb = d.K;
  }
  if (d.K % 64 != 0) {
    p->kshift = 64 - d.K % 64;
    const uint32_t kp = d.K + p->kshift;
    FI_HIP(hipMalloc(&p->Apad, (size_t)d.M * kp * sizeof(uint16_t)));
    FI_HIP(hipMalloc(&p->Bpad, (size_t)d.N * kp * sizeof(uint16_t)));
    hipLaunchKernelGGL(fi::pad_front16_kernel, dim3(1024), dim3(256), 0, s, p->A, (uint32_t)d.lda, p->Apad, d.M, d.K,
                       p->kshift);
    hipLaunchKernelGGL(fi::pad_front16_kernel, dim3(1024), dim3(256), 0, s, p->B, p->ldb, p->Bpad, d.N, d.K,
                       p->kshift);
    FI_HIP(hipGetLastError());
  }
  // statistics
  hipLaunchKernelGGL(fi::fill_u32_kernel, dim3(64), dim3(256), 0, s,
                     reinterpret_cast<uint32_t*>(p->kra), padded(d.M), 0u);
  hipLaunchKernelGGL(fi::fill_u32_kernel, dim3(64), dim3(256), 0, s,
                     reinterpret_cast<uint32_t*>(p->cb), padded(d.N), 0u);
  hipLaunchKernelGGL(fi::fill_u32_kernel, dim3(1), dim3(64), 0, s,
                     reinterpret_cast<uint32_t*>(p->scratch), (size_t)8, 0u);
  uint32_t* bad = reinterpret_cast<uint32_t*>(p->scratch + 4);
  if (d.dtype == FI_FP16) {
    hipLaunchKernelGGL(fi::row_absmax_kernel<FI_FP16>, dim3((d.M + 3) / 4), dim3(256), 0, s, p->A, (int)d.M,
                       (int)d.K, (uint32_t)d.lda, (float)d.K, p->kra, bad);
    hipLaunchKernelGGL(fi::row_absmax_kernel<FI_FP16>, dim3((d.N + 3) / 4), dim3(256), 0, s, p->B, (int)d.N,
                       (int)d.K, p->ldb, 1.0f, p->cb, bad);
  } else {
    hipLaunchKernelGGL(fi::row_absmax_kernel<FI_BF16>, dim3((d.M + 3) / 4), dim3(256), 0, s, p->A, (int)d.M,
                       (int)d.K, (uint32_t)d.lda, (float)d.K, p->kra, bad);
    hipLaunchKernelGGL(fi::row_absmax_kernel<FI_BF16>, dim3((d.N + 3) / 4), dim3(256), 0, s, p->B, (int)d.N,
                       (int)d.K, p->ldb, 1.0f, p->cb, bad);
  }
  FI_HIP(hipGetLastError());
  hipLaunchKernelGGL(fi::max_reduce_kernel, dim3(1), dim3(1024), 0, s, p->kra, (int)d.M, p->scratch + 0);
  hipLaunchKernelGGL(fi::max_reduce_kernel, dim3(1), dim3(1024), 0, s, p->cb, (int)d.N, p->scratch + 1);
  FI_HIP(hipGetLastError());
  // sign-cleared operand copies for the magnitude-sum GEMM; freed once the stream has drained
  uint16_t *absA = nullptr, *absB = nullptr;
  const size_t nA = (size_t)d.M * d.K, nB = (size_t)d.N * d.K;
  hipError_t e1 = hipMalloc(&absA, nA * sizeof(uint16_t));
  hipError_t e2 = hipMalloc(&absB, nB * sizeof(uint16_t));
  fi_status st = FI_OK;
  if (e1 != hipSuccess || e2 != hipSuccess) {
    st = fail(FI_OOM, "device allocation for the magnitude operands failed");
  } else {
    hipLaunchKernelGGL(fi::abs16_kernel, dim3(2048), dim3(256), 0, s, p->A, (uint32_t)d.lda, absA, (int)d.M, (int)d.K);
    hipLaunchKernelGGL(fi::abs16_kernel, dim3(2048), dim3(256), 0, s, p->B, p->ldb, absB, (int)d.N, (int)d.K);
    st = compute_golden(p, s, absA, absB);
  }
  hipError_t es = hipStreamSynchronize(s);
  if (absA) (void)hipFree(absA);
  if (absB) (void)hipFree(absB);
  if (st != FI_OK) return st;
  if (es != hipSuccess) return fail(FI_DEVICE, "plan kernels failed: %s", hipGetErrorString(es));
  float host[8];
  FI_HIP(hipMemcpyAsync(host, p->scratch, sizeof(host), hipMemcpyDeviceToHost, s));
  FI_HIP(hipStreamSynchronize(s));
  uint32_t badw;
  memcpy(&badw, &host[4], 4);
  if (badw) return fail(FI_INVALID_ARG, "A or B holds an Inf or NaN: the magnitude bound is undefined");
  // T = fl32(fl32(fl32(K*ra_max) * cb_max) * gamma), one rounding per product
  volatile float t = host[0] * host[1];
  t = t * d.gamma;
  p->t_global = t;
  // Exponent field >= 144 <=> NOT (|c| <= largest binary32 below 2^17)
  if (d.bound_mode == FI_BOUND_EXPONENT) p->t_global = 131071.9921875f;
  // How many elements of the fault-free result the plan's own detector flags (none under the
  // operand-derived bounds with gamma at or above the default; possible under the exponent-only
  // bound or a caller's smaller gamma).  The affected-tiles-only campaign relies on it being 0.
  {
    uint32_t* n_clean = reinterpret_cast<uint32_t*>(p->scratch + 5);
    const bool vec = d.N % 4 == 0;
    size_t gx = vec ? (size_t)d.M : (mn + 255) / 256;
    if (gx > 2048) gx = 2048;
    if (vec)
      hipLaunchKernelGGL(fi::detect_correct_kernel<4>, dim3((unsigned)gx, 1), dim3(256), 0, s, p->c_star, (int)d.M,
                         (int)d.N, p->kra, p->cb, d.gamma, (int)(d.bound_mode != FI_BOUND_ROWCOL), p->t_global,
                         (int)FI_CORRECT_NONE, (const float*)nullptr, (uint8_t*)nullptr, n_clean);
    else
      hipLaunchKernelGGL(fi::detect_correct_kernel<1>, dim3((unsigned)gx, 1), dim3(256), 0, s, p->c_star, (int)d.M,
                         (int)d.N, p->kra, p->cb, d.gamma, (int)(d.bound_mode != FI_BOUND_ROWCOL), p->t_global,
                         (int)FI_CORRECT_NONE, (const float*)nullptr, (uint8_t*)nullptr, n_clean);
    FI_HIP(hipGetLastError());
    FI_HIP(hipMemcpyAsync(&p->n_clean_flagged, n_clean, sizeof(uint32_t), hipMemcpyDeviceToHost, s));
    FI_HIP(hipStreamSynchronize(s));
  }
  return FI_OK;
}

// Where one batch of the multi-trial kernel keeps its trial order, the two part counts and the
// per-trial descriptors; all of it is rewritten by the partition kernel of every batch.
struct TrialScratch {
  uint32_t* perm = nullptr;     // [n_trials]
  uint32_t* counts = nullptr;   // [2]
  uint32_t* desc = nullptr;     // [(n_trials + 16) * kMultiDescWords]
};

fi_status check_batch_args(const fi_plan* plan, const fi_fault* d_faults, uint32_t n_trials, uint32_t policy,
                           const fi_trial_result* d_results) {
  fi_status st = check_plan(plan);
  if (st != FI_OK) return st;
  if (!d_faults || !d_results) return fail(FI_INVALID_ARG, "d_faults and d_results must be non-NULL");
  if (n_trials == 0) return fail(FI_INVALID_ARG, "n_trials is 0");
  if (policy > FI_CORRECT_RECOMPUTE) return fail(FI_INVALID_ARG, "unknown correction policy %u", policy);
  return FI_OK;
}

// One campaign batch: record fill, then either the partition kernel and the two launches of
// the multi-trial kernel (scratch in `ts`), or one launch of the one-trial kernel.
fi_status inject_batch(fi_plan* plan, const fi_fault* d_faults, uint32_t n_trials, uint32_t policy,
                       fi_trial_result* d_results, float* d_c_out, hipStream_t s, const TrialScratch& ts,
                       uint16_t* d_h_out = nullptr) {
  GemmArgs a = base_args(plan);
  const uint64_t blocks = (uint64_t)a.tiles_m * a.tiles_n * n_trials;
  if (blocks >= (1ull << 31)) return fail(FI_UNSUPPORTED, "tiles x trials exceeds 2^31 workgroups; split the batch");
  const MultiCfg mc = kMulti[plan->mcfg >= 0 ? plan->mcfg : 0];
  GemmArgs m = a;
  uint64_t mblocks = 0;
  if (plan->mcfg >= 0) {
    m.tiles_m = (a.M + mc.bm - 1) / mc.bm;
    m.tiles_n = (a.N + mc.bn - 1) / mc.bn;
    if (plan->kshift) {
      // whole k-tiles: the front-padded copies (bit-identical results, see pad_front16_kernel)
      m.A = plan->Apad; m.B = plan->Bpad;
      m.K = a.K + (int)plan->kshift;
      m.lda = m.ldb = (uint32_t)m.K;
    }
    // Persistent workgroups, as many per CU as the configuration's register budget admits, each
    // walking the work list with the grid as stride; a multiple of 8 keeps a workgroup's items
    // on one XCD.
    const uint64_t groups = ((uint64_t)n_trials + mc.r - 1) / mc.r;
    const uint64_t items = (uint64_t)m.tiles_m * m.tiles_n * groups;
    if (items >= (1ull << 31)) return fail(FI_UNSUPPORTED, "tiles x trials exceeds 2^31 work items; split the batch");
    const uint64_t cus = (uint64_t)(plan->n_cus / 8 * 8) * (uint64_t)mc.wgs;
    mblocks = items < cus ? items : cus;
  }
  const size_t words = (size_t)n_trials * (sizeof(fi_trial_result) / 4);
  hipLaunchKernelGGL(fi::fill_u32_kernel, dim3((unsigned)((words + 255) / 256 > 1024 ? 1024 : (words + 255) / 256)),
                     dim3(256), 0, s, reinterpret_cast<uint32_t*>(d_results), words, 0u);
  FI_HIP(hipGetLastError());
  for (GemmArgs* g : {&a, &m}) {
    g->n_trials = (int)n_trials;
    g->group = plan->group;
    g->faults = d_faults;
    g->results = d_results;
    g->c_out = d_c_out;
    g->h_out = d_h_out;
    g->policy = (int)policy;
    g->product_check = plan->product_check;
  }
  if (plan->mcfg < 0) {
    FI_HIP(launch_gemm(fi::MODE_CAMPAIGN, (int)plan->d.dtype, plan->cfg, a, (int)blocks, s));
    return FI_OK;
  }
  // R trials at a time share staged operands.  The batch is split on the device into the trials
  // whose fault leaves the operands alone and the operand-fault trials; each part has its own
  // instantiation of the kernel.
  if (plan->d.dtype == FI_BF16)
    hipLaunchKernelGGL(fi::partition_trials_kernel<FI_BF16>, dim3(1), dim3(1024), 0, s, d_faults, n_trials,
                       plan->d.M, plan->d.N, plan->d.K, plan->d.k_block, a.A, a.B, a.lda, a.ldb, plan->product_check,
                       (uint32_t)mc.bm, (uint32_t)mc.bn, plan->kshift, ts.perm, ts.counts, ts.desc, d_results);
  else
    hipLaunchKernelGGL(fi::partition_trials_kernel<FI_FP16>, dim3(1), dim3(1024), 0, s, d_faults, n_trials,
                       plan->d.M, plan->d.N, plan->d.K, plan->d.k_block, a.A, a.B, a.lda, a.ldb, plan->product_check,
                       (uint32_t)mc.bm, (uint32_t)mc.bn, plan->kshift, ts.perm, ts.counts, ts.desc, d_results);
  FI_HIP(hipGetLastError());
  m.perm = ts.perm;
  m.part_counts = ts.counts;
  m.desc = ts.desc;
  FI_HIP(launch_multi((int)plan->d.dtype, plan->mcfg, m, (int)mblocks, s));
  return FI_OK;
}

// ---- scratch of fi_gemm_inject_batch_noalloc: one array per GPU, held until the process ends.
constexpr uint32_t kNoAllocMaxTrials = 16384;
constexpr size_t kNoAllocPermWords = (((size_t)kNoAllocMaxTrials + 2 + 63) / 64) * 64;   // desc starts 256-byte aligned
constexpr size_t kNoAllocWords = kNoAllocPermWords + ((size_t)kNoAllocMaxTrials + 16) * fi::kMultiDescWords;
static __device__ __align__(256) uint32_t scratch[kNoAllocWords];

// The array's address on each device (the name above is only a host-side handle for the
// symbol: every use from host code goes through the looked-up pointer).
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
uint32_t* g_scratch_ptr[kMaxDevices] = {};

// Looks the address up once per device, with that device current.  Called from
// fi_plan_create (set-up), so that the entry point itself only reads the table.
fi_status resolve_static_scratch(int device) {
  if (device < 0 || device >= kMaxDevices) return fail(FI_UNSUPPORTED, "device index %d beyond %d", device, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (g_scratch_ptr[device]) return FI_OK;
  uint32_t* ptr = nullptr;
  FI_HIP(hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)));
  if (!ptr) return fail(FI_DEVICE, "hipGetSymbolAddress returned a NULL address for the static scratch");
  g_scratch_ptr[device] = ptr;
  return FI_OK;
}

uint64_t splitmix64(uint64_t* state) {
  uint64_t z = (*state += 0x9E3779B97F4A7C15ull);
  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27; z *= 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z;
}

inline uint32_t scale_to(uint32_t n, uint64_t u) { return (uint32_t)(((u >> 32) * (uint64_t)n) >> 32); }

}  // namespace

extern "C" {

const char* fi_last_error(void) { return g_err; }

#ifndef FI_SOURCES_SHA256
#define FI_SOURCES_SHA256 "unknown"
#endif
const char* fi_build_info(void) { return FI_SOURCES_SHA256; }

fi_status fi_plan_create(const fi_plan_desc* desc, const void* d_A, const void* d_B, void* stream,
                         fi_plan** out) {
  float gamma = 0.f;
  fi_status st = check_desc(desc, &gamma);
  if (st != FI_OK) return st;
  if (!d_A || !d_B || !out) return fail(FI_INVALID_ARG, "d_A, d_B and out must be non-NULL");
  const fi_plan_desc& d = *desc;
  const int64_t min_ldb = d.b_layout == 0 ? (int64_t)d.K : (int64_t)d.N;
  if (d.lda < (int64_t)d.K || d.ldb < min_ldb)
    return fail(FI_INVALID_ARG, "leading dimension smaller than the row length");
  if ((reinterpret_cast<uintptr_t>(d_A) & 15u) || (d.lda & 7))
    return fail(FI_UNSUPPORTED, "A must be 16-byte aligned with lda a multiple of 8");
  if (d.b_layout == 0 && ((reinterpret_cast<uintptr_t>(d_B) & 15u) || (d.ldb & 7)))
    return fail(FI_UNSUPPORTED, "B must be 16-byte aligned with ldb a multiple of 8");
  if ((uint64_t)d.M * (uint64_t)d.lda >= (1ull << 31) ||
      (uint64_t)d.N * (uint64_t)(d.b_layout == 0 ? d.ldb : (int64_t)d.K) >= (1ull << 31))
    return fail(FI_UNSUPPORTED, "an operand spans 2^31 elements or more");
  if ((uint64_t)d.M * (uint64_t)d.N >= (1ull << 40)) return fail(FI_UNSUPPORTED, "M*N too large");
  st = check_device();
  if (st != FI_OK) return st;

  fi_plan* p = new (std::nothrow) fi_plan();
  if (!p) return fail(FI_OOM, "host allocation failed");
  p->d = d;
  p->d.gamma = gamma;
  p->cfg = pick_cfg(d);
  p->cfg_affected = d.N <= 64 ? 2 : 1;   // small tiles: only the reached part is of interest
  p->mcfg = pick_multi(d);
  // Next-layer launches: on problems below 2^35 multiply-adds the 128 x 128 shape with two
  // workgroups per CU measured faster (one's epilogue runs under the other's MFMAs: 0.75 against
  // 0.81 ms on 512 x 768 x 3072, 256 trials), above it the 256 x 256 shape (less LDS traffic per flop).
  p->prop_cfg = (double)d.M * (double)d.N * (double)d.K >= 34359738368.0 ? fi::kMultiOneTrial[0]
                                                                         : fi::kMultiOneTrial[1];
  p->group = 32;
  (void)hipGetDevice(&p->device);
  if (hipDeviceGetAttribute(&p->n_cus, hipDeviceAttributeMultiprocessorCount, p->device) != hipSuccess ||
      p->n_cus < 8)
    p->n_cus = 8;
  st = build_plan(p, d_A, d_B, as_stream(stream));
  if (st != FI_OK) {
    (void)hipStreamSynchronize(as_stream(stream));
    free_plan_buffers(p);
    delete p;
    return st;
  }
  st = resolve_static_scratch(p->device);
  if (st != FI_OK) {
    free_plan_buffers(p);
    delete p;
    return st;
  }
  {
    std::lock_guard<std::mutex> lock(g_live_mu);
    g_live.insert(p);
  }
  *out = p;
  return FI_OK;
}

fi_status fi_plan_destroy(fi_plan* plan) {
  fi_status st = check_plan(plan);
  if (st != FI_OK) return st;
  {
    std::lock_guard<std::mutex> lock(g_live_mu);
    g_live.erase(plan);
  }
  (void)hipDeviceSynchronize();   // work that still reads the plan's buffers
  free_plan_buffers(plan);
  delete plan;
  return FI_OK;
}

fi_status fi_plan_buffer(const fi_plan* plan, uint32_t which, const void** d_ptr) {
  fi_status st = check_plan(plan);
  if (st != FI_OK) return st;
  if (!d_ptr) return fail(FI_INVALID_ARG, "d_ptr is NULL");
  switch (which) {
    case 0: *d_ptr = plan->c_star; break;
    case 1: *d_ptr = plan->s_abs; break;
    case 2: *d_ptr = plan->kra; break;
    case 3: *d_ptr = plan->cb; break;
    default: return fail(FI_INVALID_ARG, "which must be 0..3");
  }
  return FI_OK;
}

fi_status fi_plan_tune(fi_plan* plan, int32_t tile_config, int32_t trial_group, void* stream) {
  fi_status st = check_plan(plan);
  if (st != FI_OK) return st;
  if (tile_config >= kNumCfg + kNumMulti)
    return fail(FI_INVALID_ARG, "tile_config must be < %d", kNumCfg + kNumMulti);
  if (trial_group == 0 || trial_group > 4096) return fail(FI_INVALID_ARG, "trial_group must be in 1..4096");
  if (trial_group > 0) plan->group = trial_group;
  // C* does not depend on the tile shape: every shape feeds each output element the same
  // sequence of 16-wide MFMA steps in ascending k.
  if (tile_config >= kNumCfg) {
    plan->mcfg = tile_config - kNumCfg;
    if (kMulti[plan->mcfg].r == 1) plan->prop_cfg = plan->mcfg;
  } else if (tile_config >= 0) {
    plan->cfg = tile_config; plan->cfg_affected = tile_config;
    // One trial per work item.  The 256x256 and 128x128 shapes run as persistent workgroups (the
    // multi-trial kernel's item loop with one trial per item).
    const bool persistent = tile_config < 2;
    plan->mcfg = persistent ? fi::kMultiOneTrial[tile_config] : -1;
    plan->prop_cfg = persistent ? fi::kMultiOneTrial[tile_config] : -1;
  }
  (void)stream;
  return FI_OK;
}

fi_status fi_plan_reserve(fi_plan* plan, uint32_t max_trials, void* stream) {
  fi_status st = check_plan(plan);
  if (st != FI_OK) return st;
  if (max_trials == 0) return fail(FI_INVALID_ARG, "max_trials is 0");
  BatchScratch* bs = nullptr;
  return batch_scratch(plan, as_stream(stream), max_trials, &bs);
}

fi_status fi_plan_set_clock_sink(fi_plan* plan, uint64_t* d_clocks) {
  fi_status st = check_plan(plan);
  if (st != FI_OK) return st;
  if (reinterpret_cast<uintptr_t>(d_clocks) & 7u) return fail(FI_INVALID_ARG, "d_clocks must be 8-byte aligned");
  plan->clocks = reinterpret_cast<unsigned long long*>(d_clocks);
  return FI_OK;
}

fi_status fi_probe_mfma_loop(uint32_t dtype, uint32_t random_data, uint32_t iters, uint32_t n_workgroups,
                             float* d_sink, uint64_t* d_clocks, void* stream) {
  if (dtype != FI_FP16 && dtype != FI_BF16) return fail(FI_UNSUPPORTED, "dtype %u: only FP16 (0) and BF16 (1)", dtype);
  if (!d_sink) return fail(FI_INVALID_ARG, "d_sink is NULL");
  if (iters == 0 || n_workgroups == 0 || n_workgroups > 65536u || iters > (1u << 24))
    return fail(FI_INVALID_ARG, "iters must be in 1..2^24 and n_workgroups in 1..65536");
  fi_status st = check_device();
  if (st != FI_OK) return st;
  unsigned long long* clk = reinterpret_cast<unsigned long long*>(d_clocks);
  if (dtype == FI_BF16)
    hipLaunchKernelGGL(fi::mfma_loop_probe_kernel<FI_BF16>, dim3(n_workgroups), dim3(512), 0, as_stream(stream),
                       (int)random_data, (int)iters, d_sink, clk);
  else
    hipLaunchKernelGGL(fi::mfma_loop_probe_kernel<FI_FP16>, dim3(n_workgroups), dim3(512), 0, as_stream(stream),
                       (int)random_data, (int)iters, d_sink, clk);
  FI_HIP(hipGetLastError());
  return FI_OK;
}

fi_status fi_plan_set_product_check(fi_plan* plan, uint32_t mode) {
  fi_status st = check_plan(plan);
  if (st != FI_OK) return st;
  if (mode > FI_PCHECK_RANGE_FLIP) return fail(FI_INVALID_ARG, "unknown product check %u", mode);
  plan->product_check = (int)mode;
  return FI_OK;
}

fi_status fi_plan_describe(const fi_plan* plan, char* h_buf, uint64_t n) {
  fi_status st = check_plan(plan);
  if (st != FI_OK) return st;
  if (!h_buf || n == 0) return fail(FI_INVALID_ARG, "h_buf is NULL or n is 0");
  const TileCfg c = kCfg[plan->cfg];
  const char* dt = plan->d.dtype == FI_BF16 ? "bf16" : "fp16";
  if (plan->mcfg >= 0) {
    const MultiCfg m = kMulti[plan->mcfg];
    if (m.r == 1)
      snprintf(h_buf, n, "gemm_fi_multi_kernel<%s, one trial per item, %dx%d, %d threads, persistent x%d per CU>", dt,
               m.bm, m.bn, m.wm * m.wn * 64, m.wgs);
    else
    snprintf(h_buf, n, "gemm_fi_multi_kernel<%s, R=%d, %dx%d, %d threads, persistent x%d per CU> (a second, "
             "operand-patching instantiation for operand faults)", dt, m.r, m.bm, m.bn, m.wm * m.wn * 64, m.wgs);
  } else {
    snprintf(h_buf, n, "gemm_fi_kernel<%s, %dx%d, %d threads>", dt, c.bm, c.bn, c.wm * c.wn * 64);
  }
  return FI_OK;
}

fi_status fi_gemm_inject_batch(fi_plan* plan, const fi_fault* d_faults, uint32_t n_trials, uint32_t policy,
                               fi_trial_result* d_results, float* d_c_out, void* stream) {
  fi_status st = check_batch_args(plan, d_faults, n_trials, policy, d_results);
  if (st != FI_OK) return st;
  TrialScratch ts;
  if (plan->mcfg >= 0) {
    BatchScratch* bs = nullptr;
    st = batch_scratch(plan, as_stream(stream), n_trials, &bs);
    if (st != FI_OK) return st;
    ts.perm = bs->perm; ts.counts = bs->perm + bs->cap; ts.desc = bs->desc;
  }
  return inject_batch(plan, d_faults, n_trials, policy, d_results, d_c_out, as_stream(stream), ts);
}

fi_status fi_gemm_inject_batch_act(fi_plan* plan, const fi_fault* d_faults, uint32_t n_trials, uint32_t policy,
                                   fi_trial_result* d_results, void* d_h_out, void* stream) {
  fi_status st = check_batch_args(plan, d_faults, n_trials, policy, d_results);
  if (st != FI_OK) return st;
  if (!d_h_out) return fail(FI_INVALID_ARG, "d_h_out is NULL");
  if (reinterpret_cast<uintptr_t>(d_h_out) & 1u) return fail(FI_UNSUPPORTED, "d_h_out must be 2-byte aligned");
  if (plan->mcfg < 0)
    return fail(FI_UNSUPPORTED, "the fused hand-over is not available with tile_config 2; use fi_gemm_inject_batch "
                "with d_c_out and fi_activation_round");
  BatchScratch* bs = nullptr;
  st = batch_scratch(plan, as_stream(stream), n_trials, &bs);
  if (st != FI_OK) return st;
  TrialScratch ts;
  ts.perm = bs->perm; ts.counts = bs->perm + bs->cap; ts.desc = bs->desc;
  return inject_batch(plan, d_faults, n_trials, policy, d_results, nullptr, as_stream(stream), ts,
                      static_cast<uint16_t*>(d_h_out));
}

fi_status fi_gemm_inject_batch_noalloc(fi_plan* plan, const fi_fault* d_faults, uint32_t n_trials, uint32_t policy,
                                       fi_trial_result* d_results, float* d_c_out, void* stream) {
  fi_status st = check_batch_args(plan, d_faults, n_trials, policy, d_results);
  if (st != FI_OK) return st;
  if (n_trials > kNoAllocMaxTrials)
    return fail(FI_UNSUPPORTED, "n_trials %u exceeds the %u trials the static scratch holds; split the batch or use "
                "fi_gemm_inject_batch", n_trials, kNoAllocMaxTrials);
  uint32_t* base = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    base = g_scratch_ptr[plan->device];
  }
  if (!base) return fail(FI_STATE, "the static scratch of device %d was not resolved at plan creation", plan->device);
  TrialScratch ts;
  ts.perm = base;
  ts.counts = base + kNoAllocMaxTrials;          // the two words behind the trial order
  ts.desc = base + kNoAllocPermWords;
  return inject_batch(plan, d_faults, n_trials, policy, d_results, d_c_out, as_stream(stream), ts);
}

fi_status fi_gemm_inject_batch_affected(fi_plan* plan, const fi_fault* d_faults, uint32_t n_trials,
                                        uint32_t policy, fi_trial_result* d_results, void* stream) {
  fi_status st = check_plan(plan);
  if (st != FI_OK) return st;
  if (!d_faults || !d_results) return fail(FI_INVALID_ARG, "d_faults and d_results must be non-NULL");
  if (n_trials == 0) return fail(FI_INVALID_ARG, "n_trials is 0");
  if (policy > FI_CORRECT_RECOMPUTE) return fail(FI_INVALID_ARG, "unknown correction policy %u", policy);
  if (plan->n_clean_flagged != 0)
    return fail(FI_UNSUPPORTED, "the plan's detector flags %u element(s) of the fault-free result itself, which the "
                "affected-tiles-only campaign would not count; use fi_gemm_inject_batch", plan->n_clean_flagged);
  GemmArgs a = base_args(plan, plan->cfg_affected);
  const uint64_t slots = (uint64_t)(a.tiles_m > a.tiles_n ? a.tiles_m : a.tiles_n);
  const uint64_t blocks = slots * n_trials;
  if (blocks >= (1ull << 31)) return fail(FI_UNSUPPORTED, "tiles x trials exceeds 2^31 workgroups; split the batch");
  hipStream_t s = as_stream(stream);
  const size_t words = (size_t)n_trials * (sizeof(fi_trial_result) / 4);
  hipLaunchKernelGGL(fi::fill_u32_kernel, dim3((unsigned)((words + 255) / 256 > 1024 ? 1024 : (words + 255) / 256)),
                     dim3(256), 0, s, reinterpret_cast<uint32_t*>(d_results), words, 0u);
  FI_HIP(hipGetLastError());
  a.n_trials = (int)n_trials;
  a.group = plan->group;
  a.faults = d_faults;
  a.results = d_results;
  a.policy = (int)policy;
  a.product_check = plan->product_check;
  FI_HIP(launch_gemm(fi::MODE_AFFECTED, (int)plan->d.dtype, plan->cfg_affected, a, (int)blocks, s));
  return FI_OK;
}

fi_status fi_activation_round(uint32_t dtype, const float* d_c, uint64_t n, uint16_t* d_h, void* stream) {
  if (dtype != FI_FP16 && dtype != FI_BF16)
    return fail(FI_UNSUPPORTED, "dtype %u: only FP16 (0) and BF16 (1)", dtype);
  if (!d_c || !d_h) return fail(FI_INVALID_ARG, "d_c and d_h must be non-NULL");
  if (n == 0) return fail(FI_INVALID_ARG, "n is 0");
  if ((reinterpret_cast<uintptr_t>(d_c) & 15u) || (reinterpret_cast<uintptr_t>(d_h) & 15u))
    return fail(FI_UNSUPPORTED, "d_c and d_h must be 16-byte aligned");
  uint64_t blocks = (n / 8 + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  if (blocks == 0) blocks = 1;
  if (dtype == FI_BF16)
    hipLaunchKernelGGL(fi::activation_round_kernel<FI_BF16>, dim3((unsigned)blocks), dim3(256), 0, as_stream(stream),
                       d_c, (size_t)n, d_h);
  else
    hipLaunchKernelGGL(fi::activation_round_kernel<FI_FP16>, dim3((unsigned)blocks), dim3(256), 0, as_stream(stream),
                       d_c, (size_t)n, d_h);
  FI_HIP(hipGetLastError());
  return FI_OK;
}

fi_status fi_gemm_propagate_batch(fi_plan* plan, const void* d_a_stack, uint64_t trial_stride, uint32_t n_trials,
                                  uint32_t policy, fi_trial_result* d_results, float* d_c_out, void* stream) {
  fi_status st = check_plan(plan);
  if (st != FI_OK) return st;
  if (!d_a_stack || !d_results) return fail(FI_INVALID_ARG, "d_a_stack and d_results must be non-NULL");
  if (n_trials == 0) return fail(FI_INVALID_ARG, "n_trials is 0");
  if (policy > FI_CORRECT_RECOMPUTE) return fail(FI_INVALID_ARG, "unknown correction policy %u", policy);
  if ((reinterpret_cast<uintptr_t>(d_a_stack) & 15u) || (trial_stride & 7u))
    return fail(FI_UNSUPPORTED, "d_a_stack must be 16-byte aligned with trial_stride a multiple of 8");
  if (trial_stride != 0 && trial_stride < ((uint64_t)plan->d.M - 1) * (uint64_t)plan->d.lda + plan->d.K)
    return fail(FI_INVALID_ARG, "trial_stride %llu is smaller than one operand ((M-1)*lda + K elements)",
                (unsigned long long)trial_stride);
  GemmArgs a = base_args(plan);
  // C* is addressed with 32 bits; the trials' operands are the caller's, so K must hold whole k-tiles
  const bool persistent = plan->prop_cfg >= 0 && a.c_star_bytes != 0 && plan->kshift == 0;
  if (persistent) {
    const MultiCfg mc = kMulti[plan->prop_cfg];
    a.tiles_m = (a.M + mc.bm - 1) / mc.bm;
    a.tiles_n = (a.N + mc.bn - 1) / mc.bn;
  }
  const uint64_t blocks = (uint64_t)a.tiles_m * a.tiles_n * n_trials;
  if (blocks >= (1ull << 31)) return fail(FI_UNSUPPORTED, "tiles x trials exceeds 2^31 workgroups; split the batch");
  hipStream_t s = as_stream(stream);
  const size_t words = (size_t)n_trials * (sizeof(fi_trial_result) / 4);
  hipLaunchKernelGGL(fi::fill_u32_kernel, dim3((unsigned)((words + 255) / 256 > 1024 ? 1024 : (words + 255) / 256)),
                     dim3(256), 0, s, reinterpret_cast<uint32_t*>(d_results), words, 0u);
  FI_HIP(hipGetLastError());
  a.A = static_cast<const uint16_t*>(d_a_stack);
  a.a_trial_stride = trial_stride;
  a.n_trials = (int)n_trials;
  // Trials share B but not A: a trial's tiles follow each other in the work list, so the column
  // tiles of one A panel run at the same time on one XCD and the panel comes from HBM once
  // (measured on 512 x 768 x 3072, 256 trials: 0.72 ms against 0.83 ms with three trials per tile).
  a.group = 1;
  a.results = d_results;
  a.c_out = d_c_out;
  a.policy = (int)policy;
  if (persistent) {
    // persistent workgroups walking (tile, trial) items
    const MultiCfg mc = kMulti[plan->prop_cfg];
    const uint64_t cus = (uint64_t)(plan->n_cus / 8 * 8) * (uint64_t)mc.wgs;
    FI_HIP(launch_prop((int)plan->d.dtype, plan->prop_cfg, a, (int)(blocks < cus ? blocks : cus), s));
    return FI_OK;
  }
  FI_HIP(launch_gemm(fi::MODE_PROPAGATE, (int)plan->d.dtype, plan->cfg, a, (int)blocks, s));
  return FI_OK;
}

fi_status fi_detect_correct(fi_plan* plan, float* d_c, uint32_t batch, uint32_t policy, uint8_t* d_flags,
                            uint32_t* d_n_flagged, void* stream) {
  fi_status st = check_plan(plan);
  if (st != FI_OK) return st;
  if (!d_c) return fail(FI_INVALID_ARG, "d_c is NULL");
  if (batch == 0 || batch > 65535u) return fail(FI_INVALID_ARG, "batch must be in 1..65535");
  if (policy > FI_CORRECT_RECOMPUTE) return fail(FI_INVALID_ARG, "unknown correction policy %u", policy);
  hipStream_t s = as_stream(stream);
  const fi_plan_desc& d = plan->d;
  if (d_n_flagged) {
    hipLaunchKernelGGL(fi::fill_u32_kernel, dim3((batch + 255) / 256), dim3(256), 0, s, d_n_flagged,
                       (size_t)batch, 0u);
    FI_HIP(hipGetLastError());
  }
  const size_t mn = (size_t)d.M * d.N;
  const bool vec = (d.N % 4 == 0) && ((reinterpret_cast<uintptr_t>(d_c) & 15u) == 0) &&
                   (!d_flags || (reinterpret_cast<uintptr_t>(d_flags) & 3u) == 0);
  // vector path: workgroups stride over rows; scalar path: over elements
  size_t gx = vec ? (size_t)d.M : (mn + 255) / 256;
  if (gx > 2048) gx = 2048;
  dim3 grid((unsigned)gx, batch);
  if (vec) {
    hipLaunchKernelGGL(fi::detect_correct_kernel<4>, grid, dim3(256), 0, s, d_c, (int)d.M, (int)d.N, plan->kra,
                       plan->cb, d.gamma, (int)(d.bound_mode != FI_BOUND_ROWCOL), plan->t_global, (int)policy,
                       plan->c_star, d_flags, d_n_flagged);
  } else {
    hipLaunchKernelGGL(fi::detect_correct_kernel<1>, grid, dim3(256), 0, s, d_c, (int)d.M, (int)d.N, plan->kra,
                       plan->cb, d.gamma, (int)(d.bound_mode != FI_BOUND_ROWCOL), plan->t_global, (int)policy,
                       plan->c_star, d_flags, d_n_flagged);
  }
  FI_HIP(hipGetLastError());
  return FI_OK;
}

fi_status fi_classify(fi_plan* plan, const fi_trial_result* d_results, uint32_t n_trials, uint8_t* d_class,
                      uint64_t* d_counts, void* stream) {
  fi_status st = check_plan(plan);
  if (st != FI_OK) return st;
  if (!d_results || !d_counts) return fail(FI_INVALID_ARG, "d_results and d_counts must be non-NULL");
  if (n_trials == 0) return fail(FI_INVALID_ARG, "n_trials is 0");
  hipLaunchKernelGGL(fi::classify_kernel, dim3(1), dim3(1024), 0, as_stream(stream), d_results, n_trials,
                     d_class, d_counts);
  FI_HIP(hipGetLastError());
  return FI_OK;
}

fi_status fi_deviation_histogram(fi_plan* plan, const fi_fault* d_faults, const fi_trial_result* d_results,
                                 uint32_t n_trials, uint32_t which, uint64_t* d_hist, void* stream) {
  fi_status st = check_plan(plan);
  if (st != FI_OK) return st;
  if (!d_faults || !d_results || !d_hist) return fail(FI_INVALID_ARG, "d_faults, d_results and d_hist must be non-NULL");
  if (n_trials == 0) return fail(FI_INVALID_ARG, "n_trials is 0");
  if (which > FI_HIST_DEV_POST) return fail(FI_INVALID_ARG, "unknown histogram quantity %u", which);
  hipLaunchKernelGGL(fi::deviation_histogram_kernel, dim3(1), dim3(1024), 0, as_stream(stream), d_faults, d_results,
                     n_trials, (int)which, reinterpret_cast<unsigned long long*>(d_hist));
  FI_HIP(hipGetLastError());
  return FI_OK;
}

fi_status fi_sample_faults(uint64_t seed, uint32_t first_trial, uint32_t n_trials, const fi_plan_desc* desc,
                           uint32_t kind_mode, uint32_t nbits, fi_fault* h_out) {
  fi_status st = check_desc(desc, nullptr);
  if (st != FI_OK) return st;
  if (!h_out) return fail(FI_INVALID_ARG, "h_out is NULL");
  if (kind_mode > FI_KIND_ALL_PRODUCT) return fail(FI_INVALID_ARG, "unknown kind_mode %u", kind_mode);
  if (nbits < 1 || nbits > 16) return fail(FI_INVALID_ARG, "nbits must be in 1..16");
  const uint32_t nblocks = desc->K / desc->k_block;
  for (uint32_t n = 0; n < n_trials; ++n) {
    const uint64_t t = (uint64_t)first_trial + n;
    uint64_t state = seed + (t << 32);
    uint64_t u[4];
    for (int q = 0; q < 4; ++q) u[q] = splitmix64(&state);
    fi_fault f;
    uint32_t kind = kind_mode == FI_KIND_ALL_ACC ? FI_SITE_ACC
                  : kind_mode == FI_KIND_ALL_A   ? FI_SITE_A
                  : kind_mode == FI_KIND_ALL_B   ? FI_SITE_B
                  : kind_mode == FI_KIND_ALL_PRODUCT ? FI_SITE_PRODUCT
                  : ((t & 1) ? FI_SITE_A : FI_SITE_ACC);
    f.kind = kind;
    uint32_t width = 16;
    if (kind == FI_SITE_ACC) {
      f.row = scale_to(desc->M, u[0]);
      f.col = scale_to(desc->N, u[1]);
      f.kblock = scale_to(nblocks, u[2]);
      width = 32;
    } else if (kind == FI_SITE_PRODUCT) {
      f.row = scale_to(desc->M, u[0]);
      f.col = scale_to(desc->N, u[1]);
      f.kblock = scale_to(desc->K, u[2]);          // the term: k, uniform over all MMA steps and terms
    } else {
      const uint32_t s = scale_to(nblocks, u[1]);
      const uint32_t k = s * desc->k_block + scale_to(desc->k_block, u[2]);
      f.kblock = s;
      if (kind == FI_SITE_A) { f.row = scale_to(desc->M, u[0]); f.col = k; }
      else                   { f.row = k; f.col = scale_to(desc->N, u[0]); }
    }
    const uint32_t pos = scale_to(width - nbits + 1, u[3]);
    f.xor_mask = (uint32_t)(((1ull << nbits) - 1ull) << pos);
    h_out[n] = f;
  }
  return FI_OK;
}

}  // extern "C"
