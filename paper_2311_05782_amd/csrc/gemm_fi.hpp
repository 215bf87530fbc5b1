// Fault-injecting mixed-precision GEMM for gfx950 (CDNA4, wave64).
//
// One workgroup computes one BM x BN tile of C = A x B for ONE trial of a
// campaign: FP16/BF16 operands, FP32 accumulation on the matrix cores
// (paper Sec. II-B, Sec. IV-C), with the trial's single fault (Sec. IV-A)
// applied where it belongs:
//   - accumulator fault: the owning lane XORs its accumulator register right
//     after the MFMA that finishes k-block s (the paper's write-back target,
//     Sec. III-E, is the MMA destination register);
//   - operand fault: the thread staging the faulted 16-byte chunk XORs the
//     16-bit word on its way into LDS, in every workgroup that stages it.
// The epilogue is the output-side detector / corrector (Sec. VI-A, VI-B) plus
// the per-trial counters; nothing is written to HBM but a few counters unless
// the caller asks for the outputs.
//
// Data movement: A is [M][K], B is [N][K], both K-contiguous.  A k-tile of 64
// elements is 128 bytes per row = eight 16-byte chunks.  Chunks are staged
// global -> VGPR -> LDS; chunk c of row r lands in slot c ^ g(r) of its row so
// that the ds_read_b128 of 8 (and of 16) consecutive rows touches distinct
// banks.  LDS is double buffered: one barrier per k-tile.
//
// MFMA: v_mfma_f32_32x32x16_{f16,bf16}.  Lane l feeds row (l % 32) of the A
// fragment and column (l % 32) of the B fragment with the 8 consecutive k
// values 8*(l / 32) .. +7; accumulator register v of lane l holds
// C[8*(v/4) + 4*(l/32) + v%4][l % 32] of the 32 x 32 tile.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fi.h"

namespace fi {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

enum { MODE_CAMPAIGN = 0, MODE_GOLDEN = 1 };

struct GemmArgs {
  const uint16_t* A;        // [M][lda]
  const uint16_t* B;        // [N][ldb]
  uint32_t lda, ldb;        // elements; M*lda and N*ldb fit in 31 bits
  int M, N, K, kb;
  int tiles_m, tiles_n;
  int n_trials, group;      // trials that share a tile back to back on one XCD
  const fi_fault* faults;   // [n_trials]             (campaign)
  fi_trial_result* results; // [n_trials], zeroed      (campaign)
  const float* kra;         // fl32(K * ra_i), zero padded to tiles_m * BM
  const float* cb;          // cb_j, zero padded to tiles_n * BN
  float gamma;
  int bound_global;         // 1: T = t_global everywhere
  float t_global;
  const float* c_star;      // [M][N] fault-free result  (campaign)
  const float* s_abs;       // [M][N] sum_k |a b|        (campaign)
  float* c_out;             // campaign: nullable [n_trials][M][N]; golden: [M][N]
  int policy;
  uint32_t operand_and;     // golden: AND mask on every staged dword (0x7FFF7FFF = magnitudes)
};

template <int DT>
__device__ __forceinline__ f32x16 mfma_32x32x16(u32x4 a, u32x4 b, f32x16 c) {
  if constexpr (DT == FI_BF16) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
}

// Slot permutation of the eight 16-byte chunks of a 128-byte LDS row.
// Depends on row bits 0..3 only, so it is the same for row and row + 32.
__device__ __forceinline__ int lds_swizzle(int row) { return (row & 7) ^ ((row >> 3) & 1); }

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ uint32_t wave_max(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    uint32_t w = __shfl_xor(v, o, 64);
    v = w > v ? w : v;
  }
  return v;
}

// |x| with NaN and Inf mapped to +Inf, as an ordered non-negative word.
__device__ __forceinline__ float finite_or_inf(float d) {
  return (d <= 3.4028234e38f) ? d : __uint_as_float(0x7F800000u);
}

// Workgroup id -> (tile, trial).  Workgroups are dealt round-robin to the 8
// XCDs, each with its own L2; give every XCD one contiguous slice of the work
// list, and order the list so that `group` consecutive entries are the SAME
// tile for different trials: the CUs of an XCD then stream the same A and B
// panels through that XCD's L2 at the same time.
__device__ __forceinline__ void work_of_block(const GemmArgs& p, int& tile, int& trial) {
  uint32_t w = blockIdx.x, total = gridDim.x;
  uint32_t per = total >> 3;
  uint32_t L = (w < per * 8u) ? (w & 7u) * per + (w >> 3) : w;
  uint32_t G = (uint32_t)p.group, ntiles = (uint32_t)(p.tiles_m * p.tiles_n);
  uint32_t full = ((uint32_t)p.n_trials / G) * G;
  uint32_t cut = full * ntiles;
  if (L < cut) {
    uint32_t r = L / G;
    trial = (int)((r / ntiles) * G + (L % G));
    tile = (int)(r % ntiles);
  } else {
    uint32_t G2 = (uint32_t)p.n_trials - full;
    L -= cut;
    trial = (int)(full + L % G2);
    tile = (int)(L / G2);
  }
}

template <int DT, int BM, int BN, int WM, int WN, int MODE>
__global__ void __launch_bounds__(WM* WN * 64) gemm_fi_kernel(const GemmArgs p) {
  constexpr int BK = 64;
  constexpr int NT = WM * WN * 64;
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int A_CH = BM * 8 / NT, B_CH = BN * 8 / NT;
  constexpr int ROWS_PER_PASS = NT / 8;
  constexpr int STAGE = (BM + BN) * 128;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile is a multiple of the 32x32 MFMA");
  static_assert((BM * 8) % NT == 0 && (BN * 8) % NT == 0, "every thread stages whole chunks");
  static_assert(2 * STAGE <= 160 * 1024, "two stages fit the 160 KB LDS");

  __shared__ __attribute__((aligned(16))) uint8_t smem[2 * STAGE];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, keep it scalar
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, lhi = lane >> 5;

  int tile, trial;
  work_of_block(p, tile, trial);
  const int tile_m = tile / p.tiles_n, tile_n = tile % p.tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // ---- this trial's fault, and what it means for this workgroup and wave (all uniform)
  uint32_t fkind = FI_SITE_NONE, frow = 0, fcol = 0, fmask = 0;
  int hook_k = -1;          // k index (exclusive end) after which the owning wave flips its accumulator
  int sel_t = 0, sel_v = 0, sel_lane = -1;
  bool affected = false;    // this tile can differ from the fault-free result
  int opfault_kt = -1;      // k-tile in which this workgroup stages a faulted operand word
  if constexpr (MODE == MODE_CAMPAIGN) {
    const fi_fault f = p.faults[trial];
    fkind = f.kind; frow = f.row; fcol = f.col; fmask = f.xor_mask;
    bool valid = true;
    if (fkind == FI_SITE_ACC) {
      valid = frow < (uint32_t)p.M && fcol < (uint32_t)p.N && f.kblock < (uint32_t)(p.K / p.kb);
    } else if (fkind == FI_SITE_A) {
      valid = frow < (uint32_t)p.M && fcol < (uint32_t)p.K;
    } else if (fkind == FI_SITE_B) {
      valid = frow < (uint32_t)p.K && fcol < (uint32_t)p.N;
    } else if (fkind != FI_SITE_NONE) {
      valid = false;
    }
    if (!valid) {
      if (tile == 0 && tid == 0) p.results[trial].status = 1;
      fkind = FI_SITE_NONE;
    }
    if (fkind == FI_SITE_ACC) {
      int li = (int)frow - m0, lj = (int)fcol - n0;
      if (li >= 0 && li < BM && lj >= 0 && lj < BN) {
        affected = true;
        int wi = li - wm * WTM, wj = lj - wn * WTN;
        if (wi >= 0 && wi < WTM && wj >= 0 && wj < WTN) {
          int ri = wi & 31, rj = wj & 31;
          sel_t = (wi >> 5) * TN + (wj >> 5);
          sel_v = 4 * (ri >> 3) + (ri & 3);
          sel_lane = rj + 32 * ((ri >> 2) & 1);
          hook_k = ((int)f.kblock + 1) * p.kb;
        }
      }
    } else if (fkind == FI_SITE_A) {
      int li = (int)frow - m0;
      if (li >= 0 && li < BM) { affected = true; opfault_kt = (int)fcol / BK; }
    } else if (fkind == FI_SITE_B) {
      int lj = (int)fcol - n0;
      if (lj >= 0 && lj < BN) { affected = true; opfault_kt = (int)frow / BK; }
    }
  }

  // ---- staging maps
  const int st_row = tid >> 3, st_ch = tid & 7;       // pass c adds c * ROWS_PER_PASS rows
  uint32_t a_goff[A_CH], b_goff[B_CH];                // element offsets of this thread's chunks at k = 0
  bool a_ok[A_CH], b_ok[B_CH];
  int a_soff[A_CH], b_soff[B_CH];                     // byte offsets inside a stage
#pragma unroll
  for (int c = 0; c < A_CH; ++c) {
    int row = st_row + c * ROWS_PER_PASS;
    a_ok[c] = (m0 + row) < p.M;
    a_goff[c] = (uint32_t)(m0 + row) * p.lda + (uint32_t)(st_ch * 8);
    a_soff[c] = row * 128 + ((st_ch ^ lds_swizzle(row)) << 4);
  }
#pragma unroll
  for (int c = 0; c < B_CH; ++c) {
    int row = st_row + c * ROWS_PER_PASS;
    b_ok[c] = (n0 + row) < p.N;
    b_goff[c] = (uint32_t)(n0 + row) * p.ldb + (uint32_t)(st_ch * 8);
    b_soff[c] = BM * 128 + row * 128 + ((st_ch ^ lds_swizzle(row)) << 4);
  }

  u32x4 ga[A_CH], gb[B_CH];
  const u32x4 zero4 = {0u, 0u, 0u, 0u};

  auto load_tile = [&](int kt) {
    const int k0 = kt * BK;
    const bool kin = (k0 + st_ch * 8) < p.K;
#pragma unroll
    for (int c = 0; c < A_CH; ++c)
      ga[c] = (a_ok[c] && kin) ? *reinterpret_cast<const u32x4*>(p.A + a_goff[c] + k0) : zero4;
#pragma unroll
    for (int c = 0; c < B_CH; ++c)
      gb[c] = (b_ok[c] && kin) ? *reinterpret_cast<const u32x4*>(p.B + b_goff[c] + k0) : zero4;
  };

  auto store_tile = [&](int kt, int stage) {
    if constexpr (MODE == MODE_GOLDEN) {
#pragma unroll
      for (int c = 0; c < A_CH; ++c) ga[c] &= p.operand_and;
#pragma unroll
      for (int c = 0; c < B_CH; ++c) gb[c] &= p.operand_and;
    } else {
      if (kt == opfault_kt) {   // uniform, at most one k-tile of a few workgroups per trial
        const int kk = (fkind == FI_SITE_A ? (int)fcol : (int)frow) - kt * BK;   // 0..63
        const int want_row = (fkind == FI_SITE_A) ? (int)frow - m0 : (int)fcol - n0;
        const uint32_t m16 = (fmask & 0xFFFFu) << ((kk & 1) * 16);
        if (st_ch == (kk >> 3)) {
          const int dw = (kk & 7) >> 1;
          if (fkind == FI_SITE_A) {
#pragma unroll
            for (int c = 0; c < A_CH; ++c) {
              if (st_row + c * ROWS_PER_PASS == want_row) {
                uint32_t before = (ga[c][dw] >> ((kk & 1) * 16)) & 0xFFFFu;
                ga[c][dw] ^= m16;
                if (tile_n == 0) {
                  p.results[trial].site_word_before = before;
                  p.results[trial].site_word_after = before ^ (fmask & 0xFFFFu);
                }
              }
            }
          } else {
#pragma unroll
            for (int c = 0; c < B_CH; ++c) {
              if (st_row + c * ROWS_PER_PASS == want_row) {
                uint32_t before = (gb[c][dw] >> ((kk & 1) * 16)) & 0xFFFFu;
                gb[c][dw] ^= m16;
                if (tile_m == 0) {
                  p.results[trial].site_word_before = before;
                  p.results[trial].site_word_after = before ^ (fmask & 0xFFFFu);
                }
              }
            }
          }
        }
      }
    }
    uint8_t* s = smem + stage * STAGE;
#pragma unroll
    for (int c = 0; c < A_CH; ++c) *reinterpret_cast<u32x4*>(s + a_soff[c]) = ga[c];
#pragma unroll
    for (int c = 0; c < B_CH; ++c) *reinterpret_cast<u32x4*>(s + b_soff[c]) = gb[c];
  };

  // ---- fragment read maps: row = wave base + 32*t + l32, chunk = 2*kk + lhi
  const int sw = lds_swizzle(l32);
  int slot[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) slot[kk] = ((2 * kk + lhi) ^ sw) << 4;
  const int a_rd = (wm * WTM + l32) * 128;
  const int b_rd = BM * 128 + (wn * WTN + l32) * 128;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  const int nkt = (p.K + BK - 1) / BK;
  load_tile(0);
  store_tile(0, 0);
  __syncthreads();

  for (int kt = 0; kt < nkt; ++kt) {
    const int stage = kt & 1;
    if (kt + 1 < nkt) load_tile(kt + 1);
    const uint8_t* s = smem + stage * STAGE;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      u32x4 af[TM], bf[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = *reinterpret_cast<const u32x4*>(s + a_rd + i * 4096 + slot[kk]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        bf[j] = *reinterpret_cast<const u32x4*>(s + b_rd + j * 4096 + slot[kk]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = mfma_32x32x16<DT>(af[i], bf[j], acc[i][j]);

      if constexpr (MODE == MODE_CAMPAIGN) {
        // Accumulator fault: k-block s ends at k = (s+1)*kb; kb is a multiple of 16, so
        // that boundary is the end of one of these 16-wide steps.  Taken by one wave of
        // one workgroup per trial.
        if (hook_k == kt * BK + (kk + 1) * 16) {
#pragma unroll
          for (int t = 0; t < TM * TN; ++t) {
            if (t == sel_t) {
#pragma unroll
              for (int v = 0; v < 16; ++v) {
                uint32_t w = __float_as_uint(acc[t / TN][t % TN][v]);
                if (v == sel_v && lane == sel_lane) {
                  p.results[trial].site_word_before = w;
                  w ^= fmask;
                  p.results[trial].site_word_after = w;
                }
                acc[t / TN][t % TN][v] = __uint_as_float(w);
              }
            }
          }
        }
      }
    }
    if (kt + 1 < nkt) store_tile(kt + 1, stage ^ 1);
    __syncthreads();
  }

  // ---- epilogue: detector, corrector, counters
  const float inf = __uint_as_float(0x7F800000u);
  uint32_t n_flag = 0, n_bit = 0, n_pre = 0, n_post = 0, n_bT = 0, n_btau = 0;
  float mx_pre = 0.0f, mx_post = 0.0f;
  float* cout = nullptr;
  if (p.c_out) {
    cout = p.c_out + (MODE == MODE_CAMPAIGN ? (size_t)trial * (size_t)p.M * (size_t)p.N : (size_t)0);
  }

#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r0 = m0 + wm * WTM + i * 32 + 8 * q + 4 * lhi;     // rows r0 .. r0+3
      f32x4 kra4 = {0.f, 0.f, 0.f, 0.f};
      if constexpr (MODE == MODE_CAMPAIGN) kra4 = *reinterpret_cast<const f32x4*>(p.kra + r0);
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * WTN + j * 32 + l32;
        float cbj = 0.f;
        if constexpr (MODE == MODE_CAMPAIGN) cbj = p.cb[col];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int row = r0 + e;
          const bool inb = row < p.M && col < p.N;
          float c = acc[i][j][4 * q + e];
          if constexpr (MODE == MODE_GOLDEN) {
            if (inb) cout[(size_t)row * p.N + col] = c;
          } else {
            float T = p.bound_global ? p.t_global
                                     : __fmul_rn(__fmul_rn(kra4[e], cbj), p.gamma);
            const bool flag = inb && !(fabsf(c) <= T);
            n_flag += flag ? 1u : 0u;
            float cc = c;
            if (flag) {
              if (p.policy == FI_CORRECT_ZERO) cc = 0.0f;
              else if (p.policy == FI_CORRECT_RECOMPUTE) cc = p.c_star[(size_t)row * p.N + col];
            }
            if (affected && inb) {
              const size_t idx = (size_t)row * p.N + col;
              const float cs = p.c_star[idx];
              const float tau = p.s_abs[idx] * 0.000244140625f;   // 2^-12, exact scaling
              const float dpre = finite_or_inf(fabsf(c - cs));
              const float dpost = finite_or_inf(fabsf(cc - cs));
              const bool changed = __float_as_uint(c) != __float_as_uint(cs);
              n_bit += changed ? 1u : 0u;
              n_pre += !(dpre <= tau) ? 1u : 0u;
              n_post += !(dpost <= tau) ? 1u : 0u;
              mx_pre = fmaxf(mx_pre, dpre);
              mx_post = fmaxf(mx_post, dpost);
              if (changed) {
                const float band = fmaxf(2.0f * tau, T * 0.015625f);
                const float mag = fabsf(c);
                n_bT += (mag <= 3.4028234e38f && fabsf(mag - T) <= band) ? 1u : 0u;
                n_btau += (tau > 0.0f && dpre >= 0.5f * tau && dpre <= 2.0f * tau) ? 1u : 0u;
              }
            }
            if (cout && inb) cout[(size_t)row * p.N + col] = cc;
          }
        }
      }
    }
  }

  if constexpr (MODE == MODE_CAMPAIGN) {
    fi_trial_result* r = p.results + trial;
    if (__ballot(n_flag != 0)) {
      uint32_t s = wave_sum(n_flag);
      if (lane == 0) atomicAdd(&r->n_flagged, s);
    }
    if (affected) {
      uint32_t s;
      s = wave_sum(n_bit);  if (lane == 0 && s) atomicAdd(&r->n_bitdiff, s);
      s = wave_sum(n_pre);  if (lane == 0 && s) atomicAdd(&r->n_dev_pre, s);
      s = wave_sum(n_post); if (lane == 0 && s) atomicAdd(&r->n_dev_post, s);
      s = wave_sum(n_bT);   if (lane == 0 && s) atomicAdd(&r->n_border_T, s);
      s = wave_sum(n_btau); if (lane == 0 && s) atomicAdd(&r->n_border_tau, s);
      // non-negative floats (and +Inf) order like their words
      s = wave_max(__float_as_uint(mx_pre));
      if (lane == 0 && s) atomicMax(reinterpret_cast<uint32_t*>(&r->max_dev_pre), s);
      s = wave_max(__float_as_uint(mx_post));
      if (lane == 0 && s) atomicMax(reinterpret_cast<uint32_t*>(&r->max_dev_post), s);
    }
  }
  (void)inf;
}

}  // namespace fi
