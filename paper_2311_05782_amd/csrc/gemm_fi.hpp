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
// elements is 128 bytes per row = eight 16-byte chunks.  Chunks go global -> LDS
// directly (global_load_lds, no staging registers); chunk c of row r lands in
// slot c ^ g(r) of its row so that the ds_read_b128 of 8 (and of 16) consecutive
// rows touches distinct banks.  LDS is double buffered: one barrier per k-tile.
//
// MFMA: v_mfma_f32_32x32x16_{f16,bf16}.  Lane l feeds row (l % 32) of the A
// fragment and column (l % 32) of the B fragment with the 8 consecutive k
// values 8*(l / 32) .. +7; accumulator register v of lane l holds
// C[8*(v/4) + 4*(l/32) + v%4][l % 32] of the 32 x 32 tile.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "fi.h"

namespace fi {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// CAMPAIGN: every tile of every trial.  GOLDEN: the plan's fault-free pass.  AFFECTED: only the
// tiles a trial's fault can reach (one workgroup slot per trial and candidate tile).  PROPAGATE:
// no fault of its own; every trial multiplies its OWN A operand (the activations a faulty
// previous layer handed on) and every output element is compared with the fault-free result.
enum { MODE_CAMPAIGN = 0, MODE_GOLDEN = 1, MODE_AFFECTED = 2, MODE_PROPAGATE = 3 };

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
  // Bytes the c_star allocation spans, or 0.  The plan pads it to whole 256-row tiles plus one
  // tile width, so that a tile reaching over the edge of a ragged problem reads allocated memory.
  uint32_t c_star_bytes;
  float* c_out;             // campaign: nullable [n_trials][M][N]; golden: [M][N]
  // Campaign (multi-trial kernel), nullable: [n_trials][M][N] words of the operand format, the
  // corrected output after ReLU and rounding - the next layer's operand, written by the epilogue
  // instead of an FP32 output that a second kernel would read back.
  uint16_t* h_out;
  int policy;
  int product_check;        // FI_PCHECK_* applied to the erroneous product of PRODUCT faults
  // For the multi-trial kernel: the batch split in two parts (trials that leave the operands
  // alone, operand-fault trials): part_counts = {c0, c1}, perm = the trial order, desc = 6 words
  // per trial in that order, see gemm_fi_multi.hpp.
  const uint32_t* perm;
  const uint32_t* part_counts;
  const uint32_t* desc;
  uint64_t a_trial_stride;  // PROPAGATE: trial t reads A + t * a_trial_stride (elements)
  // Measurement aid, nullable: workgroup 0 of the persistent kernel writes the shader-clock
  // counter and the constant-rate (100 MHz) counter when it starts and when it has finished its
  // last item - {cycles, ticks, cycles, ticks} at clocks + 4 * VAR - from which the host derives
  // the shader clock the launch sustained.
  unsigned long long* clocks;
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

// Exact value of a 16-bit operand word as a float (Sec. II-A formats).
template <int DT>
__device__ __forceinline__ float decode16(uint32_t w) {
  if constexpr (DT == FI_BF16) {
    return __uint_as_float(w << 16);
  } else {
    unsigned short h = (unsigned short)w;
    return (float)__builtin_bit_cast(_Float16, h);
  }
}

// binary32 -> FP16 / BF16 word, round to nearest even, in integer arithmetic (no dependence on
// the wave's denormal or rounding modes).  The paper's fault model holds a product in the
// operand format (Sec. IV-C).
template <int DT>
__device__ __forceinline__ uint32_t round16(float x) {
  const uint32_t b = __float_as_uint(x);
  const uint32_t sign = (b >> 16) & 0x8000u;
  const uint32_t mag = b & 0x7FFFFFFFu;
  if constexpr (DT == FI_BF16) {
    if (mag > 0x7F800000u) return sign | 0x7FC0u;
    return sign | ((mag + 0x7FFFu + ((mag >> 16) & 1u)) >> 16);          // a carry may reach Inf
  } else {
    if (mag > 0x7F800000u) return sign | 0x7E00u;
    if (mag >= 0x477FF000u) return sign | 0x7C00u;                       // >= 65520: Inf
    if (mag < 0x38800000u) {                                             // below 2^-14: subnormal grid
      if (mag <= 0x33000000u) return sign;                               // <= 2^-25 (tie to even): 0
      const uint32_t e = mag >> 23;                                      // 102 .. 112
      const uint32_t m = (mag & 0x7FFFFFu) | 0x800000u;                  // value = m * 2^(e - 150)
      const uint32_t shift = 126u - e;                                   // multiples of 2^-24
      uint32_t q = m >> shift;
      const uint32_t rem = m & ((1u << shift) - 1u), half = 1u << (shift - 1u);
      if (rem > half || (rem == half && (q & 1u))) ++q;
      return sign | q;
    }
    const uint32_t e = (mag >> 23) - 112u;                               // FP16 biased exponent
    const uint32_t m = mag & 0x7FFFFFu;
    uint32_t h = (e << 10) | (m >> 13);
    const uint32_t rem = m & 0x1FFFu;
    if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) ++h;              // a carry bumps the exponent
    return sign | h;
  }
}

// round16(relu(x)) without a branch or a select, for the output paths that convert every element:
// relu keeps a NaN (quieted, sign kept) and maps negatives and -0 to +0.  Same integer arithmetic
// as round16: adding (half - 1) + (the bit that becomes the last place) before the shift rounds to
// nearest even, a carry moves into the exponent; FP16 merges the normal grid (clamped to Inf) with
// the subnormal grid (multiples of 2^-24; inputs below 2^-25 shift out entirely).  Conditions are
// sign masks merged bitwise: written as selects, the compiler moves each arm into a branch of its
// own (exec-mask juggling per element).
template <int DT>
__device__ __forceinline__ uint32_t relu_round16(float x) {
  const uint32_t b = __float_as_uint(x);
  const uint32_t nan_mask = (uint32_t)((int32_t)(0x7F800000u - (b & 0x7FFFFFFFu)) >> 31);   // magnitude above Inf
  const uint32_t r = b & ~(uint32_t)((int32_t)b >> 31);                                     // negative words -> +0
  uint32_t h, nan_word = (b >> 16) & 0x8000u;
  if constexpr (DT == FI_BF16) {
    h = (r + 0x7FFFu + ((r >> 16) & 1u)) >> 16;
    nan_word |= 0x7FC0u;
  } else {
    const uint32_t hn = min((r - 0x38000000u + 0xFFFu + ((r >> 13) & 1u)) >> 13, 0x7C00u);
    const uint32_t sh = min(126u - min(r >> 23, 126u), 25u);
    const uint32_t m = (r & 0x7FFFFFu) | 0x800000u;
    const uint32_t hs = (m + ((1u << (sh - 1u)) - 1u) + ((m >> sh) & 1u)) >> sh;
    const uint32_t sub_mask = (uint32_t)((int32_t)(r - 0x38800000u) >> 31);                 // below 2^-14 (r < 2^31)
    h = (hs & sub_mask) | (hn & ~sub_mask);
    nan_word |= 0x7E00u;
  }
  return (nan_word & nan_mask) | (h & ~nan_mask);
}

// Exponent-only check of an erroneous product word (Sec. VI-A).  Bound check (BF16): exponent
// 1eeexxxx with a 1 among eee means |value| >= 2^17; the three bits are cleared.  Range check:
// the product's exponent field cannot exceed be_a + be_b - bias + 1 (from m1*m2 < 4); "max"
// replaces a larger field by the bound, "flip" clears its 1 bits from the right until it fits.
template <int DT>
__device__ __forceinline__ uint32_t product_check(uint32_t w_err, uint32_t a_word, uint32_t b_word, int mode,
                                                  bool& fired) {
  constexpr int MB = DT == FI_BF16 ? 7 : 10, EB = DT == FI_BF16 ? 8 : 5, BIAS = DT == FI_BF16 ? 127 : 15;
  constexpr uint32_t EMASK = (1u << EB) - 1u;
  uint32_t e = (w_err >> MB) & EMASK;
  fired = false;
  if (mode == FI_PCHECK_BOUND) {
    if (DT == FI_BF16 && (e & 0x80u) && (e & 0x70u)) { fired = true; e &= ~0x70u; }
  } else if (mode == FI_PCHECK_RANGE_MAX || mode == FI_PCHECK_RANGE_FLIP) {
    const int bound = max((int)((a_word >> MB) & EMASK) + (int)((b_word >> MB) & EMASK) - BIAS + 1, 0);
    if ((int)e > bound) {
      fired = true;
      if (mode == FI_PCHECK_RANGE_MAX) {
        e = (uint32_t)bound;
      } else {
#pragma unroll
        for (int bit = 0; bit < EB; ++bit)
          if ((int)e > bound) e &= ~(1u << bit);
      }
    }
  }
  return (w_err & ~(EMASK << MB) & 0xFFFFu) | (e << MB);
}

// Product-term fault (Sec. III-E): re = a*b held in the operand format, re_err = its word XOR
// mask, passed through the exponent-only check if one is enabled.
template <int DT>
__device__ __forceinline__ void product_fault_terms(uint32_t a_word, uint32_t b_word, uint32_t mask, int check,
                                                    float& re, float& re_err, bool& fired) {
  const uint32_t w = round16<DT>(__fmul_rn(decode16<DT>(a_word), decode16<DT>(b_word)));
  uint32_t w_err = (w ^ mask) & 0xFFFFu;
  fired = false;
  if (check != FI_PCHECK_NONE) w_err = product_check<DT>(w_err, a_word, b_word, check, fired);
  re = decode16<DT>(w);
  re_err = decode16<DT>(w_err);
}
// The write-back of Eq. (1)-(2): two binary32 operations, each rounded once.
__device__ __forceinline__ float write_back(float re_sum, float re, float re_err) {
  return __fadd_rn(__fsub_rn(re_sum, re), re_err);
}

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>).  Keeps every
// accumulator index a constant from the front end on, whatever the optimiser's unrolling does.
template <int... I, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F&&>(f));
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

// Workgroup id -> (tile, item), item = a trial or a group of trials.  Workgroups are dealt
// round-robin to the 8 XCDs, each with its own L2; give every XCD one contiguous slice of the
// work list, and order the list so that `group` consecutive entries are the SAME tile for
// different items: the CUs of an XCD then stream the same A and B panels through that XCD's L2
// at the same time.  The list holds total = n_tiles * n_items entries; w is a position in
// dispatch order (a workgroup id, or a persistent workgroup's id plus a multiple of a grid
// size divisible by 8).  n_items may be a count only the device knows, so a grid may be
// larger than the list: work_of_block returns false for a workgroup beyond it.
__device__ __forceinline__ void work_of_index(uint32_t w, uint32_t total, int n_tiles, int n_items, int group,
                                              int& tile, int& item) {
  uint32_t per = total >> 3;
  uint32_t L = (w < per * 8u) ? (w & 7u) * per + (w >> 3) : w;
  uint32_t G = (uint32_t)min(group, n_items), ntiles = (uint32_t)n_tiles;
  uint32_t full = ((uint32_t)n_items / G) * G;
  uint32_t cut = full * ntiles;
  if (L < cut) {
    uint32_t r = L / G;
    item = (int)((r / ntiles) * G + (L % G));
    tile = (int)(r % ntiles);
  } else {
    uint32_t G2 = (uint32_t)n_items - full;
    L -= cut;
    item = (int)(full + L % G2);
    tile = (int)(L / G2);
  }
}
__device__ __forceinline__ bool work_of_block(int n_tiles, int n_items, int group, int& tile, int& item) {
  const uint32_t total = (uint32_t)n_tiles * (uint32_t)n_items;
  if (blockIdx.x >= total) return false;
  work_of_index(blockIdx.x, total, n_tiles, n_items, group, tile, item);
  return true;
}

template <int DT, int BM, int BN, int WM, int WN, int MODE>
__global__ void __launch_bounds__(WM* WN * 64) gemm_fi_kernel(const GemmArgs p) {
  constexpr int BK = 64;
  constexpr int NT = WM * WN * 64;
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int STAGE = (BM + BN) * 128;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile is a multiple of the 32x32 MFMA");
  static_assert(2 * STAGE <= 160 * 1024, "two stages fit the 160 KB LDS");

  __shared__ __attribute__((aligned(16))) uint8_t smem[2 * STAGE];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, keep it scalar
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, lhi = lane >> 5;

  int tile, trial;
  if constexpr (MODE == MODE_AFFECTED) {
    // Slot q of trial t: an accumulator or product-term fault reaches one tile (slot 0), an A
    // fault the tiles_n tiles of its tile row, a B fault the tiles_m tiles of its tile column.
    // The grid holds max(tiles_m, tiles_n) slots per trial, slot-major: consecutive workgroup
    // ids are the same slot of consecutive trials, so the working ones spread over all XCDs.
    trial = (int)(blockIdx.x % (uint32_t)p.n_trials);
    const int q = (int)(blockIdx.x / (uint32_t)p.n_trials);
    const fi_fault f = p.faults[trial];
    if (f.kind == FI_SITE_ACC || f.kind == FI_SITE_PRODUCT) {
      const bool valid = f.row < (uint32_t)p.M && f.col < (uint32_t)p.N &&
                         f.kblock < (uint32_t)(f.kind == FI_SITE_ACC ? p.K / p.kb : p.K);
      if (!valid && q == 0 && tid == 0) p.results[trial].status = 1;
      if (!valid || q != 0) return;
      tile = (int)(f.row / BM) * p.tiles_n + (int)(f.col / BN);
    } else if (f.kind == FI_SITE_A) {
      const bool valid = f.row < (uint32_t)p.M && f.col < (uint32_t)p.K;
      if (!valid && q == 0 && tid == 0) p.results[trial].status = 1;
      if (!valid || q >= p.tiles_n) return;
      tile = (int)(f.row / BM) * p.tiles_n + q;
    } else if (f.kind == FI_SITE_B) {
      const bool valid = f.row < (uint32_t)p.K && f.col < (uint32_t)p.N;
      if (!valid && q == 0 && tid == 0) p.results[trial].status = 1;
      if (!valid || q >= p.tiles_m) return;
      tile = q * p.tiles_n + (int)(f.col / BN);
    } else {
      if (f.kind != FI_SITE_NONE && q == 0 && tid == 0) p.results[trial].status = 1;
      return;                                            // nothing can differ
    }
  } else {
    work_of_block(p.tiles_m * p.tiles_n, p.n_trials, p.group, tile, trial);
  }
  const int tile_m = tile / p.tiles_n, tile_n = tile % p.tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // ---- this trial's fault, and what it means for this workgroup and wave (all uniform)
  uint32_t fkind = FI_SITE_NONE, frow = 0, fcol = 0, fmask = 0;
  int hook_kt = -1;         // owning wave: flip the accumulator after this k-tile
  int fk = 0;               // product-term fault: k of the term
  int kshift = 0;           // this workgroup's k-tiles start at -kshift (see below)
  int sel_t = 0, sel_v = 0, sel_lane = -1;
  bool affected = false;    // this tile can differ from the fault-free result
  int opfault_kt = -1;      // k-tile in which this workgroup stages a faulted operand word
  if constexpr (MODE == MODE_PROPAGATE) affected = true;
  if constexpr (MODE == MODE_CAMPAIGN || MODE == MODE_AFFECTED) {
    const fi_fault f = p.faults[trial];
    fkind = f.kind; frow = f.row; fcol = f.col; fmask = f.xor_mask;
    bool valid = true;
    if (fkind == FI_SITE_ACC) {
      valid = frow < (uint32_t)p.M && fcol < (uint32_t)p.N && f.kblock < (uint32_t)(p.K / p.kb);
    } else if (fkind == FI_SITE_PRODUCT) {
      valid = frow < (uint32_t)p.M && fcol < (uint32_t)p.N && f.kblock < (uint32_t)p.K;
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
    if (fkind == FI_SITE_ACC || fkind == FI_SITE_PRODUCT) {
      const int li = (int)frow - m0, lj = (int)fcol - n0;
      if (li >= 0 && li < BM && lj >= 0 && lj < BN) {
        affected = true;
        // k-block s ends at k = (s+1)*kb, a multiple of 16 but not always of the 64-wide
        // k-tile.  The workgroup that owns the site shifts its k-tiling down by kshift so that
        // this boundary is the end of a k-tile: its first tile starts at k = -kshift with the
        // part below 0 read as zeros.  The sequence of 16-wide MFMA steps over real data is
        // unchanged (steps over zeros leave the +0 accumulators as they are), so every other
        // element of the tile still equals the fault-free result bit for bit.
        // A product-term fault is written back after the 16-wide MMA step holding its k.
        const int hook_k = fkind == FI_SITE_ACC ? ((int)f.kblock + 1) * p.kb : ((int)f.kblock / 16 + 1) * 16;
        fk = (int)f.kblock;
        kshift = (BK - hook_k % BK) % BK;
        const int wi = li - wm * WTM, wj = lj - wn * WTN;
        if (wi >= 0 && wi < WTM && wj >= 0 && wj < WTN) {
          const int ri = wi & 31, rj = wj & 31;
          sel_t = (wi >> 5) * TN + (wj >> 5);
          sel_v = 4 * (ri >> 3) + (ri & 3);
          sel_lane = rj + 32 * ((ri >> 2) & 1);
          hook_kt = (hook_k + kshift) / BK - 1;
        }
      }
    } else if (fkind == FI_SITE_A) {
      const int li = (int)frow - m0;
      if (li >= 0 && li < BM) { affected = true; opfault_kt = (int)fcol / BK; }   // kshift is 0 here
    } else if (fkind == FI_SITE_B) {
      const int lj = (int)fcol - n0;
      if (lj >= 0 && lj < BN) { affected = true; opfault_kt = (int)frow / BK; }
    }
  }

  // ---- staging: global -> LDS without passing through registers.  One global_load_lds of 16
  // bytes per lane fills 1024 contiguous LDS bytes = 8 rows x 8 slots: lane l lands in row
  // (l >> 3), slot (l & 7) of its row group, so it must FETCH chunk slot ^ g(row).  Wave w issues
  // the row groups w*A_CH .. of the A tile and w*B_CH .. of the B tile.  Rows past the end of A
  // or B are clamped to the last row (they feed only outputs that are never stored or counted).
  constexpr int NW = WM * WN;
  constexpr int A_G = BM / 8 / NW, B_G = BN / 8 / NW;      // row groups per wave
  static_assert((BM / 8) % NW == 0 && (BN / 8) % NW == 0, "row groups divide among the waves");
  const int lrow = lane >> 3, lslot = lane & 7;
  uint32_t a_goff[A_G], b_goff[B_G];                  // element offsets of this lane's chunks at k = 0
#pragma unroll
  for (int c = 0; c < A_G; ++c) {
    const int row = (wave * A_G + c) * 8 + lrow;
    a_goff[c] = (uint32_t)min(m0 + row, p.M - 1) * p.lda + (uint32_t)((lslot ^ lds_swizzle(row)) * 8);
  }
#pragma unroll
  for (int c = 0; c < B_G; ++c) {
    const int row = (wave * B_G + c) * 8 + lrow;
    b_goff[c] = (uint32_t)min(n0 + row, p.N - 1) * p.ldb + (uint32_t)((lslot ^ lds_swizzle(row)) * 8);
  }

  typedef __attribute__((address_space(3))) void lds_void;
  typedef const __attribute__((address_space(1))) void glb_void;
  const uint16_t* const Ap = MODE == MODE_PROPAGATE ? p.A + (size_t)trial * p.a_trial_stride : p.A;

  // Issue the loads of k-tile kt into `stage`.  Returns false if the tile is not wholly inside
  // [0, K): then fix_tile() must zero what lies outside once the loads have landed.
  auto issue_tile = [&](int kt, int stage) {
    const int k0 = kt * BK - kshift;
    const bool inside = k0 >= 0 && k0 + BK <= p.K;       // uniform
    uint8_t* sA = smem + stage * STAGE + wave * (A_G * 1024);
    uint8_t* sB = smem + stage * STAGE + BM * 128 + wave * (B_G * 1024);
    if (inside) {
#pragma unroll
      for (int c = 0; c < A_G; ++c)
        __builtin_amdgcn_global_load_lds((glb_void*)(Ap + a_goff[c] + k0), (lds_void*)(sA + c * 1024), 16, 0, 0);
#pragma unroll
      for (int c = 0; c < B_G; ++c)
        __builtin_amdgcn_global_load_lds((glb_void*)(p.B + b_goff[c] + k0), (lds_void*)(sB + c * 1024), 16, 0, 0);
    } else {
      // chunks outside [0, K) are fetched from the start of their row (always inside the operand,
      // also when K < 64) and zeroed later
#pragma unroll
      for (int c = 0; c < A_G; ++c) {
        const int ch = (lslot ^ lds_swizzle((wave * A_G + c) * 8 + lrow)) * 8;
        const bool kin = (k0 + ch) >= 0 && (k0 + ch) < p.K;
        __builtin_amdgcn_global_load_lds((glb_void*)(Ap + a_goff[c] + (kin ? k0 : -ch)), (lds_void*)(sA + c * 1024), 16, 0, 0);
      }
#pragma unroll
      for (int c = 0; c < B_G; ++c) {
        const int ch = (lslot ^ lds_swizzle((wave * B_G + c) * 8 + lrow)) * 8;
        const bool kin = (k0 + ch) >= 0 && (k0 + ch) < p.K;
        __builtin_amdgcn_global_load_lds((glb_void*)(p.B + b_goff[c] + (kin ? k0 : -ch)), (lds_void*)(sB + c * 1024), 16, 0, 0);
      }
    }
  };

  // After the loads of k-tile kt have landed (and before the barrier that publishes them): zero
  // the chunks outside [0, K) and apply an operand fault.  Each lane touches only the 16 bytes it
  // fetched itself.  Both cases are rare and uniform.
  auto fix_tile = [&](int kt, int stage) {
    const int k0 = kt * BK - kshift;
    uint8_t* sA = smem + stage * STAGE + wave * (A_G * 1024) + lane * 16;
    uint8_t* sB = smem + stage * STAGE + BM * 128 + wave * (B_G * 1024) + lane * 16;
    if (!(k0 >= 0 && k0 + BK <= p.K)) {
      const u32x4 zero4 = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int c = 0; c < A_G; ++c) {
        const int ch = (lslot ^ lds_swizzle((wave * A_G + c) * 8 + lrow)) * 8;
        if (!((k0 + ch) >= 0 && (k0 + ch) < p.K)) *reinterpret_cast<u32x4*>(sA + c * 1024) = zero4;
      }
#pragma unroll
      for (int c = 0; c < B_G; ++c) {
        const int ch = (lslot ^ lds_swizzle((wave * B_G + c) * 8 + lrow)) * 8;
        if (!((k0 + ch) >= 0 && (k0 + ch) < p.K)) *reinterpret_cast<u32x4*>(sB + c * 1024) = zero4;
      }
    }
    if constexpr (MODE == MODE_CAMPAIGN || MODE == MODE_AFFECTED) {
      if (kt == opfault_kt) {
        const bool isA = fkind == FI_SITE_A;
        const int kk = (isA ? (int)fcol : (int)frow) - kt * BK;            // 0..63 (kshift is 0 here)
        const int want_row = isA ? (int)frow - m0 : (int)fcol - n0;        // row inside the tile
        const int groups = isA ? A_G : B_G;
        const int g = want_row >> 3;                                       // row group inside the tile
        // the lane that fetched chunk (kk >> 3) of that row
        const int want_lane = ((want_row & 7) << 3) | ((kk >> 3) ^ lds_swizzle(want_row));
        if (g / groups == wave && lane == want_lane) {
          uint8_t* base = (isA ? sA : sB) + (g % groups) * 1024;
          uint16_t* w16 = reinterpret_cast<uint16_t*>(base) + (kk & 7);
          const uint32_t before = *w16;
          *w16 = (uint16_t)(before ^ (fmask & 0xFFFFu));
          if (isA ? tile_n == 0 : tile_m == 0) {
            p.results[trial].site_word_before = before;
            p.results[trial].site_word_after = before ^ (fmask & 0xFFFFu);
          }
        }
      }
    }
  };

  // ---- fragment read maps: row = wave base + 32*t + l32, chunk = 2*kk + lhi
  const int sw = lds_swizzle(l32);
  const int a_rd = (wm * WTM + l32) * 128;
  const int b_rd = BM * 128 + (wn * WTN + l32) * 128;

  f32x16 acc[TM][TN];
  static_for<TM * TN>([&](auto t) {
    acc[t / TN][t % TN] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  });

  // Fragments of one 16-wide k-step: TM + TN ds_read_b128.  Two sets, so the reads of step
  // kk + 1 are in flight while the TM x TN MFMAs of step kk run.
  struct Frags { u32x4 a[TM]; u32x4 b[TN]; };
  auto read_frags = [&](Frags& f, const uint8_t* s, int kk) {
    const int slot = ((2 * kk + lhi) ^ sw) << 4;
#pragma unroll
    for (int i = 0; i < TM; ++i) f.a[i] = *reinterpret_cast<const u32x4*>(s + a_rd + i * 4096 + slot);
#pragma unroll
    for (int j = 0; j < TN; ++j) f.b[j] = *reinterpret_cast<const u32x4*>(s + b_rd + j * 4096 + slot);
  };
  // One MFMA step; `mid` (the fragment read for the next step) is issued after the first two
  // MFMAs, so it lands under the rest of the burst and is never waited for right after its issue.
  auto mma_step = [&](const Frags& f, auto&& mid) __attribute__((always_inline)) {
    static_for<TM * TN>([&](auto t) {
      constexpr int i = t / TN, j = t % TN;
      if constexpr (t == (TM * TN >= 8 ? 2 : 1)) {
        __builtin_amdgcn_sched_barrier(0);
        mid();
        __builtin_amdgcn_sched_barrier(0);
      }
      acc[i][j] = mfma_32x32x16<DT>(f.a[i], f.b[j], acc[i][j]);
    });
  };

  // Accumulator fault: XOR the owning lane's register.  Which 32x32 tile is a uniform choice
  // among TM*TN static ones; the register inside the tile's 16 is picked by a dynamic vector
  // index, which stays in registers for a 16-element vector.
  auto accumulator_fault = [&]() {
    const bool product = fkind == FI_SITE_PRODUCT;
    float re = 0.0f, re_err = 0.0f;
    bool fired = false;
    if (product)
      product_fault_terms<DT>(p.A[(size_t)frow * p.lda + fk], p.B[(size_t)fcol * p.ldb + fk], fmask,
                              p.product_check, re, re_err, fired);
    uint32_t before = 0, after = 0;
    static_for<TM * TN>([&](auto tt) {
      constexpr int i = tt / TN, j = tt % TN;
      if (tt == sel_t) {
        f32x16 t = acc[i][j];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const bool here = v == sel_v;                       // uniform
          const uint32_t w = __float_as_uint(t[v]);
          const uint32_t nw = product ? __float_as_uint(write_back(t[v], re, re_err)) : (w ^ fmask);
          before = here ? w : before;
          after = here ? nw : after;
          t[v] = __uint_as_float((here && lane == sel_lane) ? nw : w);
        }
        acc[i][j] = t;
      }
    });
    if (lane == sel_lane) {
      p.results[trial].site_word_before = before;
      p.results[trial].site_word_after = after;
      if (fired) p.results[trial].product_flag = 1;
    }
    // Leave nothing of this rare path in flight: the compiler places its waits statically, and
    // memory traffic pending here would make every iteration of the main loop wait for it.
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  };

  const int nkt = (p.K + kshift + BK - 1) / BK;
  issue_tile(0, 0);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  fix_tile(0, 0);
  __syncthreads();

  // One barrier per k-tile, placed before the last of the four MFMA steps (the wave already
  // holds that step's fragments); every fragment read is issued inside the MFMA burst of the step
  // before the one that uses it, the next tile's first read inside the last burst.
  Frags f0, f1;
  read_frags(f0, smem, 0);
  for (int kt = 0; kt < nkt; ++kt) {
    const int stage = kt & 1;
    const bool more = kt + 1 < nkt;
    if (more) issue_tile(kt + 1, stage ^ 1);
    const uint8_t* s = smem + stage * STAGE;
    const uint8_t* s_other = smem + (stage ^ 1) * STAGE;
    __builtin_amdgcn_sched_barrier(0);
    mma_step(f0, [&]() { read_frags(f1, s, 1); });
    __builtin_amdgcn_sched_barrier(0);
    mma_step(f1, [&]() { read_frags(f0, s, 2); });
    __builtin_amdgcn_sched_barrier(0);
    mma_step(f0, [&]() { read_frags(f1, s, 3); });
    __builtin_amdgcn_sched_barrier(0);
    if (more) {
      __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's loads have landed
      fix_tile(kt + 1, stage ^ 1);
    }
    __syncthreads();
    mma_step(f1, [&]() { if (more) read_frags(f0, s_other, 0); });
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (MODE == MODE_CAMPAIGN || MODE == MODE_AFFECTED) {
      if (kt == hook_kt) accumulator_fault();   // one wave of one workgroup per trial
    }
  }

  // ---- epilogue 1: detector, corrector, optional store (every tile of every trial).
  // Each 32x32 accumulator tile is copied out of the accumulator file once, as a whole vector.
  const int row_base = m0 + wm * WTM + 4 * lhi;       // + 32*i + 8*q + e
  const int col_base = n0 + wn * WTN + l32;           // + 32*j
  if constexpr (MODE == MODE_GOLDEN) {
    static_for<TM * TN>([&](auto tt) {
      constexpr int i = tt / TN, j = tt % TN;
      const f32x16 t = acc[i][j];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = row_base + 32 * i + 8 * (v >> 2) + (v & 3), col = col_base + 32 * j;
        if (row < p.M && col < p.N) p.c_out[(size_t)row * p.N + col] = t[v];
      }
    });
    return;
  } else {
    uint32_t n_flag = 0;                                 // wave-uniform: popcounts of lane masks
    float* cout = p.c_out ? p.c_out + (size_t)trial * (size_t)p.M * (size_t)p.N : nullptr;
    fi_trial_result* r = p.results + trial;
    uint32_t n_bit = 0, n_pre = 0, n_post = 0, n_bT = 0, n_btau = 0;
    float mx_pre = 0.0f, mx_post = 0.0f;
    static_for<TM * TN>([&](auto tt) {
      {
        constexpr int i = tt / TN, j = tt % TN;
        f32x16 t = acc[i][j];
        const int col = col_base + 32 * j;
        const float cbj = p.cb[col];
        // Elements outside the problem (clamped staging rows made them copies of the last row)
        // get T = +Inf and the value 0: never flagged, stored or counted.
        f32x16 T;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 kra4 = *reinterpret_cast<const f32x4*>(p.kra + row_base + 32 * i + 8 * q);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const bool inb = row_base + 32 * i + 8 * q + e < p.M && col < p.N;
            const float th = p.bound_global ? p.t_global : __fmul_rn(__fmul_rn(kra4[e], cbj), p.gamma);
            T[4 * q + e] = inb ? th : __builtin_inff();
            t[4 * q + e] = inb ? t[4 * q + e] : 0.0f;
          }
        }
        // one compare and one scalar OR per element; exact counts only where some flag is set
        uint64_t any = 0;
#pragma unroll
        for (int v = 0; v < 16; ++v) any |= __ballot(!(fabsf(t[v]) <= T[v]));
        if (any != 0) {
#pragma unroll
          for (int v = 0; v < 16; ++v) n_flag += (uint32_t)__builtin_popcountll(__ballot(!(fabsf(t[v]) <= T[v])));
        }
        if (cout) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int row = row_base + 32 * i + 8 * (v >> 2) + (v & 3);
            float cc = t[v];
            if (!(fabsf(cc) <= T[v])) {
              if (p.policy == FI_CORRECT_ZERO) cc = 0.0f;
              else if (p.policy == FI_CORRECT_RECOMPUTE) cc = p.c_star[(size_t)row * p.N + col];
            }
            if (row < p.M && col < p.N) cout[(size_t)row * p.N + col] = cc;
          }
        }
        // ---- epilogue 2: deviation from the fault-free result, only where a fault can reach
        if (affected) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int row = row_base + 32 * i + 8 * (v >> 2) + (v & 3);
            // Only what the fault can reach differs from the fault-free result: the element
            // itself, or its output row (A fault) / column (B fault).
            const bool reach = MODE == MODE_PROPAGATE ||
                               ((fkind == FI_SITE_B || row == (int)frow) && (fkind == FI_SITE_A || col == (int)fcol));
            if (row < p.M && col < p.N && reach) {
              const float c = t[v];
              const size_t idx = (size_t)row * p.N + col;
              const float cs = p.c_star[idx];
              const float tau = p.s_abs[idx] * 0.000244140625f;   // 2^-12, exact scaling
              const bool flag = !(fabsf(c) <= T[v]);
              float cc = c;
              if (flag && p.policy == FI_CORRECT_ZERO) cc = 0.0f;
              if (flag && p.policy == FI_CORRECT_RECOMPUTE) cc = cs;
              const float dpre = finite_or_inf(fabsf(c - cs));
              const float dpost = finite_or_inf(fabsf(cc - cs));
              const bool changed = __float_as_uint(c) != __float_as_uint(cs);
              n_bit += changed ? 1u : 0u;
              n_pre += !(dpre <= tau) ? 1u : 0u;
              n_post += !(dpost <= tau) ? 1u : 0u;
              mx_pre = fmaxf(mx_pre, dpre);
              mx_post = fmaxf(mx_post, dpost);
              const float band = fmaxf(2.0f * tau, T[v] * 0.015625f);
              const float mag = fabsf(c);
              n_bT += (changed && mag <= 3.4028234e38f && fabsf(mag - T[v]) <= band) ? 1u : 0u;
              n_btau += (changed && tau > 0.0f && dpre >= 0.5f * tau && dpre <= 2.0f * tau) ? 1u : 0u;
            }
          }
        }
      }
    });
    if (n_flag != 0 && lane == 0) atomicAdd(&r->n_flagged, n_flag);
    if (affected) {
      uint32_t sum;
      sum = wave_sum(n_bit);  if (lane == 0 && sum) atomicAdd(&r->n_bitdiff, sum);
      sum = wave_sum(n_pre);  if (lane == 0 && sum) atomicAdd(&r->n_dev_pre, sum);
      sum = wave_sum(n_post); if (lane == 0 && sum) atomicAdd(&r->n_dev_post, sum);
      sum = wave_sum(n_bT);   if (lane == 0 && sum) atomicAdd(&r->n_border_T, sum);
      sum = wave_sum(n_btau); if (lane == 0 && sum) atomicAdd(&r->n_border_tau, sum);
      // non-negative floats (and +Inf) order like their words
      sum = wave_max(__float_as_uint(mx_pre));
      if (lane == 0 && sum) atomicMax(reinterpret_cast<uint32_t*>(&r->max_dev_pre), sum);
      sum = wave_max(__float_as_uint(mx_post));
      if (lane == 0 && sum) atomicMax(reinterpret_cast<uint32_t*>(&r->max_dev_post), sum);
    }
  }
}

}  // namespace fi
