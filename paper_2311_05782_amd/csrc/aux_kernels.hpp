// Small kernels around the fault-injecting GEMM: plan statistics, the
// standalone detector / corrector, classification, fills and a transpose.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fi.h"
#include "gemm_fi.hpp"

namespace fi {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// Clears counters and records.  A kernel rather than a memset so that callers
// may capture the library's calls into a HIP graph.
__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t step = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += step) p[i] = v;
}

// out[r] = scale * max_k |x_rk| for the rows of a K-contiguous 16-bit matrix:
// the operand magnitude maxima behind the detector's bound (Sec. VI-A: the
// result's magnitude is bounded by the operands').  Magnitudes of finite
// FP16/BF16 numbers order like their low 15 bits.  One wave per row.
template <int DT>
__global__ void __launch_bounds__(256) row_absmax_kernel(const uint16_t* __restrict__ X, int rows,
                                                        int K, uint32_t ld, float scale,
                                                        float* __restrict__ out,
                                                        uint32_t* __restrict__ nonfinite) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const uint16_t* x = X + (size_t)row * ld;
  uint32_t m = 0;
  for (int c = lane; c < K / 8; c += 64) {
    u32x4_t v = *reinterpret_cast<const u32x4_t*>(x + c * 8);
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      uint32_t lo = v[d] & 0x7FFFu, hi = (v[d] >> 16) & 0x7FFFu;
      m = lo > m ? lo : m;
      m = hi > m ? hi : m;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    uint32_t w = __shfl_xor(m, o, 64);
    m = w > m ? w : m;
  }
  if (lane == 0) {
    const uint32_t first_nonfinite = (DT == FI_BF16) ? 0x7F80u : 0x7C00u;
    if (m >= first_nonfinite) atomicOr(nonfinite, 1u);
    out[row] = __fmul_rn(scale, decode16<DT>(m));
  }
}

// out[0] = max(v[0..n)) for non-negative floats; one workgroup.
__global__ void __launch_bounds__(1024) max_reduce_kernel(const float* __restrict__ v, int n,
                                                         float* __restrict__ out) {
  __shared__ uint32_t part[16];
  uint32_t m = 0;
  for (int i = threadIdx.x; i < n; i += 1024) {
    uint32_t w = __float_as_uint(v[i]);
    m = w > m ? w : m;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    uint32_t w = __shfl_xor(m, o, 64);
    m = w > m ? w : m;
  }
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int i = 1; i < 16; ++i) m = part[i] > m ? part[i] : m;
    out[0] = __uint_as_float(m);
  }
}

// out = |in| for FP16/BF16 words (clear the sign bits), 8 words per thread; `in` has rows of
// ld_in elements of which the first K are copied, `out` is packed [rows][K].  Used once per plan
// to build the operands of the magnitude-sum GEMM behind the tolerance.
__global__ void __launch_bounds__(256) abs16_kernel(const uint16_t* __restrict__ in, uint32_t ld_in,
                                                   uint16_t* __restrict__ out, int rows, int K) {
  const size_t per_row = (size_t)K / 8, total = per_row * (size_t)rows;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t step = (size_t)gridDim.x * 256;
  for (; i < total; i += step) {
    const size_t r = i / per_row, c = i % per_row;
    u32x4_t v = *reinterpret_cast<const u32x4_t*>(in + r * ld_in + c * 8);
    v &= 0x7FFF7FFFu;
    *reinterpret_cast<u32x4_t*>(out + r * (size_t)K + c * 8) = v;
  }
}

// [K][N] -> [N][K] for 16-bit words.
__global__ void __launch_bounds__(256) transpose16_kernel(const uint16_t* __restrict__ in, uint32_t ld_in,
                                                         uint16_t* __restrict__ out, uint32_t ld_out,
                                                         int K, int N) {
  __shared__ uint16_t t[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  const int k0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
  for (int r = ty; r < 32; r += 8) {
    int k = k0 + r, n = n0 + tx;
    t[r][tx] = (k < K && n < N) ? in[(size_t)k * ld_in + n] : (uint16_t)0;
  }
  __syncthreads();
  for (int r = ty; r < 32; r += 8) {
    int n = n0 + r, k = k0 + tx;
    if (n < N && k < K) out[(size_t)n * ld_out + k] = t[tx][r];
  }
}

// Detector and corrector on materialised outputs (Sec. VI-A detection,
// Sec. VI-B correction only where detection fired).  HBM-bound: 4 bytes read per element,
// writes only where a flag is set (plus 1 flag byte per element if asked for).
// The threshold is built with the same three roundings as the fused epilogue:
// fl32(fl32(kra_i * cb_j) * gamma).
//
// VEC == 4 (N % 4 == 0, 16-byte aligned): grid = (row slices, batch); a workgroup walks rows
// blockIdx.x, + gridDim.x, ...; per row each thread takes groups of four 16-byte column chunks,
// issuing the four loads before it looks at any of them (64 bytes in flight per lane), with
// the column maxima read as 16-byte vectors too.  No division in the loop.
// VEC == 1: one element per thread, any N and alignment.
template <int VEC>
__global__ void __launch_bounds__(256) detect_correct_kernel(
    float* __restrict__ C, int M, int N, const float* __restrict__ kra, const float* __restrict__ cb,
    float gamma, int bound_global, float t_global, int policy, const float* __restrict__ c_star,
    uint8_t* __restrict__ flags, uint32_t* __restrict__ n_flagged) {
  const size_t mn = (size_t)M * N;
  float* c = C + (size_t)blockIdx.y * mn;
  uint8_t* fl = flags ? flags + (size_t)blockIdx.y * mn : nullptr;
  uint32_t cnt = 0;
  if constexpr (VEC == 4) {
    const int nv = N / 4;                                   // 16-byte chunks per row
    for (int row = blockIdx.x; row < M; row += gridDim.x) {
      const float kr = kra[row];
      float* crow = c + (size_t)row * N;
      const float* srow = c_star ? c_star + (size_t)row * N : nullptr;
      for (int base = 0; base < nv; base += 4 * 256) {
        f32x4_t v[4], w[4];
        int cv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          cv[u] = base + u * 256 + (int)threadIdx.x;
          if (cv[u] < nv) {
            v[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(crow + 4 * cv[u]));   // streamed once
            w[u] = *reinterpret_cast<const f32x4_t*>(cb + 4 * cv[u]);
          }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (cv[u] < nv) {
            uint32_t fbits = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float T = bound_global ? t_global : __fmul_rn(__fmul_rn(kr, w[u][e]), gamma);
              const bool f = !(fabsf(v[u][e]) <= T);
              fbits |= (f ? 1u : 0u) << (8 * e);
            }
            if (fbits) {                                    // rare: correct element by element
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                if ((fbits >> (8 * e)) & 1u) {
                  cnt += 1;
                  if (policy == FI_CORRECT_ZERO) crow[4 * cv[u] + e] = 0.0f;
                  else if (policy == FI_CORRECT_RECOMPUTE) crow[4 * cv[u] + e] = srow[4 * cv[u] + e];
                }
              }
            }
            if (fl) *reinterpret_cast<uint32_t*>(fl + (size_t)row * N + 4 * cv[u]) = fbits;
          }
        }
      }
    }
  } else {
    for (size_t e0 = (size_t)blockIdx.x * 256 + threadIdx.x; e0 < mn; e0 += (size_t)gridDim.x * 256) {
      const int row = (int)(e0 / (size_t)N), col = (int)(e0 % (size_t)N);
      const float T = bound_global ? t_global : __fmul_rn(__fmul_rn(kra[row], cb[col]), gamma);
      const bool f = !(fabsf(c[e0]) <= T);
      if (f) {
        cnt += 1;
        if (policy == FI_CORRECT_ZERO) c[e0] = 0.0f;
        else if (policy == FI_CORRECT_RECOMPUTE) c[e0] = c_star[e0];
      }
      if (fl) fl[e0] = f ? 1 : 0;
    }
  }
  if (n_flagged && __ballot(cnt != 0)) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
    if ((threadIdx.x & 63) == 0 && cnt) atomicAdd(n_flagged + blockIdx.y, cnt);
  }
}

// Hand-over between two layers: h = RNE_fmt(relu(c)).  relu keeps a NaN and maps negatives
// and -0 to +0; the rounding is the integer one of round16 (no dependence on the wave's float
// modes), in its branch-free form relu_round16.  HBM bound: 4 bytes read, 2 written per element;
// eight elements per lane and step (two 16-byte loads in flight, one 16-byte store).
template <int DT>
__global__ void __launch_bounds__(256) activation_round_kernel(const float* __restrict__ c, size_t n,
                                                              uint16_t* __restrict__ h) {
  const size_t n8 = n / 8;
  const size_t step = (size_t)gridDim.x * 256;
  const size_t first = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (size_t i = first; i < n8; i += step) {
    // streamed once: loads and the store bypass cache retention
    const f32x4_t v0 = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(c) + 2 * i);
    const f32x4_t v1 = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(c) + 2 * i + 1);
    uint32_t w[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float x = v0[e], y = v1[e];
      w[e] = relu_round16<DT>(x);
      w[4 + e] = relu_round16<DT>(y);
    }
    u32x4_t o;
    o[0] = w[0] | (w[1] << 16);
    o[1] = w[2] | (w[3] << 16);
    o[2] = w[4] | (w[5] << 16);
    o[3] = w[6] | (w[7] << 16);
    __builtin_nontemporal_store(o, reinterpret_cast<u32x4_t*>(h) + i);
  }
  for (size_t i = n8 * 8 + first; i < n; i += step) {
    const float x = c[i];
    h[i] = (uint16_t)relu_round16<DT>(x);
  }
}

// dst[r][0 .. shift) = 0, dst[r][shift + k] = src[r][k]: an operand padded IN FRONT to whole
// 64-wide k-tiles.  Leading zero products leave an accumulator that starts at +0 at +0 exactly,
// and the real terms keep their grouping into 16-wide MFMA steps (shift is a multiple of 16),
// so a GEMM over the padded operands equals the unpadded one bit for bit.
__global__ void __launch_bounds__(256) pad_front16_kernel(const uint16_t* __restrict__ src, uint32_t ld,
                                                          uint16_t* __restrict__ dst, uint32_t rows, uint32_t K,
                                                          uint32_t shift) {
  const uint32_t Kp = K + shift;
  const size_t n = (size_t)rows * Kp;
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n; e += (size_t)gridDim.x * 256) {
    const size_t r = e / Kp;
    const uint32_t c = (uint32_t)(e % Kp);
    dst[e] = c < shift ? (uint16_t)0 : src[r * ld + (c - shift)];
  }
}

// Splits a batch: trials the multi-trial GEMM kernel can take (no fault, an accumulator flip or
// a product-term fault; out-of-range sites count as "no fault" and get status 1 in their zeroed
// record) go to the front of perm in list order, all others (operand faults) behind them,
// ordered by the tile row (A) or tile column (B) of a bm x bn tiling that their fault reaches.
// counts = {front, back}.  For front position q, desc[6q .. 6q+5] = {trial, row, col, event,
// w0, w1}: event = -1 for no fault, else the 16-wide MFMA step after which the accumulator
// changes - (s+1)*kb/16 - 1 for a flip with w0 = the XOR mask; k/16, with bit 30 set, for a
// product-term fault with w0, w1 = the words of re and re_err (Sec. III-E).  desc is padded
// with fault-free entries up to the next multiple of 8 positions.  The operand faults' descriptors
// follow from that position on: event = k/16 with bit 29 set, w0 = the 16-bit mask, w1 = kind;
// their site words (the operand word before and after) are written here.  B is [N][ldb], k contiguous.
// kshift: zeros the GEMM kernel's operand copies carry in front of every row (K not a multiple of
// 64): every event step moves up by kshift / 16; A, B, K here are the caller's unpadded operands.
// One workgroup.
template <int DT>
__global__ void __launch_bounds__(1024) partition_trials_kernel(const fi_fault* __restrict__ f, uint32_t n,
                                                               uint32_t M, uint32_t N, uint32_t K, uint32_t kb,
                                                               const uint16_t* __restrict__ A,
                                                               const uint16_t* __restrict__ B, uint32_t lda,
                                                               uint32_t ldb, int product_check_mode,
                                                               uint32_t bm, uint32_t bn, uint32_t kshift,
                                                               uint32_t* __restrict__ perm,
                                                               uint32_t* __restrict__ counts,
                                                               uint32_t* __restrict__ desc,
                                                               fi_trial_result* __restrict__ results) {
  __shared__ uint32_t total_fast;
  // Operand faults are ordered by the tile row (A) or tile column (B) their fault reaches, so
  // that the R trials of a group mostly share it: the other tiles' work items then carry no
  // event at all.  1024 buckets; more tile rows + columns than that are merged pairwise.
  __shared__ uint32_t bucket[1024];
  const uint32_t tiles_m = (M + bm - 1) / bm, n_keys = tiles_m + (N + bn - 1) / bn;
  uint32_t key_shift = 0;
  while (((n_keys - 1u) >> key_shift) >= 1024u) ++key_shift;
  const uint32_t n_major = ((n_keys - 1u) >> key_shift) + 1u;            // <= 1024
  // Inside a tile row / column the trials are ordered by the 64-wide k-tile of the faulted word
  // (as finely as the buckets left over allow): the R trials of a group then have their events
  // in the same k-tile or in neighbouring ones, and a work item runs one or two k-tiles of the
  // checking copy of the loop instead of up to R.
  const uint32_t n_kt = (K + kshift + 63) / 64;          // k-tiles of the (front-padded) operands
  const uint32_t kq = max(1u, min(n_kt, 1024u / n_major));               // keys < n_major * kq <= 1024
  auto key_of = [&](const fi_fault& x) -> uint32_t {
    const uint32_t major = (x.kind == FI_SITE_A ? x.row / bm : tiles_m + x.col / bn) >> key_shift;
    const uint32_t kt = min(((x.kind == FI_SITE_A ? x.col : x.row) + kshift) / 64u, n_kt - 1u);
    return major * kq + kt * kq / n_kt;
  };
  bucket[threadIdx.x] = 0;
  __syncthreads();
  const uint32_t chunk = (n + 1023) / 1024;
  const uint32_t lo = min(threadIdx.x * chunk, n), hi = min(lo + chunk, n);
  // 0: operand fault (other kernel); 1: runs fault-free; 2: accumulator flip; 3: bad site;
  // 4: product-term fault
  auto kind_of = [&](const fi_fault& x) -> int {
    if (x.kind == FI_SITE_ACC) return (x.row < M && x.col < N && x.kblock < K / kb) ? 2 : 3;
    if (x.kind == FI_SITE_PRODUCT) return (x.row < M && x.col < N && x.kblock < K) ? 4 : 3;
    if (x.kind == FI_SITE_A) return (x.row < M && x.col < K) ? 0 : 3;
    if (x.kind == FI_SITE_B) return (x.row < K && x.col < N) ? 0 : 3;
    return x.kind == FI_SITE_NONE ? 1 : 3;
  };
  // Batches of up to 8 x 1024 trials: step i of thread tid looks at trial i * 1024 + tid, so a
  // wave reads 64 consecutive fault records and writes the descriptors of consecutive positions
  // (a thread walking a contiguous chunk of its own made every access of a wave touch 64
  // different cache lines: 40 us for 8192 trials, most of it this one CU's memory pipeline).  The
  // records are read once, all loads in flight together, and kept in registers for both passes.
  // Positions in the first part follow list order: a table of counts per (step, wave), scanned
  // once, plus the lane's rank among the wave's fast trials of that step.  Longer batches: each
  // thread walks a contiguous chunk, reading it in place.
  constexpr int kLocal = 8;
  const bool local = n <= (uint32_t)kLocal * 1024u;
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  __shared__ uint32_t tab[kLocal * 16];
  fi_fault loc[kLocal];
  uint32_t wa[kLocal], wb[kLocal];          // operand words the second pass needs
  unsigned long long fast_mask[kLocal];     // the wave's fast trials of step i
  uint32_t c = 0;                           // long batches: fast trials in my chunk
  auto operand_words = [&](const fi_fault& x, int k, uint32_t& w0, uint32_t& w1) {
    w0 = 0; w1 = 0;
    if (k == 0) w0 = x.kind == FI_SITE_A ? A[(size_t)x.row * lda + x.col] : B[(size_t)x.col * ldb + x.row];
    if (k == 4) { w0 = A[(size_t)x.row * lda + x.kblock]; w1 = B[(size_t)x.col * ldb + x.kblock]; }
  };
  if (local) {
#pragma unroll
    for (int i = 0; i < kLocal; ++i) {
      const uint32_t t = (uint32_t)i * 1024u + threadIdx.x;
      fi_fault x;
      x.kind = 0xFFFFFFFFu; x.row = 0; x.col = 0; x.kblock = 0; x.xor_mask = 0;
      if (t < n) x = f[t];
      loc[i] = x;
    }
#pragma unroll
    for (int i = 0; i < kLocal; ++i) {
      const bool valid = (uint32_t)i * 1024u + threadIdx.x < n;
      const int k = valid ? kind_of(loc[i]) : 3;
      wa[i] = 0; wb[i] = 0;
      if (valid) operand_words(loc[i], k, wa[i], wb[i]);
      fast_mask[i] = __ballot(valid && k != 0);
      if (lane == 0) tab[i * 16 + wave] = (uint32_t)__builtin_popcountll(fast_mask[i]);
      if (valid && k == 0) atomicAdd(&bucket[key_of(loc[i])], 1u);
    }
  } else {
    for (uint32_t t = lo; t < hi; ++t) {
      const fi_fault x = f[t];
      if (kind_of(x) != 0) c += 1u;
      else atomicAdd(&bucket[key_of(x)], 1u);
    }
  }
  __syncthreads();
  // exclusive prefix sums of the buckets and of the per-thread counts, one entry per thread:
  // a shuffle scan inside each wave, then one wave scans the 16 wave totals (three barriers)
  uint32_t pf = 0;                                       // long batches: fast trials before my chunk
  {
    __shared__ uint32_t wave_tot[16], wave_tot_c[16];
    auto wave_scan = [&](uint32_t v) -> uint32_t {       // inclusive
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t u = __shfl_up(v, o, 64);
        v += lane >= (uint32_t)o ? u : 0u;
      }
      return v;
    };
    const uint32_t own = bucket[threadIdx.x], own_c = c;
    uint32_t incl = wave_scan(own), incl_c = wave_scan(own_c);
    if (lane == 63u) { wave_tot[wave] = incl; wave_tot_c[wave] = incl_c; }
    __syncthreads();
    if (wave == 0) {
      const uint32_t v = lane < 16u ? wave_tot[lane] : 0u, vc = lane < 16u ? wave_tot_c[lane] : 0u;
      const uint32_t sc = wave_scan(v), scc = wave_scan(vc);
      if (lane < 16u) { wave_tot[lane] = sc - v; wave_tot_c[lane] = scc - vc; }
      uint32_t total = scc;                              // long batches: read at lane 15
      if (local) {
        // the (step, wave) table in list order, two entries per lane
        static_assert(kLocal * 16 == 128, "two table entries per lane");
        const uint32_t a = tab[2 * lane], b = tab[2 * lane + 1];
        const uint32_t st = wave_scan(a + b);
        tab[2 * lane] = st - (a + b);
        tab[2 * lane + 1] = st - b;
        total = __shfl(st, 63, 64);
      }
      if (lane == 15u) {
        total_fast = total;
        counts[0] = total;
        counts[1] = n - total;
      }
    }
    __syncthreads();
    bucket[threadIdx.x] = incl - own + wave_tot[wave];
    pf = incl_c - own_c + wave_tot_c[wave];
    __syncthreads();
  }
  const uint32_t n_fast = total_fast;
  // x: the fault of trial t; w0, w1: the operand words it needs (an operand fault: the faulted
  // word; a product-term fault: a_ik and b_kj); q: its position if it belongs to the first part
  auto place_one = [&](uint32_t t, const fi_fault& x, uint32_t w0, uint32_t w1, uint32_t q) {
    const int k = kind_of(x);
    if (k == 0) {
      // operand fault: second part of the batch; its descriptors start at the next multiple of 8
      const bool isA = x.kind == FI_SITE_A;
      const uint32_t kk = isA ? x.col : x.row, m16 = x.xor_mask & 0xFFFFu;
      const uint32_t pos = atomicAdd(&bucket[key_of(x)], 1u);      // order inside a bucket is arbitrary
      uint32_t* d = desc + ((size_t)((n_fast + 7u) & ~7u) + pos) * 6;
      d[0] = t; d[1] = x.row; d[2] = x.col; d[3] = ((kk + kshift) / 16) | 0x20000000u; d[4] = m16; d[5] = x.kind;
      results[t].site_word_before = w0;
      results[t].site_word_after = w0 ^ m16;
      perm[n_fast + pos] = t;
      return;
    }
    uint32_t* d = desc + (size_t)q * 6;
    d[0] = t; d[1] = x.row; d[2] = x.col;
    if (k == 2) {
      d[3] = ((x.kblock + 1) * kb + kshift) / 16 - 1; d[4] = x.xor_mask; d[5] = 0;
    } else if (k == 4) {
      float re, re_err;
      bool fired;
      product_fault_terms<DT>((uint16_t)w0, (uint16_t)w1, x.xor_mask, product_check_mode, re, re_err, fired);
      if (fired) results[t].product_flag = 1;
      d[3] = ((x.kblock + kshift) / 16) | 0x40000000u; d[4] = __float_as_uint(re); d[5] = __float_as_uint(re_err);
    } else {
      d[3] = 0xFFFFFFFFu; d[4] = 0; d[5] = 0;
    }
    if (k == 3) results[t].status = 1;
    perm[q] = t;
  };
  if (local) {
    const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
    for (int i = 0; i < kLocal; ++i) {
      const uint32_t t = (uint32_t)i * 1024u + threadIdx.x;
      if (t < n)
        place_one(t, loc[i], wa[i], wb[i], tab[i * 16 + wave] + (uint32_t)__builtin_popcountll(fast_mask[i] & below));
    }
  } else {
    for (uint32_t t = lo; t < hi; ++t) {
      const fi_fault x = f[t];
      const int k = kind_of(x);
      uint32_t w0, w1;
      operand_words(x, k, w0, w1);
      place_one(t, x, w0, w1, pf);
      if (k != 0) ++pf;
    }
  }
  if (threadIdx.x < 16) {
    // fault-free padding behind each part, up to the next multiple of 8 positions
    const uint32_t base2 = (n_fast + 7u) & ~7u, n_slow = n - n_fast;
    const uint32_t q = threadIdx.x < 8 ? n_fast + threadIdx.x : base2 + n_slow + (threadIdx.x - 8);
    const uint32_t end = threadIdx.x < 8 ? base2 : base2 + ((n_slow + 7u) & ~7u);
    if (q < end) {
      uint32_t* d = desc + (size_t)q * 6;
      d[0] = 0; d[1] = 0; d[2] = 0; d[3] = 0xFFFFFFFFu; d[4] = 0; d[5] = 0;
    }
  }
}

// Log2-binned histogram of a per-trial deviation (Sec. V-B, Fig. 7 / Fig. 9): the bin is the
// exponent field of the binary32 value.  One workgroup, counts gathered in LDS.
__global__ void __launch_bounds__(1024) deviation_histogram_kernel(const fi_fault* __restrict__ f,
                                                                  const fi_trial_result* __restrict__ r,
                                                                  uint32_t n, int which,
                                                                  unsigned long long* __restrict__ hist) {
  __shared__ uint32_t bins[256];
  if (threadIdx.x < 256) bins[threadIdx.x] = 0;
  __syncthreads();
  for (uint32_t t = threadIdx.x; t < n; t += 1024) {
    const fi_trial_result x = r[t];
    if (x.status != 0) continue;
    float d;
    if (which == FI_HIST_SITE) {
      const uint32_t kind = f[t].kind;
      if (kind != FI_SITE_ACC && kind != FI_SITE_PRODUCT) continue;
      d = __fsub_rn(__uint_as_float(x.site_word_after), __uint_as_float(x.site_word_before));
    } else {
      d = which == FI_HIST_DEV_PRE ? x.max_dev_pre : x.max_dev_post;
    }
    atomicAdd(&bins[(__float_as_uint(d) >> 23) & 0xFFu], 1u);
  }
  __syncthreads();
  if (threadIdx.x < 256) hist[threadIdx.x] = bins[threadIdx.x];
}

// Measurement aid: what the matrix cores sustain when a wave does nothing but issue MFMAs, in the
// campaign kernel's occupancy (8 waves per workgroup, one workgroup per CU, 128 accumulator
// registers per lane).  Each wave holds eight 32 x 32 accumulators and two sets of operand
// fragments that alternate from step to step (so operand bits toggle as they do when fragments
// arrive from LDS); random_data = 0 fills them with 1.0, else with seeded values in [-2, 2).
// The part lowers its clock under matrix load depending on the data, so this - not the nominal
// peak - is what a GEMM kernel on such data can approach.  Workgroup 0 records the counters
// described at GemmArgs::clocks.  sink keeps the result alive.
template <int DT>
__global__ void __launch_bounds__(512, 2) mfma_loop_probe_kernel(int random_data, int iters, float* __restrict__ sink,
                                                                unsigned long long* __restrict__ clocks) {
  const int tid = threadIdx.x;
  if (clocks && blockIdx.x == 0 && tid == 0) {
    clocks[0] = __builtin_readcyclecounter();
    clocks[1] = __builtin_amdgcn_s_memrealtime();
  }
  u32x4 fa[2][2], fb[2][4];
  const uint32_t one = DT == FI_BF16 ? 0x3F803F80u : 0x3C003C00u;
  uint32_t h = (uint32_t)(blockIdx.x * 512 + tid) * 2654435761u + 12345u;
  auto word = [&]() -> uint32_t {
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13; h *= 3266489917u; h ^= h >> 16;
    // two 16-bit values with random sign and mantissa, exponent of 1.0: magnitudes in [1, 2)
    const uint32_t keep = DT == FI_BF16 ? 0x807F807Fu : 0x83FF83FFu;
    return random_data ? ((h & keep) | one) : one;
  };
#pragma unroll
  for (int s = 0; s < 2; ++s) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int w = 0; w < 4; ++w) fa[s][i][w] = word();
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int w = 0; w < 4; ++w) fb[s][j][w] = word();
  }
  f32x16 acc[2][4];
  static_for<8>([&](auto t) {
    acc[t / 4][t % 4] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  });
  for (int it = 0; it < iters; ++it) {
    static_for<2>([&](auto ss) {
      constexpr int s = ss;
      static_for<8>([&](auto t) {
        constexpr int i = t / 4, j = t % 4;
        acc[i][j] = mfma_32x32x16<DT>(fa[s][i], fb[s][j], acc[i][j]);
      });
      __builtin_amdgcn_sched_barrier(0);
    });
  }
  float x = 0.0f;
  static_for<8>([&](auto t) {
#pragma unroll
    for (int v = 0; v < 16; ++v) x += acc[t / 4][t % 4][v];
  });
  sink[(size_t)blockIdx.x * 512 + tid] = x;
  if (clocks && blockIdx.x == 0 && tid == 0) {
    clocks[2] = __builtin_readcyclecounter();
    clocks[3] = __builtin_amdgcn_s_memrealtime();
  }
}

// Outcome per trial and campaign totals, one workgroup, no atomics:
// DETECTED if anything was flagged, else SDC if anything deviates beyond the
// tolerance, else MASKED.
__global__ void __launch_bounds__(1024) classify_kernel(const fi_trial_result* __restrict__ r, uint32_t n,
                                                       uint8_t* __restrict__ cls,
                                                       uint64_t* __restrict__ counts) {
  __shared__ uint32_t part[3][16];
  uint32_t c0 = 0, c1 = 0, c2 = 0;
  for (uint32_t t = threadIdx.x; t < n; t += 1024) {
    uint32_t k = r[t].n_flagged > 0 ? FI_DETECTED : (r[t].n_dev_pre > 0 ? FI_SDC : FI_MASKED);
    if (cls) cls[t] = (uint8_t)k;
    c0 += (k == FI_MASKED); c1 += (k == FI_SDC); c2 += (k == FI_DETECTED);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    c0 += __shfl_xor(c0, o, 64); c1 += __shfl_xor(c1, o, 64); c2 += __shfl_xor(c2, o, 64);
  }
  if ((threadIdx.x & 63) == 0) {
    part[0][threadIdx.x >> 6] = c0; part[1][threadIdx.x >> 6] = c1; part[2][threadIdx.x >> 6] = c2;
  }
  __syncthreads();
  if (threadIdx.x < 3) {
    uint64_t s = 0;
    for (int i = 0; i < 16; ++i) s += part[threadIdx.x][i];
    counts[threadIdx.x] = s;
  }
}

}  // namespace fi
