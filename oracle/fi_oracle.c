/*
 * CPU oracle for fault-injected mixed-precision GEMM campaigns.
 * TEST INFRASTRUCTURE: see fi_oracle.h.  Build with
 *   gcc -O2 -std=c99 -ffp-contract=off -fno-fast-math [-fopenmp] -shared -fPIC
 * No intrinsics, no blocking beyond the k-blocks the method itself defines, no
 * reordering: every loop is the definition written out.
 */
#include "fi_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ words */

static uint32_t word_of(float x) { uint32_t w; memcpy(&w, &x, 4); return w; }
static float float_of(uint32_t w) { float x; memcpy(&x, &w, 4); return x; }

/* ------------------------------------------------- O1: operand decoding
 * Sec. II-A / Fig. 1: FP16 = 1 sign, 5 exponent (bias 15), 10 mantissa bits;
 * BF16 = 1 sign, 8 exponent (bias 127), 7 mantissa bits.  Value of a normal
 * number: (-1)^s * 2^(E-bias) * (1 + m/2^p); of a subnormal (E = 0):
 * (-1)^s * 2^(1-bias) * (m/2^p).  Both formats embed exactly in binary32, so
 * ldexpf of a small integer is exact, subnormal binary32 results included. */
float orc_decode16(uint16_t w, int fmt) {
  int ebits = (fmt == ORC_FP16) ? 5 : 8;
  int mbits = (fmt == ORC_FP16) ? 10 : 7;
  int bias = (1 << (ebits - 1)) - 1;
  int sign = (w >> 15) & 1;
  int E = (w >> mbits) & ((1 << ebits) - 1);
  int m = w & ((1 << mbits) - 1);
  float v;
  if (E == (1 << ebits) - 1) {
    v = (m == 0) ? INFINITY : NAN;
  } else if (E == 0) {
    v = ldexpf((float)m, 1 - bias - mbits);
  } else {
    v = ldexpf((float)((1 << mbits) + m), E - bias - mbits);
  }
  return sign ? -v : v;
}

/* Memo of the pure function above over all 65536 patterns per format. */
static float g_tab[2][65536];
__attribute__((constructor)) static void fill_tables(void) {
  for (int fmt = 0; fmt < 2; ++fmt)
    for (uint32_t w = 0; w < 65536; ++w) g_tab[fmt][w] = orc_decode16((uint16_t)w, fmt);
}
static float dec(uint16_t w, int fmt) { return g_tab[fmt][w]; }

void orc_decode_array(const uint16_t* in, size_t n, int fmt, float* out) {
  for (size_t t = 0; t < n; ++t) out[t] = orc_decode16(in[t], fmt);
}

/* ------------------------------------------------------------ accessors */

static uint16_t a_word(const orc_problem* p, const uint16_t* A, int i, int k) {
  return A[(size_t)i * (size_t)p->lda + (size_t)k];
}
static uint16_t b_word(const orc_problem* p, const uint16_t* B, int k, int j) {
  return p->b_layout == 0 ? B[(size_t)j * (size_t)p->ldb + (size_t)k]
                          : B[(size_t)k * (size_t)p->ldb + (size_t)j];
}

static int check_problem(const orc_problem* p) {
  if (!p) return 1;
  if (p->M <= 0 || p->N <= 0 || p->K <= 0 || p->kb <= 0) return 1;
  if (p->K % p->kb != 0) return 1;
  if (p->fmt != ORC_FP16 && p->fmt != ORC_BF16) return 1;
  if (p->b_layout != 0 && p->b_layout != 1) return 1;
  if (!(p->gamma >= 1.0f)) return 1;
  return 0;
}

/* Row i of A and column j of B as contiguous float vectors of length K. */
static void load_a_row(const orc_problem* p, const uint16_t* A, int i, float* out) {
  for (int k = 0; k < p->K; ++k) out[k] = dec(a_word(p, A, i, k), p->fmt);
}
static void load_b_col(const orc_problem* p, const uint16_t* B, int j, float* out) {
  for (int k = 0; k < p->K; ++k) out[k] = dec(b_word(p, B, k, j), p->fmt);
}

/* ------------------------------------ binary32 -> FP16 / BF16, nearest-even
 * The paper's fault corrupts what one multiplication produces (Sec. IV-C)
 * and its detectors read the register holding that BF16 product (Sec. VI-A):
 * the product is held in the operand format.  This is the IEEE round-to-nearest-even conversion written out case
 * by case: NaN, overflow to infinity at the midpoint above the largest finite
 * value, the subnormal range as a fixed-point grid, normal numbers as
 * exponent + rounded significand (a carry out of the significand bumps the
 * exponent). */
uint16_t orc_round16(float x, int fmt) {
  uint32_t w32 = word_of(x);
  uint16_t sign = (uint16_t)((w32 >> 16) & 0x8000u);
  float ax = fabsf(x);
  if (fmt == ORC_BF16) {
    /* 8 exponent bits as binary32: keep the top 16 bits, round on the 16 dropped ones. */
    if (isnan(x)) return (uint16_t)(sign | 0x7FC0u);
    uint32_t mag = w32 & 0x7FFFFFFFu;
    uint32_t keep = mag >> 16, drop = mag & 0xFFFFu;
    if (drop > 0x8000u || (drop == 0x8000u && (keep & 1u))) keep += 1;   /* may carry up to Inf */
    return (uint16_t)(sign | keep);
  }
  /* FP16: 5 exponent bits (bias 15), 10 fraction bits. */
  if (isnan(x)) return (uint16_t)(sign | 0x7E00u);
  if (ax >= 65520.0f) return (uint16_t)(sign | 0x7C00u);       /* halfway to 65536 ties to even = Inf */
  if (ax < 0x1p-14f) {
    /* subnormal grid: multiples of 2^-24; scaling by 2^24 is exact */
    float q = rintf(ax * 0x1p24f);                                /* ties to even */
    return (uint16_t)(sign | (uint16_t)q);                        /* q == 1024 is the smallest normal */
  }
  int e2;
  float m = frexpf(ax, &e2);                                      /* ax = m * 2^e2, m in [0.5, 1) */
  int e = e2 - 1;                                                 /* ax = (2m) * 2^e, 2m in [1, 2) */
  float frac = rintf((2.0f * m - 1.0f) * 1024.0f);                /* exact scaling, ties to even */
  int q = (int)frac;
  if (q == 1024) { q = 0; e += 1; }
  return (uint16_t)(sign | (uint16_t)((e + 15) << 10) | (uint16_t)q);
}

/* ------------------------ Sec. VI-A: exponent-only checks of a product
 * They read only the exponent field of the register holding the (possibly
 * corrupted) product.
 *   Bound check (BF16): with the exponent's most significant bit set, a 1 in any
 *     of the next three bits (1eeexxxx) means |value| >= 2^17 = 131072 (the
 *     paper's Table IV) - not a plausible partial weight/activation product.
 *     Correction: clear those three bits.
 *   Range check: m1*m2 < 4 gives e_m <= e_1 + e_2 + 1; with biased fields
 *     be_m <= be_1 + be_2 - bias + 1 (not below 0: products that underflow have
 *     field 0).  A larger erroneous exponent is detected.  Correction "max":
 *     replace it by the bound; "flip": clear its 1 bits starting from the
 *     rightmost until it no longer exceeds the bound. */
uint16_t orc_product_check(uint16_t w_err, uint16_t w_a, uint16_t w_b, int fmt, int mode, int* fired) {
  int mb = fmt == ORC_BF16 ? 7 : 10, eb = fmt == ORC_BF16 ? 8 : 5, bias = fmt == ORC_BF16 ? 127 : 15;
  unsigned emask = (1u << eb) - 1u;
  unsigned e = ((unsigned)w_err >> mb) & emask;
  int hit = 0;
  if (mode == ORC_PCHECK_BOUND) {
    if (fmt == ORC_BF16 && (e & 0x80u) && (e & 0x70u)) {
      hit = 1;
      e &= ~0x70u;
    }
  } else if (mode == ORC_PCHECK_RANGE_MAX || mode == ORC_PCHECK_RANGE_FLIP) {
    int e1 = (int)(((unsigned)w_a >> mb) & emask), e2 = (int)(((unsigned)w_b >> mb) & emask);
    int bound = e1 + e2 - bias + 1;
    if (bound < 0) bound = 0;
    if ((int)e > bound) {
      hit = 1;
      if (mode == ORC_PCHECK_RANGE_MAX) {
        e = (unsigned)bound;
      } else {
        for (int bit = 0; bit < eb && (int)e > bound; ++bit)
          if ((e >> bit) & 1u) e &= ~(1u << bit);
      }
    }
  }
  if (fired) *fired = hit;
  return (uint16_t)(((unsigned)w_err & ~(emask << mb)) | (e << mb));
}

/* --------------------------------- O2 / O3: blocked FP32 dot product
 * Sec. IV-C: low-precision products accumulated into one FP32 number.
 * acc starts at +0; k ascends; each product is rounded once to binary32
 * (exact for FP16 and, inside the binary32 range, for BF16), each addition is
 * rounded once, no fused multiply-add.
 *
 * Accumulator fault (acc_s >= 0): the accumulator word is XORed with acc_mask
 * immediately after the last addition of k-block acc_s (Sec. III-E: the
 * corrupted value lands in the MMA destination register and the following
 * MMAs accumulate onto it).
 *
 * Product-term fault (prod_k >= 0), the paper's own model (Sec. III-E "write-
 * back", Eq. 1-2; Sec. IV-A: a term of one MMA instruction, 16 terms for FP16
 * and BF16): the MMA step is the group of 16 consecutive k holding prod_k.
 * After its last addition the destination holds re_sum.  re = the product
 * a*b rounded to the operand format, re_err = the same 16-bit word XOR
 * prod_mask; then re' = re_sum - re and re'_sum = re' + re_err, each rounded
 * once in binary32, replace the destination. */
typedef struct {
  int acc_s;  uint32_t acc_mask;
  int prod_k; uint32_t prod_mask; int fmt;
  int check;          /* ORC_PCHECK_*: exponent-only check applied to re_err (Sec. VI-A) */
  uint32_t* fired;    /* where to note that it fired, or NULL */
} elem_fault;
static const elem_fault NO_FAULT = {-1, 0, -1, 0, 0, 0, NULL};

static float dot_blocked(const float* a, const float* b, int K, int kb, elem_fault ef,
                         uint32_t* word_before, uint32_t* word_after) {
  float acc = 0.0f;
  int S = K / kb;
  int step_last = ef.prod_k >= 0 ? (ef.prod_k / 16) * 16 + 15 : -1;
  for (int s = 0; s < S; ++s) {
    for (int k = s * kb; k < (s + 1) * kb; ++k) {
      float prod = a[k] * b[k];
      acc = acc + prod;
      if (k == step_last) {
        float exact = a[ef.prod_k] * b[ef.prod_k];
        uint16_t w = orc_round16(exact, ef.fmt);
        float re = dec(w, ef.fmt);
        uint16_t w_err = (uint16_t)(w ^ (ef.prod_mask & 0xFFFFu));
        if (ef.check != ORC_PCHECK_NONE) {
          /* the operand words: decoded operands convert back exactly */
          int hit = 0;
          w_err = orc_product_check(w_err, orc_round16(a[ef.prod_k], ef.fmt), orc_round16(b[ef.prod_k], ef.fmt),
                                    ef.fmt, ef.check, &hit);
          if (ef.fired) *ef.fired = (uint32_t)hit;
        }
        float re_err = dec(w_err, ef.fmt);
        if (word_before) *word_before = word_of(acc);
        float re_prime = acc - re;
        acc = re_prime + re_err;
        if (word_after) *word_after = word_of(acc);
      }
    }
    if (s == ef.acc_s) {
      uint32_t w = word_of(acc);
      if (word_before) *word_before = w;
      w ^= ef.acc_mask;
      if (word_after) *word_after = w;
      acc = float_of(w);
    }
  }
  return acc;
}

/* Double-precision sum R and sum of magnitudes Sabs of the same products. */
static void dot_double(const float* a, const float* b, int K, double* R, double* Sabs) {
  double r = 0.0, s = 0.0;
  for (int k = 0; k < K; ++k) {
    double prod = (double)a[k] * (double)b[k];
    r += prod;
    s += fabs(prod);
  }
  *R = r;
  *Sabs = s;
}

float orc_dot(const orc_problem* p, const uint16_t* A, const uint16_t* B, int i, int j) {
  float* a = (float*)malloc(sizeof(float) * (size_t)p->K);
  float* b = (float*)malloc(sizeof(float) * (size_t)p->K);
  load_a_row(p, A, i, a);
  load_b_col(p, B, j, b);
  float c = dot_blocked(a, b, p->K, p->kb, NO_FAULT, NULL, NULL);
  free(a);
  free(b);
  return c;
}

int orc_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Whole-matrix O2 with an optional fault ef in element (fi, fj).
 * Af is M x K, Bt is N x K (column j of B stored as row j), both decoded. */
static void gemm_decoded(int M, int N, int K, int kb, const float* Af, const float* Bt,
                         int fi, int fj, elem_fault ef,
                         float* C, double* R, double* S,
                         uint32_t* word_before, uint32_t* word_after) {
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
  for (int i = 0; i < M; ++i) {
    for (int j = 0; j < N; ++j) {
      const float* a = Af + (size_t)i * K;
      const float* b = Bt + (size_t)j * K;
      int here = (i == fi && j == fj);
      C[(size_t)i * N + j] = dot_blocked(a, b, K, kb, here ? ef : NO_FAULT,
                                         here ? word_before : NULL, here ? word_after : NULL);
      if (R || S) {
        double r, s;
        dot_double(a, b, K, &r, &s);
        if (R) R[(size_t)i * N + j] = r;
        if (S) S[(size_t)i * N + j] = s;
      }
    }
  }
}

static int decode_operands(const orc_problem* p, const uint16_t* A, const uint16_t* B,
                           float** Af, float** Bt) {
  *Af = (float*)malloc(sizeof(float) * (size_t)p->M * p->K);
  *Bt = (float*)malloc(sizeof(float) * (size_t)p->N * p->K);
  if (!*Af || !*Bt) { free(*Af); free(*Bt); return 3; }
  for (int i = 0; i < p->M; ++i) load_a_row(p, A, i, *Af + (size_t)i * p->K);
  for (int j = 0; j < p->N; ++j) load_b_col(p, B, j, *Bt + (size_t)j * p->K);
  return 0;
}

int orc_gemm(const orc_problem* p, const uint16_t* A, const uint16_t* B,
             float* C, double* R, double* S) {
  if (check_problem(p) || !A || !B || !C) return 1;
  float *Af, *Bt;
  int rc = decode_operands(p, A, B, &Af, &Bt);
  if (rc) return rc;
  gemm_decoded(p->M, p->N, p->K, p->kb, Af, Bt, -1, -1, NO_FAULT, C, R, S, NULL, NULL);
  free(Af);
  free(Bt);
  return 0;
}

/* ---------------------------------------------------- O4: the detector
 * Sec. VI-A bounds the exponent of ONE product by the operands' exponents
 * (m1*m2 < 4  =>  e_m <= e1+e2+1).  Summed over the K products of an output
 * element the same argument gives |c_ij| <= K * max_k|a_ik| * max_k|b_kj|;
 * anything above that (times a rounding slack gamma) cannot be a fault-free
 * result.  Magnitudes are compared on the 15 value bits, which orders finite
 * FP16/BF16 numbers exactly. */
int orc_rowcol_absmax(const orc_problem* p, const uint16_t* A, const uint16_t* B,
                      float* ra, float* cb) {
  if (check_problem(p) || !A || !B || !ra || !cb) return 1;
  int bad = 0;
  for (int i = 0; i < p->M; ++i) {
    float m = 0.0f;
    for (int k = 0; k < p->K; ++k) {
      float v = fabsf(dec(a_word(p, A, i, k), p->fmt));
      if (!(v <= 3.0e38f)) bad = 1;   /* Inf or NaN */
      if (v > m) m = v;
    }
    ra[i] = m;
  }
  for (int j = 0; j < p->N; ++j) {
    float m = 0.0f;
    for (int k = 0; k < p->K; ++k) {
      float v = fabsf(dec(b_word(p, B, k, j), p->fmt));
      if (!(v <= 3.0e38f)) bad = 1;
      if (v > m) m = v;
    }
    cb[j] = m;
  }
  return bad ? 2 : 0;
}

/* Default slack factor.  With exact products (two 16-bit operands multiply exactly in
 * binary32) the K - 1 rounded additions of any summation order inflate a sum of magnitudes by
 * at most (1 + 2^-24)^(K-1), about 1 + K * 2^-24, and the three roundings of the threshold
 * itself lose at most three ulps.  gamma = 1 + 2^-11 * ceil(K / 4096) is at least 1 + 2 K 2^-24:
 * twice what is needed, so a fault-free element is never flagged (for K <= 4096 this is the
 * constant 1 + 2^-11). */
float orc_default_gamma(int K) {
  int units = (K + 4095) / 4096;
  if (units < 1) units = 1;
  return 1.0f + (float)units / 2048.0f;
}

float orc_threshold(int K, float ra, float cb, float gamma) {
  float t = (float)K * ra;   /* one rounding each */
  t = t * cb;
  t = t * gamma;
  return t;
}

static float vec_max(const float* v, int n) {
  float m = 0.0f;
  for (int t = 0; t < n; ++t) if (v[t] > m) m = v[t];
  return m;
}

static float threshold_at(const orc_problem* p, const float* ra, const float* cb,
                          float ra_max, float cb_max, int i, int j) {
  if (p->bound_mode == ORC_BOUND_GLOBAL) return orc_threshold(p->K, ra_max, cb_max, p->gamma);
  /* Exponent field >= 128 + 16 <=> |c| >= 2^17 <=> NOT (|c| <= the float just below 2^17). */
  if (p->bound_mode == ORC_BOUND_EXPONENT) return 131071.9921875f;
  return orc_threshold(p->K, ra[i], cb[j], p->gamma);
}

/* flag <=> NOT (|c| <= T): true for NaN and +-Inf as well. */
static int flagged(float c, float T) { return !(fabsf(c) <= T); }

/* O5: correction only where detection fired (Sec. VI-B). */
static float corrected(float c, int flag, int policy, float c_star) {
  if (!flag) return c;
  if (policy == ORC_CORRECT_ZERO) return 0.0f;
  if (policy == ORC_CORRECT_RECOMPUTE) return c_star;
  return c;
}

int orc_detect_correct(const orc_problem* p, const float* ra, const float* cb,
                       float* C, int batch, int policy, const float* c_star,
                       uint8_t* flags, uint32_t* n_flagged) {
  if (check_problem(p) || !ra || !cb || !C || batch < 0) return 1;
  if (policy == ORC_CORRECT_RECOMPUTE && !c_star) return 1;
  float ra_max = vec_max(ra, p->M), cb_max = vec_max(cb, p->N);
  for (int t = 0; t < batch; ++t) {
    uint32_t n = 0;
    for (int i = 0; i < p->M; ++i) {
      for (int j = 0; j < p->N; ++j) {
        size_t e = ((size_t)t * p->M + i) * p->N + j;
        float T = threshold_at(p, ra, cb, ra_max, cb_max, i, j);
        int fl = flagged(C[e], T);
        if (flags) flags[e] = (uint8_t)fl;
        n += (uint32_t)fl;
        C[e] = corrected(C[e], fl, policy, c_star ? c_star[(size_t)i * p->N + j] : 0.0f);
      }
    }
    if (n_flagged) n_flagged[t] = n;
  }
  return 0;
}

/* ------------------------------------------- O6: per-element accounting */

static double deviation(float x, float ref) {
  double d = fabs((double)x - (double)ref);
  if (!(d <= 1.79e308)) return INFINITY;   /* NaN or Inf */
  return d;
}

static void account(orc_record* r, float c_f, float c_star, double Sabs, float T, int policy) {
  double tau = ldexp(Sabs, -12);
  int fl = flagged(c_f, T);
  float c_c = corrected(c_f, fl, policy, c_star);
  double dpre = deviation(c_f, c_star);
  double dpost = deviation(c_c, c_star);
  r->n_flagged += (uint32_t)fl;
  r->n_bitdiff += (uint32_t)(word_of(c_f) != word_of(c_star));
  r->n_dev_pre += (uint32_t)!(dpre <= tau);
  r->n_dev_post += (uint32_t)!(dpost <= tau);
  if (dpre > r->max_dev_pre) r->max_dev_pre = dpre;
  if (dpost > r->max_dev_post) r->max_dev_post = dpost;
  /* Guard bands: decisions that a different (but admissible) FP32 summation
   * order could take the other way.  Only elements the fault changed can be
   * borderline: an unchanged element is C*, which never exceeds T. */
  if (word_of(c_f) == word_of(c_star)) return;
  double band = 2.0 * tau;
  if (ldexp((double)T, -6) > band) band = ldexp((double)T, -6);
  double mag = fabs((double)c_f);
  if (mag <= 1.79e308 && fabs(mag - (double)T) <= band) r->n_border_T += 1;
  if (tau > 0.0 && dpre >= 0.5 * tau && dpre <= 2.0 * tau) r->n_border_tau += 1;
}

static void finish(orc_record* r) {
  if (r->n_flagged > 0) r->cls = ORC_DETECTED;
  else if (r->n_dev_pre > 0) r->cls = ORC_SDC;
  else r->cls = ORC_MASKED;
}

static int site_valid(const orc_problem* p, const orc_fault* f) {
  switch (f->kind) {
    case ORC_SITE_NONE: return 1;
    case ORC_SITE_ACC:
      return f->row < (uint32_t)p->M && f->col < (uint32_t)p->N &&
             f->kblock < (uint32_t)(p->K / p->kb);
    case ORC_SITE_A: return f->row < (uint32_t)p->M && f->col < (uint32_t)p->K;
    case ORC_SITE_B: return f->row < (uint32_t)p->K && f->col < (uint32_t)p->N;
    case ORC_SITE_PRODUCT:
      return f->row < (uint32_t)p->M && f->col < (uint32_t)p->N && f->kblock < (uint32_t)p->K;
    default: return 0;
  }
}

/* The fault of one output element: accumulator flip after k-block `kblock`, or a
 * product-term fault on the product with k = `kblock`. */
static elem_fault element_fault(const orc_problem* p, const orc_fault* f, orc_record* rec) {
  elem_fault ef = NO_FAULT;
  ef.check = p->product_check;
  ef.fired = rec ? &rec->product_flag : NULL;
  if (f->kind == ORC_SITE_ACC) { ef.acc_s = (int)f->kblock; ef.acc_mask = f->xor_mask; }
  if (f->kind == ORC_SITE_PRODUCT) { ef.prod_k = (int)f->kblock; ef.prod_mask = f->xor_mask; ef.fmt = p->fmt; }
  return ef;
}

/* ----------------------------------------------------- O3-O6: one trial */

static int trial_full(const orc_problem* p, const uint16_t* A, const uint16_t* B,
                      const orc_fault* f, int policy, float* cf_out, float* cc_out,
                      orc_record* rec) {
  int M = p->M, N = p->N, K = p->K;
  size_t mn = (size_t)M * N;
  float *Af = NULL, *Bt = NULL;
  int rc = decode_operands(p, A, B, &Af, &Bt);
  if (rc) return rc;
  float* Cstar = (float*)malloc(sizeof(float) * mn);
  float* Cf = (float*)malloc(sizeof(float) * mn);
  double* S = (double*)malloc(sizeof(double) * mn);
  float* ra = (float*)malloc(sizeof(float) * (size_t)M);
  float* cb = (float*)malloc(sizeof(float) * (size_t)N);
  orc_rowcol_absmax(p, A, B, ra, cb);     /* statistics of the GOLDEN operands */
  float ra_max = vec_max(ra, M), cb_max = vec_max(cb, N);

  gemm_decoded(M, N, K, p->kb, Af, Bt, -1, -1, NO_FAULT, Cstar, NULL, S, NULL, NULL);

  /* The faulty execution: every element is recomputed with the fault in place. */
  if (f->kind == ORC_SITE_ACC || f->kind == ORC_SITE_PRODUCT) {
    gemm_decoded(M, N, K, p->kb, Af, Bt, (int)f->row, (int)f->col, element_fault(p, f, rec),
                 Cf, NULL, NULL, &rec->site_word_before, &rec->site_word_after);
  } else if (f->kind == ORC_SITE_A) {
    uint16_t w = a_word(p, A, (int)f->row, (int)f->col);
    uint16_t wf = (uint16_t)(w ^ (f->xor_mask & 0xFFFFu));
    rec->site_word_before = w;
    rec->site_word_after = wf;
    Af[(size_t)f->row * K + f->col] = dec(wf, p->fmt);
    gemm_decoded(M, N, K, p->kb, Af, Bt, -1, -1, NO_FAULT, Cf, NULL, NULL, NULL, NULL);
  } else if (f->kind == ORC_SITE_B) {
    uint16_t w = b_word(p, B, (int)f->row, (int)f->col);
    uint16_t wf = (uint16_t)(w ^ (f->xor_mask & 0xFFFFu));
    rec->site_word_before = w;
    rec->site_word_after = wf;
    Bt[(size_t)f->col * K + f->row] = dec(wf, p->fmt);
    gemm_decoded(M, N, K, p->kb, Af, Bt, -1, -1, NO_FAULT, Cf, NULL, NULL, NULL, NULL);
  } else {
    memcpy(Cf, Cstar, sizeof(float) * mn);
  }

  for (int i = 0; i < M; ++i) {
    for (int j = 0; j < N; ++j) {
      size_t e = (size_t)i * N + j;
      float T = threshold_at(p, ra, cb, ra_max, cb_max, i, j);
      account(rec, Cf[e], Cstar[e], S[e], T, policy);
      if (cf_out) cf_out[e] = Cf[e];
      if (cc_out) cc_out[e] = corrected(Cf[e], flagged(Cf[e], T), policy, Cstar[e]);
    }
  }
  free(Af); free(Bt); free(Cstar); free(Cf); free(S); free(ra); free(cb);
  return 0;
}

/* Only the elements the fault can reach are recomputed; every other element
 * equals C* bit for bit by construction and a clean element is never flagged
 * (|C*_ij| <= T_ij), so it contributes nothing to any counter. */
static int trial_affected(const orc_problem* p, const uint16_t* A, const uint16_t* B,
                          const float* ra, const float* cb, float ra_max, float cb_max,
                          const orc_fault* f, int policy, orc_record* rec) {
  int K = p->K;
  float* a = (float*)malloc(sizeof(float) * (size_t)K);
  float* b = (float*)malloc(sizeof(float) * (size_t)K);
  float* g = (float*)malloc(sizeof(float) * (size_t)K);   /* golden copy of the faulted vector */
  if (f->kind == ORC_SITE_ACC || f->kind == ORC_SITE_PRODUCT) {
    int i = (int)f->row, j = (int)f->col;
    load_a_row(p, A, i, a);
    load_b_col(p, B, j, b);
    float c_star = dot_blocked(a, b, K, p->kb, NO_FAULT, NULL, NULL);
    float c_f = dot_blocked(a, b, K, p->kb, element_fault(p, f, rec),
                            &rec->site_word_before, &rec->site_word_after);
    double R, S;
    dot_double(a, b, K, &R, &S);
    account(rec, c_f, c_star, S, threshold_at(p, ra, cb, ra_max, cb_max, i, j), policy);
  } else if (f->kind == ORC_SITE_A) {
    int i = (int)f->row, kf = (int)f->col;
    uint16_t w = a_word(p, A, i, kf);
    uint16_t wf = (uint16_t)(w ^ (f->xor_mask & 0xFFFFu));
    rec->site_word_before = w;
    rec->site_word_after = wf;
    load_a_row(p, A, i, g);
    memcpy(a, g, sizeof(float) * (size_t)K);
    a[kf] = dec(wf, p->fmt);
    for (int j = 0; j < p->N; ++j) {
      load_b_col(p, B, j, b);
      float c_star = dot_blocked(g, b, K, p->kb, NO_FAULT, NULL, NULL);
      float c_f = dot_blocked(a, b, K, p->kb, NO_FAULT, NULL, NULL);
      double R, S;
      dot_double(g, b, K, &R, &S);
      account(rec, c_f, c_star, S, threshold_at(p, ra, cb, ra_max, cb_max, i, j), policy);
    }
  } else if (f->kind == ORC_SITE_B) {
    int kf = (int)f->row, j = (int)f->col;
    uint16_t w = b_word(p, B, kf, j);
    uint16_t wf = (uint16_t)(w ^ (f->xor_mask & 0xFFFFu));
    rec->site_word_before = w;
    rec->site_word_after = wf;
    load_b_col(p, B, j, g);
    memcpy(b, g, sizeof(float) * (size_t)K);
    b[kf] = dec(wf, p->fmt);
    for (int i = 0; i < p->M; ++i) {
      load_a_row(p, A, i, a);
      float c_star = dot_blocked(a, g, K, p->kb, NO_FAULT, NULL, NULL);
      float c_f = dot_blocked(a, b, K, p->kb, NO_FAULT, NULL, NULL);
      double R, S;
      dot_double(a, g, K, &R, &S);
      account(rec, c_f, c_star, S, threshold_at(p, ra, cb, ra_max, cb_max, i, j), policy);
    }
  }
  free(a); free(b); free(g);
  return 0;
}

static void clear_record(orc_record* rec) {
  memset(rec, 0, sizeof(*rec));
  rec->valid = 1;
}

int orc_trial(const orc_problem* p, const uint16_t* A, const uint16_t* B,
              const orc_fault* f, int policy, int mode,
              float* cf_out, float* cc_out, orc_record* rec) {
  if (check_problem(p) || !A || !B || !f || !rec) return 1;
  if (policy < 0 || policy > 2) return 1;
  clear_record(rec);
  orc_fault nofault = {ORC_SITE_NONE, 0, 0, 0, 0};
  if (!site_valid(p, f)) { rec->valid = 0; f = &nofault; }
  int rc;
  if (mode == ORC_MODE_FULL) {
    rc = trial_full(p, A, B, f, policy, cf_out, cc_out, rec);
  } else {
    if (cf_out || cc_out) return 1;
    float* ra = (float*)malloc(sizeof(float) * (size_t)p->M);
    float* cb = (float*)malloc(sizeof(float) * (size_t)p->N);
    orc_rowcol_absmax(p, A, B, ra, cb);
    rc = trial_affected(p, A, B, ra, cb, vec_max(ra, p->M), vec_max(cb, p->N), f, policy, rec);
    free(ra); free(cb);
  }
  if (rc == 0) finish(rec);
  return rc;
}

int orc_campaign(const orc_problem* p, const uint16_t* A, const uint16_t* B,
                 const orc_fault* faults, int n_trials, int policy, int mode,
                 orc_record* recs) {
  if (check_problem(p) || !A || !B || !faults || !recs || n_trials < 0) return 1;
  if (policy < 0 || policy > 2) return 1;
  if (mode == ORC_MODE_FULL) {
    for (int t = 0; t < n_trials; ++t) {
      int rc = orc_trial(p, A, B, &faults[t], policy, ORC_MODE_FULL, NULL, NULL, &recs[t]);
      if (rc) return rc;
    }
    return 0;
  }
  float* ra = (float*)malloc(sizeof(float) * (size_t)p->M);
  float* cb = (float*)malloc(sizeof(float) * (size_t)p->N);
  orc_rowcol_absmax(p, A, B, ra, cb);
  float ra_max = vec_max(ra, p->M), cb_max = vec_max(cb, p->N);
  orc_fault nofault = {ORC_SITE_NONE, 0, 0, 0, 0};
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 4)
#endif
  for (int t = 0; t < n_trials; ++t) {
    const orc_fault* f = &faults[t];
    clear_record(&recs[t]);
    if (!site_valid(p, f)) { recs[t].valid = 0; f = &nofault; }
    trial_affected(p, A, B, ra, cb, ra_max, cb_max, f, policy, &recs[t]);
    finish(&recs[t]);
  }
  free(ra); free(cb);
  return 0;
}

/* ------------------------------------------- two layers: hand-over and propagation
 * Sec. I asks for the gap between the resilience of one matrix multiplication and of what the
 * application computes from it.  The smallest such application is a second layer: the (possibly
 * faulty, possibly corrected) output of the first GEMM passes a ReLU, is rounded to the operand
 * format and becomes the A operand of the next GEMM. */
uint16_t orc_activation_round_one(float c, int fmt) {
  float r;
  if (isnan(c)) r = c;            /* a NaN stays a NaN */
  else if (c > 0.0f) r = c;
  else r = 0.0f;                  /* negatives and -0 become +0 */
  return orc_round16(r, fmt);
}

void orc_activation_round(const float* c, size_t n, int fmt, uint16_t* h) {
  for (size_t e = 0; e < n; ++e) h[e] = orc_activation_round_one(c[e], fmt);
}

/* Trial t multiplies ITS OWN A operand, A_stack + t * trial_stride (same leading dimension as
 * A), by the plan's B; nothing is injected.  Every output element is compared with the
 * fault-free C* = A x B, passed through the detector / corrector and counted (O4-O6), the
 * statistics and tolerances being those of the GOLDEN operands.  Mode FULL recomputes every
 * element; mode AFFECTED takes the rows whose operand words all equal the golden row's from
 * C* (the same deterministic dot products would reproduce them bit for bit). */
int orc_propagate(const orc_problem* p, const uint16_t* A, const uint16_t* B,
                  const uint16_t* A_stack, size_t trial_stride, int n_trials, int policy,
                  int mode, float* cc_out, orc_record* recs) {
  if (check_problem(p) || !A || !B || !A_stack || !recs || n_trials < 0) return 1;
  if (policy < 0 || policy > 2) return 1;
  int M = p->M, N = p->N, K = p->K;
  size_t mn = (size_t)M * N;
  float *Af = NULL, *Bt = NULL;
  int rc = decode_operands(p, A, B, &Af, &Bt);
  if (rc) return rc;
  float* Cstar = (float*)malloc(sizeof(float) * mn);
  double* S = (double*)malloc(sizeof(double) * mn);
  float* ra = (float*)malloc(sizeof(float) * (size_t)M);
  float* cb = (float*)malloc(sizeof(float) * (size_t)N);
  orc_rowcol_absmax(p, A, B, ra, cb);
  float ra_max = vec_max(ra, M), cb_max = vec_max(cb, N);
  gemm_decoded(M, N, K, p->kb, Af, Bt, -1, -1, NO_FAULT, Cstar, NULL, S, NULL, NULL);
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1)
#endif
  for (int t = 0; t < n_trials; ++t) {
    const uint16_t* At = A_stack + (size_t)t * trial_stride;
    float* a = (float*)malloc(sizeof(float) * (size_t)K);
    orc_record* rec = &recs[t];
    clear_record(rec);
    for (int i = 0; i < M; ++i) {
      int same = 1;
      for (int k = 0; k < K; ++k) {
        uint16_t w = a_word(p, At, i, k);
        if (w != a_word(p, A, i, k)) same = 0;
        a[k] = dec(w, p->fmt);
      }
      for (int j = 0; j < N; ++j) {
        size_t e = (size_t)i * N + j;
        float c_f = (mode == ORC_MODE_AFFECTED && same)
                        ? Cstar[e]
                        : dot_blocked(a, Bt + (size_t)j * K, K, p->kb, NO_FAULT, NULL, NULL);
        float T = threshold_at(p, ra, cb, ra_max, cb_max, i, j);
        account(rec, c_f, Cstar[e], S[e], T, policy);
        if (cc_out) cc_out[(size_t)t * mn + e] = corrected(c_f, flagged(c_f, T), policy, Cstar[e]);
      }
    }
    finish(rec);
    free(a);
  }
  free(Af); free(Bt); free(Cstar); free(S); free(ra); free(cb);
  return 0;
}

void orc_classify(const orc_record* recs, int n, uint8_t* cls, uint64_t counts[3]) {
  counts[0] = counts[1] = counts[2] = 0;
  for (int t = 0; t < n; ++t) {
    uint32_t c;
    if (recs[t].n_flagged > 0) c = ORC_DETECTED;
    else if (recs[t].n_dev_pre > 0) c = ORC_SDC;
    else c = ORC_MASKED;
    if (cls) cls[t] = (uint8_t)c;
    counts[c] += 1;
  }
}

/* ------------------------------------------- deviation histogram (Sec. V-B)
 * 256 log2 bins - the exponent field of the binary32 value - of a per-trial
 * quantity: the change of the destination register (Fig. 7's statistic) or the
 * largest output deviation before / after correction (Fig. 9). */
void orc_deviation_histogram(const orc_record* recs, const orc_fault* faults, int n, int which,
                             uint64_t hist[256]) {
  for (int b = 0; b < 256; ++b) hist[b] = 0;
  for (int t = 0; t < n; ++t) {
    if (!recs[t].valid) continue;
    float d;
    if (which == ORC_HIST_SITE) {
      if (faults[t].kind != ORC_SITE_ACC && faults[t].kind != ORC_SITE_PRODUCT) continue;
      d = fabsf(float_of(recs[t].site_word_after) - float_of(recs[t].site_word_before));
    } else {
      d = (float)(which == ORC_HIST_DEV_PRE ? recs[t].max_dev_pre : recs[t].max_dev_post);
    }
    unsigned bin = (word_of(d) >> 23) & 0xFFu;   /* d >= 0 or NaN: the sign bit is dropped by the mask */
    hist[bin] += 1;
  }
}

/* --------------------------------------------------------- O7: sampler
 * Sec. IV-A picks the injection target uniformly at random and flips one or
 * several random bits of it.  Owning the GEMM, the site space is closed-form:
 * (i, j, s) for an accumulator fault, (i, k) for an A-operand fault, (k, j)
 * for a B-operand fault, times the position of an nbits-wide burst.  Draws
 * come from SplitMix64 (Steele, Lea, Flood 2014) keyed by the trial index so
 * any trial can be regenerated alone. */
uint64_t orc_splitmix64_next(uint64_t* state) {
  *state += 0x9E3779B97F4A7C15ull;
  uint64_t z = *state;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

static uint32_t unif(uint32_t n, uint64_t u) {
  return (uint32_t)(((u >> 32) * (uint64_t)n) >> 32);
}

int orc_sample_faults(uint64_t seed, uint32_t first_trial, uint32_t n_trials,
                      const orc_problem* p, int kind_mode, int nbits, orc_fault* out) {
  if (check_problem(p) || !out) return 1;
  if (kind_mode < 0 || kind_mode > 4) return 1;
  if (nbits < 1 || nbits > 16) return 1;
  uint32_t S = (uint32_t)(p->K / p->kb);
  for (uint32_t n = 0; n < n_trials; ++n) {
    uint64_t t = (uint64_t)first_trial + n;
    uint64_t state = seed + (t << 32);
    uint64_t u0 = orc_splitmix64_next(&state);
    uint64_t u1 = orc_splitmix64_next(&state);
    uint64_t u2 = orc_splitmix64_next(&state);
    uint64_t u3 = orc_splitmix64_next(&state);
    uint32_t kind;
    switch (kind_mode) {
      case ORC_KIND_ALL_ACC: kind = ORC_SITE_ACC; break;
      case ORC_KIND_ALL_A: kind = ORC_SITE_A; break;
      case ORC_KIND_ALL_B: kind = ORC_SITE_B; break;
      case ORC_KIND_ALL_PRODUCT: kind = ORC_SITE_PRODUCT; break;
      default: kind = (t % 2 == 0) ? ORC_SITE_ACC : ORC_SITE_A; break;
    }
    orc_fault f;
    f.kind = kind;
    uint32_t width;
    if (kind == ORC_SITE_ACC) {
      f.row = unif((uint32_t)p->M, u0);
      f.col = unif((uint32_t)p->N, u1);
      f.kblock = unif(S, u2);
      width = 32;
    } else if (kind == ORC_SITE_PRODUCT) {
      /* Sec. IV-A: an MMA instruction, one of its results, one of its 16 terms - uniform
       * over (i, j, k) - and a random bit(s) of the 16-bit product. */
      f.row = unif((uint32_t)p->M, u0);
      f.col = unif((uint32_t)p->N, u1);
      f.kblock = unif((uint32_t)p->K, u2);
      width = 16;
    } else if (kind == ORC_SITE_A) {
      uint32_t s = unif(S, u1), kk = unif((uint32_t)p->kb, u2);
      f.row = unif((uint32_t)p->M, u0);
      f.col = s * (uint32_t)p->kb + kk;
      f.kblock = s;
      width = 16;
    } else {
      uint32_t s = unif(S, u1), kk = unif((uint32_t)p->kb, u2);
      f.col = unif((uint32_t)p->N, u0);
      f.row = s * (uint32_t)p->kb + kk;
      f.kblock = s;
      width = 16;
    }
    uint32_t pos = unif(width - (uint32_t)nbits + 1u, u3);
    f.xor_mask = (uint32_t)(((1ull << nbits) - 1ull) << pos);
    out[n] = f;
  }
  return 0;
}
