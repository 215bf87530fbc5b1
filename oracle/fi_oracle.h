/*
 * CPU oracle for fault-injected mixed-precision GEMM campaigns.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct
 * statement of what one campaign computes.  Only the tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it; the product library never
 * does, and the two share no code, headers, tables or helpers.
 *
 * What is modelled (paper sections in parentheses):
 *   - operands in FP16 (1/5/10) or BF16 (1/8/7), decoded exactly   (Sec. II-A, Fig. 1)
 *   - D = A x B with FP32 accumulation of low-precision products    (Sec. II-B, Sec. IV-C)
 *   - one fault per trial: a 1/2/4-bit XOR mask                      (Sec. IV-A, Sec. IV-C)
 *     applied to the FP32 accumulator word of one output element
 *     after k-block s, or to one 16-bit operand word for the whole
 *     trial
 *   - an output-side magnitude-bound detector that generalises the
 *     per-product range argument e_m <= e_1+e_2+1 to a K-term sum,
 *     with correction only when detection fires                     (Sec. VI-A, Sec. VI-B)
 *   - outcome per trial: masked / SDC / detected                     (Sec. I, Sec. V-B)
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py
 * against closed forms, the paper's Table IV, worked flips, invariants and an
 * independent step-by-step NumPy float32 reference.  The masked/SDC/detected
 * *rates* on the synthetic workloads have no published value: parity unpinned
 * for the rates (they are compared GPU-vs-oracle only).
 */
#ifndef FI_ORACLE_H
#define FI_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_FP16 = 0, ORC_BF16 = 1 };
enum { ORC_SITE_NONE = 0, ORC_SITE_ACC = 1, ORC_SITE_A = 2, ORC_SITE_B = 3, ORC_SITE_PRODUCT = 4 };
enum { ORC_CORRECT_NONE = 0, ORC_CORRECT_ZERO = 1, ORC_CORRECT_RECOMPUTE = 2 };
enum { ORC_BOUND_ROWCOL = 0, ORC_BOUND_GLOBAL = 1,
       /* Sec. VI-A bound check read on a binary32 output word: exponent 1eeexxxx with a 1 among
        * eee, i.e. |value| >= 2^17 (or Inf / NaN); needs no operand statistics. */
       ORC_BOUND_EXPONENT = 2 };
enum { ORC_MASKED = 0, ORC_SDC = 1, ORC_DETECTED = 2 };
enum { ORC_MODE_FULL = 0, ORC_MODE_AFFECTED = 1 };
/* Exponent-only checks of an erroneous product (Sec. VI-A). */
enum { ORC_PCHECK_NONE = 0, ORC_PCHECK_BOUND = 1, ORC_PCHECK_RANGE_MAX = 2, ORC_PCHECK_RANGE_FLIP = 3 };
enum { ORC_KIND_ALL_ACC = 0, ORC_KIND_ALL_A = 1, ORC_KIND_ALL_B = 2, ORC_KIND_MIX_ACC_A = 3,
       ORC_KIND_ALL_PRODUCT = 4 };

/* Problem: A is M x K (row i at A + i*lda, K contiguous).  B is K x N
 * mathematically; b_layout 0 stores it as N rows of K (b_kj at B[j*ldb+k]),
 * b_layout 1 as K rows of N (b_kj at B[k*ldb+j]).  All 16-bit words. */
typedef struct {
  int M, N, K, kb;      /* kb = k-block size, K % kb == 0 */
  int fmt;              /* ORC_FP16 / ORC_BF16 */
  int b_layout;
  int bound_mode;
  float gamma;          /* slack factor on the bound, >= 1 */
  long lda, ldb;        /* leading dimensions in elements */
  int product_check;    /* ORC_PCHECK_*: applied to the erroneous product of a PRODUCT fault */
} orc_problem;

/* One fault.  ACC: (row=i, col=j, kblock=s, 32-bit mask).
 * A: (row=i, col=k, low 16 bits of mask).  B: (row=k, col=j, low 16 bits).
 * PRODUCT (the paper's own model, Sec. III-E, Sec. IV-A): (row=i, col=j,
 * kblock=k, low 16 bits of mask): the product a_ik*b_kj, held in the operand
 * format, has its word XORed; after the 16-term MMA step containing k the
 * destination is rewritten as (re_sum - re) + re_err in binary32. */
typedef struct {
  uint32_t kind, row, col, kblock, xor_mask;
} orc_fault;

/* Per-trial record (the oracle's own layout). */
typedef struct {
  double   max_dev_pre;       /* max |c^f - C*| over affected elements, +Inf for NaN/Inf */
  double   max_dev_post;      /* same after correction */
  uint32_t n_flagged;         /* elements with !(|c^f| <= T) */
  uint32_t n_bitdiff;         /* elements whose word differs from C* */
  uint32_t n_dev_pre;         /* elements with !(|c^f - C*| <= tau) */
  uint32_t n_dev_post;        /* same on the corrected output */
  uint32_t site_word_before;  /* ACC: accumulator word at the injection point; A/B: operand word */
  uint32_t site_word_after;
  uint32_t n_border_T;        /* affected elements inside the guard band around T */
  uint32_t n_border_tau;      /* affected elements inside the guard band around tau */
  uint32_t valid;             /* 0: site out of range, trial ran fault-free */
  uint32_t cls;               /* ORC_MASKED / ORC_SDC / ORC_DETECTED */
  uint32_t product_flag;      /* PRODUCT fault: 1 if the exponent-only check fired */
  uint32_t reserved;
} orc_record;

/* Sec. V-B's analysis of numeric deviations (Fig. 7) and Fig. 9: log2-binned histogram of a
 * per-trial deviation, from which the empirical CDF follows by a running sum.
 *   which 0: |re'_sum - re_sum|, the change of the destination register, computed in binary32
 *            from the two site words (accumulator and product-term faults only);
 *   which 1: the trial's largest output deviation before correction, 2: after correction
 *            (rounded to binary32).
 * bin = biased exponent field of that binary32 value: 0 for zero (and subnormal), b for
 * [2^(b-127), 2^(b-126)), 255 for Inf or NaN.  Trials with an invalid site are skipped. */
enum { ORC_HIST_SITE = 0, ORC_HIST_DEV_PRE = 1, ORC_HIST_DEV_POST = 2 };
void orc_deviation_histogram(const orc_record* recs, const orc_fault* faults, int n, int which,
                             uint64_t hist[256]);

/* O1: exact value of a 16-bit pattern, held in a float. */
float orc_decode16(uint16_t w, int fmt);

/* binary32 -> FP16 / BF16 word, round to nearest even (the format a product is held in,
 * Sec. IV-C, Sec. VI-A). */
uint16_t orc_round16(float x, int fmt);

/* Sec. VI-A: exponent-only detection and correction of an erroneous product word w_err given
 * the two operand words.  Returns the corrected word (w_err itself when nothing fires or mode
 * is NONE); *fired = 1 if the detection criterion was violated.  BoundCheck is defined for
 * BF16 only (the paper's Table IV) and never fires for FP16. */
uint16_t orc_product_check(uint16_t w_err, uint16_t w_a, uint16_t w_b, int fmt, int mode, int* fired);
void  orc_decode_array(const uint16_t* in, size_t n, int fmt, float* out);

/* O2: blocked FP32 dot product of row i of A and column j of B, no fault. */
float orc_dot(const orc_problem* p, const uint16_t* A, const uint16_t* B, int i, int j);

/* O2 over the whole matrix.  C is M x N row-major.  R and S (nullable) get
 * the double-precision sum and sum of magnitudes of the products. */
int orc_gemm(const orc_problem* p, const uint16_t* A, const uint16_t* B,
             float* C, double* R, double* S);

/* O4 statistics: ra[i] = max_k |a_ik|, cb[j] = max_k |b_kj|.
 * Returns nonzero if an operand is Inf/NaN. */
int orc_rowcol_absmax(const orc_problem* p, const uint16_t* A, const uint16_t* B,
                      float* ra, float* cb);

/* O4 default slack factor: 1 + 2^-11 * ceil(K / 4096). */
float orc_default_gamma(int K);
/* O4 threshold: fl32(fl32(fl32(K*ra)*cb)*gamma). */
float orc_threshold(int K, float ra, float cb, float gamma);

/* O4+O5 on a materialised batch of outputs, in place.  c_star is needed for
 * RECOMPUTE only.  flags (nullable) is [batch][M][N] bytes; n_flagged [batch]. */
int orc_detect_correct(const orc_problem* p, const float* ra, const float* cb,
                       float* C, int batch, int policy, const float* c_star,
                       uint8_t* flags, uint32_t* n_flagged);

/* O3-O6 for one trial.  mode FULL recomputes every output element with the
 * fault in place and compares all of them; mode AFFECTED recomputes only the
 * element / row / column a fault can reach.  cf_out / cc_out (nullable, FULL
 * only) receive the faulty and the corrected M x N outputs. */
int orc_trial(const orc_problem* p, const uint16_t* A, const uint16_t* B,
              const orc_fault* f, int policy, int mode,
              float* cf_out, float* cc_out, orc_record* rec);

/* A whole campaign; trials are independent. */
int orc_campaign(const orc_problem* p, const uint16_t* A, const uint16_t* B,
                 const orc_fault* faults, int n_trials, int policy, int mode,
                 orc_record* recs);

/* Hand-over between two layers: h = RNE_fmt(relu(c)), relu keeping NaN and mapping negatives
 * and -0 to +0 (Sec. I: from the resilience of one GEMM to that of what is computed from it). */
uint16_t orc_activation_round_one(float c, int fmt);
void orc_activation_round(const float* c, size_t n, int fmt, uint16_t* h);

/* The next layer's GEMM with a per-trial A operand (trial t reads A_stack + t*trial_stride,
 * leading dimension p->lda) and no fault of its own; records compare every output element
 * with C* = A x B.  cc_out (nullable) is [n_trials][M][N].  mode: ORC_MODE_FULL recomputes
 * every element, ORC_MODE_AFFECTED only the rows whose operand words differ from A's. */
int orc_propagate(const orc_problem* p, const uint16_t* A, const uint16_t* B,
                  const uint16_t* A_stack, size_t trial_stride, int n_trials, int policy,
                  int mode, float* cc_out, orc_record* recs);

/* O6 classification totals: counts[0..2] = masked, sdc, detected. */
void orc_classify(const orc_record* recs, int n, uint8_t* cls, uint64_t counts[3]);

/* O7 sampler. */
uint64_t orc_splitmix64_next(uint64_t* state);
int orc_sample_faults(uint64_t seed, uint32_t first_trial, uint32_t n_trials,
                      const orc_problem* p, int kind_mode, int nbits, orc_fault* out);

/* Number of threads the row-parallel loops use (1 without OpenMP). */
int orc_threads(void);

#ifdef __cplusplus
}
#endif
#endif
