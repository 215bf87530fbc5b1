/*
 * fi.h - C ABI of the MI355X (gfx950) fault-injection campaign engine for
 * mixed-precision GEMM.
 *
 * One campaign = many independent trials of the same GEMM C = A x B, FP16 or
 * BF16 operands, FP32 accumulation (paper Sec. II-B, Sec. IV-C).  Each trial
 * carries exactly one fault (Sec. IV-A): an XOR mask of 1, 2 or 4 (any number
 * of) bits applied either to the FP32 accumulator word of one output element
 * right after k-block s - the register the paper's write-back finally
 * overwrites (Sec. III-E) - or to one 16-bit operand word for the whole trial.
 * An output-side detector then flags every element whose magnitude exceeds
 * what K products of the operands could ever sum to - the K-term form of the
 * paper's per-product range argument e_m <= e_1 + e_2 + 1 (Sec. VI-A) - and a
 * corrector acts only where the detector fired (Sec. VI-B).  Each trial is
 * finally classified masked / SDC / detected (Sec. I, Sec. V-B).
 *
 * Conventions
 *   - Every pointer whose name starts with d_ is DEVICE memory on the current
 *     HIP device; h_ is host memory.  The library never allocates memory it
 *     hands to the caller and never frees caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All
 *     device work is enqueued on it.  Three calls allocate device memory and
 *     synchronise, and so must stay outside stream capture: fi_plan_create (it
 *     reads back an operand-validity word), fi_plan_reserve, and
 *     fi_gemm_inject_batch on the FIRST batch a plan sees on a given stream or
 *     on a batch larger than any before on that stream (it sizes that
 *     stream's trial-order scratch; fi_plan_reserve does this ahead of time).
 *     fi_plan_destroy waits for the device.  No other call allocates or
 *     synchronises, so device-side failures surface at the caller's next
 *     synchronising call.
 *   - A plan may have batches in flight on several streams at once (each
 *     stream has its own scratch; at most 64 streams per plan).  Calls on one
 *     plan are not thread-safe: serialise them on the host.
 *   - Every function returns an fi_status; on failure output parameters are
 *     untouched and fi_last_error() describes the problem.  Nothing throws or
 *     aborts across this boundary.
 *   - Bit numbering: bit 0 = least significant bit of the word.  FP32 words:
 *     bits 0..22 mantissa, 23..30 exponent, 31 sign.  FP16: 10 mantissa, 5
 *     exponent bits; BF16: 7 mantissa, 8 exponent bits (Sec. II-A, Fig. 1).
 */
#ifndef FI_H
#define FI_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t fi_status;
enum {
  FI_OK = 0,
  FI_INVALID_ARG = 1,   /* NULL pointer, zero dimension, K % k_block != 0, ... */
  FI_UNSUPPORTED = 2,   /* dtype / alignment / size the kernels do not handle */
  FI_OOM = 3,           /* device allocation failed */
  FI_DEVICE = 4,        /* a HIP call failed; see fi_last_error() */
  FI_STATE = 5          /* no gfx950 device, or a destroyed plan */
};

enum { FI_FP16 = 0, FI_BF16 = 1 };
enum { FI_SITE_NONE = 0, FI_SITE_ACC = 1, FI_SITE_A = 2, FI_SITE_B = 3, FI_SITE_PRODUCT = 4 };
enum { FI_CORRECT_NONE = 0, FI_CORRECT_ZERO = 1, FI_CORRECT_RECOMPUTE = 2 };
enum { FI_BOUND_ROWCOL = 0, FI_BOUND_GLOBAL = 1, FI_BOUND_EXPONENT = 2 };
enum { FI_MASKED = 0, FI_SDC = 1, FI_DETECTED = 2 };
/* Exponent-only checks of the erroneous product of a PRODUCT fault (Sec. VI-A). */
enum { FI_PCHECK_NONE = 0, FI_PCHECK_BOUND = 1, FI_PCHECK_RANGE_MAX = 2, FI_PCHECK_RANGE_FLIP = 3 };
enum { FI_KIND_ALL_ACC = 0, FI_KIND_ALL_A = 1, FI_KIND_ALL_B = 2, FI_KIND_MIX_ACC_A = 3,
       FI_KIND_ALL_PRODUCT = 4 };

/* One fault (Sec. IV-A: one target, a random bit or bits, one fault per trial).
 *   ACC : row = i, col = j, kblock = s; xor_mask applies to the 32-bit
 *         accumulator word of element (i, j) after the last product of
 *         k-block s has been added.
 *   A   : row = i, col = k; the low 16 bits of xor_mask apply to a_ik for
 *         every use in this trial (kblock is ignored).
 *   B   : row = k, col = j; same for b_kj.
 *   PRODUCT : the paper's own fault (Sec. III-E write-back, Eq. 1-2; Sec. IV-A one term of
 *         one 16-term MMA step): row = i, col = j, kblock = k.  re = a_ik * b_kj rounded to
 *         the operand format, re_err = the same 16-bit word XOR the low 16 bits of
 *         xor_mask.  Right after the 16-wide MMA step that holds k, the accumulator of
 *         element (i, j) becomes fl32(fl32(acc - re) + re_err).
 *   NONE: a fault-free trial.
 * A site outside the problem makes the trial run fault-free with
 * fi_trial_result.status = 1. */
typedef struct {
  uint32_t kind, row, col, kblock, xor_mask;
} fi_fault;

/* Per-trial record.  "Affected" elements are those a fault can reach: the element
 * itself (ACC, PRODUCT), its output row (A) or its output column (B); all other
 * elements are bit-identical to the fault-free result.
 *   tau_ij = 2^-12 * sum_k |a_ik * b_kj| is the deviation a trial may show and
 *   still count as masked (Sec. V-B: small mantissa changes are absorbed
 *   during accumulation).  Deviations are taken against the plan's own
 *   fault-free result C*. */
typedef struct {
  uint32_t n_flagged;        /* elements with NOT(|c| <= T_ij), whole output       */
  uint32_t n_bitdiff;        /* affected elements whose word differs from C*        */
  uint32_t n_dev_pre;        /* affected elements with NOT(|c - C*| <= tau_ij)      */
  uint32_t n_dev_post;       /* same, after correction                              */
  float    max_dev_pre;      /* max |c - C*| before correction (+Inf for NaN/Inf)   */
  float    max_dev_post;     /* ... after correction                                */
  uint32_t site_word_before; /* ACC, PRODUCT: accumulator word at the injection     */
  uint32_t site_word_after;  /*   point (Sec. V-B's re_sum, re'_sum); A/B: the operand word */
  uint32_t n_border_T;       /* changed elements within max(2 tau, T/64) of T       */
  uint32_t n_border_tau;     /* changed elements with tau/2 <= |c - C*| <= 2 tau    */
  uint32_t status;           /* 0 ok, 1 site out of range (trial ran fault-free)    */
  uint32_t product_flag;     /* PRODUCT fault: 1 if the exponent-only check fired   */
} fi_trial_result;

/* Problem description.  A is M x K, row i at dA + i*lda (K contiguous).
 * b_layout 0: B is stored as N rows of K (b_kj at dB[j*ldb + k]) - the layout
 * of a linear layer's weight; b_layout 1: K rows of N (b_kj at dB[k*ldb + j]),
 * transposed once into plan-owned memory at plan creation.
 * Requirements: k_block a multiple of 16, K a multiple of k_block, K <= 65536;
 * dA/dB 16-byte aligned and lda/ldb multiples of 8 elements. */
/* gamma: slack factor on the detector's bound, >= 1.  0 selects the default,
 * 1 + 2^-11 * ceil(K / 4096): a K-term FP32 accumulation can exceed the exact sum of
 * magnitudes by (1 + 2^-24)^(K-1), and the three roundings of the bound itself lose three more
 * ulps; the default is about twice that, so a fault-free element is never flagged. */
typedef struct {
  uint32_t M, N, K, k_block;
  uint32_t dtype;        /* FI_FP16 / FI_BF16 */
  uint32_t b_layout;
  uint32_t bound_mode;   /* FI_BOUND_ROWCOL: T_ij = gamma*K*ra_i*cb_j, ra_i = max_k|a_ik|,
                            cb_j = max_k|b_kj|; FI_BOUND_GLOBAL: gamma*K*max ra*max cb;
                            FI_BOUND_EXPONENT: the bound check of Sec. VI-A read on the binary32
                            output word, exponent 1eeexxxx with a 1 among eee, i.e. flag where
                            |c| >= 2^17 (and Inf, NaN); uses no operand statistics or gamma */
  float    gamma;        /* >= 1; 0 selects the default 1 + 2^-11 */
  int64_t  lda, ldb;     /* in elements */
} fi_plan_desc;

typedef struct fi_plan fi_plan;

/* Build a plan for one (A, B): row/column magnitude maxima, the fault-free
 * result C* (Sec. II-B: D = A x B, C_in = 0) and the magnitude sums behind
 * tau.  d_A and d_B must stay alive and unmodified until fi_plan_destroy.
 * The plan owns its scratch (C*, sums, maxima; a transposed copy of B for
 * b_layout 1) and frees it in fi_plan_destroy.
 * Errors: INVALID_ARG (NULLs, zero dims, K % k_block, k_block % 16, gamma < 1,
 * Inf/NaN operand), UNSUPPORTED (dtype, alignment), OOM, DEVICE, STATE. */
fi_status fi_plan_create(const fi_plan_desc* desc, const void* d_A, const void* d_B,
                         void* stream, fi_plan** out);
fi_status fi_plan_destroy(fi_plan* plan);

/* Device pointers to plan-owned arrays, valid until fi_plan_destroy:
 * which 0: C* [M][N] float, 1: sum_k|a_ik b_kj| [M][N] float,
 * 2: fl32(K*ra_i) [M] float, 3: cb_j [N] float. */
fi_status fi_plan_buffer(const fi_plan* plan, uint32_t which, const void** d_ptr);

/* Optional tuning.  tile_config: -1 keep, else an index into the kernel table:
 *   0..2  one trial per work item on a 256x256, 128x128 or 256x64 output tile (every fault
 *         kind, any K).  The first two run as persistent workgroups - the item loop of the
 *         multi-trial kernel below with one trial per item (also reachable as 7 and 8) -
 *         and fi_gemm_propagate_batch uses the same persistent kernel.
 *   3..8  R trials per workgroup sharing one staged operand tile: R=4 on 128x128, R=2 on
 *         128x128, R=8 on 128x64 (the default on large problems), and, with two workgroups of
 *         four waves per compute unit instead of one of eight, R=8 on 64x64 (the default
 *         below 2^35 multiply-adds); 7 and 8: R=1 (see above).  Any K: when K is not a
 *         multiple of 64 the plan keeps copies of A and B with zeros in front of every row
 *         up to whole 64-wide k-tiles (bit-identical results: leading zero products leave
 *         an accumulator at +0).
 *         The batch is split on the device into the trials whose fault leaves the operands
 *         alone and the operand-fault trials; the latter run in a second instantiation that
 *         XORs the faulted word in the fragment registers around the faulted trial's MFMAs.
 * trial_group: -1 keep, else how many trials (groups of R trials) of the same
 * output tile are scheduled next to each other, 1..4096.  Results do not depend on
 * either (every shape accumulates each element in the same order); `stream` is unused. */
fi_status fi_plan_tune(fi_plan* plan, int32_t tile_config, int32_t trial_group, void* stream);

/* Sizes the trial-order scratch `stream` uses for this plan's batches to max_trials, so that
 * fi_gemm_inject_batch with n_trials <= max_trials on that stream neither allocates nor
 * synchronises (a caller about to capture the calls into a HIP graph wants this).
 * Errors: INVALID_ARG (max_trials == 0), OOM, STATE (more than 64 streams). */
fi_status fi_plan_reserve(fi_plan* plan, uint32_t max_trials, void* stream);

/* Exponent-only detection / correction applied to the erroneous product re_err of every
 * PRODUCT fault before the write-back (Sec. VI-A; correction only where detection fires,
 * Sec. VI-B).  It reads the exponent field of the 16-bit product word:
 *   FI_PCHECK_BOUND      BF16 only (never fires for FP16): exponent 1eeexxxx with a 1 among
 *                        eee, i.e. |value| >= 2^17; correction clears those three bits;
 *   FI_PCHECK_RANGE_MAX  exponent field above be_a + be_b - bias + 1 (not below 0): replaced
 *                        by that bound;
 *   FI_PCHECK_RANGE_FLIP same detection; correction clears the field's 1 bits from the
 *                        rightmost until it no longer exceeds the bound.
 * fi_trial_result.product_flag says whether it fired.  Default FI_PCHECK_NONE.
 * INVALID_ARG for an unknown mode. */
fi_status fi_plan_set_product_check(fi_plan* plan, uint32_t mode);

/* Writes a NUL-terminated description of the kernels the plan launches for a
 * campaign (template shape, threads, trials per workgroup) into h_buf (HOST memory,
 * n bytes; truncated to fit).  INVALID_ARG if h_buf is NULL or n == 0. */
fi_status fi_plan_describe(const fi_plan* plan, char* h_buf, uint64_t n);

/* Run n_trials faulty executions of the whole GEMM in one launch, each with
 * its fault from d_faults[t], followed in the same kernel by the detector,
 * the corrector (policy) and the per-trial counters (Sec. IV-A trial,
 * Sec. VI-A/B detect then correct).  d_results[t] is overwritten.
 * d_c_out is NULL or [n_trials][M][N] floats receiving the corrected outputs
 * (policy FI_CORRECT_NONE: the raw faulty outputs).
 * Errors: INVALID_ARG (NULL plan/faults/results, bad policy, n_trials == 0). */
fi_status fi_gemm_inject_batch(fi_plan* plan, const fi_fault* d_faults, uint32_t n_trials,
                               uint32_t policy, fi_trial_result* d_results, float* d_c_out,
                               void* stream);

/* fi_gemm_inject_batch with the hand-over to a next layer fused into its epilogue (Sec. I:
 * what an error in one GEMM does to what is computed from it; Sec. V-B (i): activations zero
 * many values): instead of FP32 outputs it writes d_h_out[t][i][j] = RNE_fmt(relu(c)), c the
 * corrected output (policy FI_CORRECT_NONE: the raw faulty one) - 16-bit words of the plan's
 * operand format, [n_trials][M][N], device memory owned by the caller.  Bit-identical to
 * fi_gemm_inject_batch with d_c_out followed by fi_activation_round, without writing and
 * re-reading 4 bytes per element.  Records as fi_gemm_inject_batch.  Allocation and
 * synchronisation as fi_gemm_inject_batch (per-stream scratch).
 * Errors: INVALID_ARG (NULLs, bad policy, n_trials == 0); UNSUPPORTED when d_h_out is not
 * 2-byte aligned or the plan runs the one-trial kernel
 * (fi_plan_tune(plan, 2, ...)). */
fi_status fi_gemm_inject_batch_act(fi_plan* plan, const fi_fault* d_faults, uint32_t n_trials,
                                   uint32_t policy, fi_trial_result* d_results, void* d_h_out,
                                   void* stream);

/* fi_gemm_inject_batch for callers that cannot allocate device memory or synchronise: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels, same records and outputs; the trial order, the part counts and the
 * per-trial descriptors of the batch live in a static device array of the library (about
 * 460 KB per GPU, held until the process ends) instead of plan-owned buffers, so the call
 * allocates nothing and never synchronises.  Limits: n_trials <= 16384 (FI_UNSUPPORTED beyond);
 * every call on a GPU - whatever the plan or stream - uses that GPU's one array, which is
 * rewritten by each call's partition kernel before it is read, so calls that overlap on one
 * GPU race: order them (one stream, or events).  The array's address is looked up when a plan
 * is created on that GPU.  Errors otherwise as fi_gemm_inject_batch. */
fi_status fi_gemm_inject_batch_noalloc(fi_plan* plan, const fi_fault* d_faults, uint32_t n_trials,
                                       uint32_t policy, fi_trial_result* d_results, float* d_c_out,
                                       void* stream);

/* The same campaign restricted to what a fault can reach: for each trial only the output
 * tiles holding the faulted element (ACC, PRODUCT), its output row (A) or its output column
 * (B) are computed; every other element of a trial equals the fault-free result bit for bit
 * and must not be flagged: the plan counts, when it is created, the elements of the fault-free
 * result its own detector flags (none under FI_BOUND_ROWCOL / FI_BOUND_GLOBAL with gamma at or
 * above the default; possible under FI_BOUND_EXPONENT, where any |C*_ij| >= 2^17 is flagged, or
 * with a smaller gamma), and this call returns FI_UNSUPPORTED if there are any.  d_results[t] then
 * equals the record fi_gemm_inject_batch writes.  This is a different product - trials per second, not
 * matrix-core throughput: a trial costs 2*K (element) to 2*N*K or 2*M*K (row, column) useful
 * flops instead of 2*M*N*K - and its rate is never reported against the MFMA roof.
 * Errors as fi_gemm_inject_batch, and UNSUPPORTED as described above. */
fi_status fi_gemm_inject_batch_affected(fi_plan* plan, const fi_fault* d_faults, uint32_t n_trials,
                                        uint32_t policy, fi_trial_result* d_results, void* stream);

/* Hand-over between two layers (Sec. I: from the resilience of one matrix multiplication to
 * that of what the application computes from it; Sec. V-B (i): zeros are common in
 * activations): d_h[e] = RNE_fmt(relu(d_c[e])) for n elements, as 16-bit words of `dtype`.
 * relu keeps a NaN (handed on as the format's quiet NaN) and maps negatives and -0 to +0;
 * values beyond the format's range round to +Inf.  d_c (device, 16-byte aligned) is not
 * modified; d_h (device, 16-byte aligned) is overwritten.  No plan is needed.
 * Errors: UNSUPPORTED (dtype, alignment), INVALID_ARG (NULLs, n == 0). */
fi_status fi_activation_round(uint32_t dtype, const float* d_c, uint64_t n, uint16_t* d_h, void* stream);

/* The next layer of a two-layer workload: n_trials executions of the plan's GEMM in one launch,
 * trial t with ITS OWN A operand d_a_stack + t * trial_stride (device, 16-bit words, [M][lda]
 * like the plan's A; trial_stride in elements, a multiple of 8, at least (M-1)*lda + K, or 0
 * to give every trial the same operand) and the plan's B; no fault is injected.  Every output
 * element of every trial passes the plan's detector / corrector and is compared with the
 * plan's fault-free result C* = A x B under the plan's tolerance: d_results[t] holds
 * n_flagged, n_bitdiff, n_dev_pre, n_dev_post, the largest deviations and the guard-band
 * counts over the whole output (site words 0).  Rows of a trial's operand that equal the
 * plan's A word for word reproduce the rows of C* bit for bit.  A trial's operand may hold
 * Inf or NaN (they propagate as IEEE and are flagged).  d_c_out as in fi_gemm_inject_batch.
 * The caller owns d_a_stack and keeps it unmodified until the work has run.  All 2*M*N*K
 * flops of every trial are executed (one trial per work item; tile configurations 0..2, of
 * which 0 and 1 run as persistent workgroups when K is a multiple of 64, the default chosen
 * by problem size).
 * Errors: INVALID_ARG (NULLs, n_trials == 0, bad policy, trial_stride too small),
 * UNSUPPORTED (alignment; tiles x trials >= 2^31). */
fi_status fi_gemm_propagate_batch(fi_plan* plan, const void* d_a_stack, uint64_t trial_stride,
                                  uint32_t n_trials, uint32_t policy, fi_trial_result* d_results,
                                  float* d_c_out, void* stream);

/* The detector / corrector alone on materialised outputs (Sec. VI-A/B):
 * d_c is [batch][M][N], corrected in place; d_flags is NULL or
 * [batch][M][N] bytes (1 = flagged); d_n_flagged is NULL or [batch] counters,
 * overwritten.  Flags equal those of the fused epilogue on the same values. */
fi_status fi_detect_correct(fi_plan* plan, float* d_c, uint32_t batch, uint32_t policy,
                            uint8_t* d_flags, uint32_t* d_n_flagged, void* stream);

/* Outcome per trial (Sec. I: SDC; Sec. V-B: unchanged results; Sec. VI-B):
 * DETECTED if n_flagged > 0, else SDC if n_dev_pre > 0, else MASKED.
 * d_class is NULL or [n_trials] bytes; d_counts is [3] totals
 * (masked, sdc, detected), overwritten. */
fi_status fi_classify(fi_plan* plan, const fi_trial_result* d_results, uint32_t n_trials,
                      uint8_t* d_class, uint64_t* d_counts, void* stream);

/* Log2-binned histogram of a per-trial deviation (Sec. V-B, the analysis of how far results move; Fig. 7;
 * Fig. 9), from which the empirical CDF follows by a running sum.
 *   FI_HIST_SITE     |re'_sum - re_sum|: the change of the destination register, in binary32 from
 *                    the two site words (accumulator and product-term faults only);
 *   FI_HIST_DEV_PRE  the trial's largest output deviation before correction (max_dev_pre);
 *   FI_HIST_DEV_POST after correction.
 * Bin = biased exponent field of that binary32 value: 0 for zero (and subnormal), b for
 * [2^(b-127), 2^(b-126)), 255 for Inf or NaN.  Trials with status != 0 are skipped.
 * d_hist is [256] counters, overwritten.  Errors: INVALID_ARG (NULLs, n_trials == 0, which). */
enum { FI_HIST_SITE = 0, FI_HIST_DEV_PRE = 1, FI_HIST_DEV_POST = 2 };
fi_status fi_deviation_histogram(fi_plan* plan, const fi_fault* d_faults, const fi_trial_result* d_results,
                                 uint32_t n_trials, uint32_t which, uint64_t* d_hist, void* stream);

/* Host-side site selection (Sec. IV-A: uniform target, random bit(s)).
 * Trial t = first_trial + n draws from SplitMix64 seeded with seed + t*2^32:
 * u0 -> row (A: i; B: column j), u1, u2 -> (column, k-block) for ACC,
 * (column, k) for PRODUCT, (k-block, offset in block) for operands, u3 ->
 * position of an nbits-wide run of ones in the 32-bit (ACC) or 16-bit word; unif(n, u) = floor((u >> 32) * n / 2^32).
 * h_out is HOST memory for n_trials faults.  No device is needed. */
fi_status fi_sample_faults(uint64_t seed, uint32_t first_trial, uint32_t n_trials,
                           const fi_plan_desc* desc, uint32_t kind_mode, uint32_t nbits,
                           fi_fault* h_out);

/* Measurement aids (no counterpart in the paper; they serve the roofline report).
 *
 * fi_plan_set_clock_sink: d_clocks is NULL (off, the default) or DEVICE memory for 12 64-bit
 * words, 8-byte aligned, alive while batches of this plan run.  Workgroup 0 of each persistent
 * campaign kernel then writes {shader-clock counter, 100 MHz counter} when it starts and when it
 * has finished its last item: words 0..3 for the launch over the trials that leave the operands
 * alone, 4..7 for the operand-fault launch, 8..11 for fi_gemm_propagate_batch.  (cycles_end -
 * cycles_start) / ((ticks_end - ticks_start) / 1e8) is the shader clock that launch sustained.
 *
 * fi_probe_mfma_loop: launches n_workgroups workgroups of 8 waves that do nothing but issue
 * 2 * 8 * iters 32x32x16 MFMAs per wave on register-resident operands (random_data 0: all 1.0;
 * else seeded values of magnitude in [1, 2) with random signs), i.e. 2 * 8 * iters * 32768
 * flops per wave; the caller times it.  d_sink: DEVICE, n_workgroups * 512 floats, overwritten.
 * d_clocks: NULL or DEVICE [4] words as above.  Errors: UNSUPPORTED (dtype), INVALID_ARG, STATE. */
fi_status fi_plan_set_clock_sink(fi_plan* plan, uint64_t* d_clocks);
fi_status fi_probe_mfma_loop(uint32_t dtype, uint32_t random_data, uint32_t iters, uint32_t n_workgroups,
                             float* d_sink, uint64_t* d_clocks, void* stream);

/* Thread-local description of the last failure on this thread. */
const char* fi_last_error(void);

/* Hex SHA-256 of the kernel and ABI sources this binary was compiled from ("unknown" for a
 * build that did not record it), so that a loader can refuse a binary older than the sources
 * beside it.  A static string; never NULL.  Needs no device. */
const char* fi_build_info(void);

#ifdef __cplusplus
}
#endif
#endif
