/*
 * imunpack.h -- C ABI of the MI355X (gfx950) exact low-bit integer GEMM library.
 *
 * The operations are those of "IM-Unpack: Training and Inference with Arbitrarily Low
 * Precision Integers" (arXiv 2403.07339):
 *
 *   Sec. 1, Eq. (gemm)            C = A B^T,  A: n x d,  B: h x d,  C: n x h
 *   Sec. 2, Eq. (quantized_A)     A_q = round(A / scale)            (all entries, no clipping)
 *   Sec. 2, Eq. (quantized_gemm)  C  ~= scale_A * scale_B * (A_q B_q^T)
 *   Sec. 4                        s = 2^(b-1); an entry v is In-Bound iff |v| <= s-1, else
 *                                 Out-of-Bound (OB, a "heavy hitter")
 *   Sec. 4, Eq. (mod)             digits m(v, s, i), each In-Bound, v = sum_i s^i m(v, s, i)
 *   Alg. 1 / 2 / 4 / 5            UnpackRow, UnpackColumn, UnpackBoth and the dispatcher Unpack
 *   Sec. 4 "Combining everything" (A_u, B_e, S_u, Pi_A)    = Unpack(A,   B,   I,   b, strategy_A)
 *                                 (B_eu, A_ue, S_uu, Pi_B) = Unpack(B_e, A_u, S_u, b, strategy_B)
 *                                 A B^T = Pi_A A_ue S_uu B_eu^T Pi_B^T
 *   Alg. 3                        ScaledMatMul: one low-bit GEMM per distinct diagonal entry of S
 *   Sec. 4.2                      unpack ratio r = n' d' h' / (n d h)
 *
 * Throughout, "row" is the non-contracted index (n or h) and "column" the contracted one (d).
 * Digits follow the sign-magnitude reading of floor/mod: digit i of v is
 * sign(v) * ((|v| >> (b-1) i) & (s-1)), which is the only reading under which every digit lies in
 * the symmetric In-Bound interval the paper states.  Rounding is IEEE binary32 division followed
 * by round-half-to-even.  UnpackBoth breaks ties between equal OB counts by the lowest index
 * (rows before columns when the two top counts are equal, as Alg. 4 prints).
 *
 * Conventions
 *   - Every pointer named "device" is GPU memory owned by the caller (hipMalloc / a PyTorch
 *     tensor); "host" pointers are ordinary host memory.  The library owns only plan objects and
 *     batch contexts.
 *   - A plan object belongs to one thread at a time.  Calls that take a const plan only read it;
 *     the others (re-planning, unpack, GEMM, the bound queries and the exports) update state kept in
 *     it (host mirrors of device results, lazily built tables) and must not run concurrently on the
 *     same plan.  Different plans are independent.
 *   - Every function returns IMUNPACK_OK (0) or a negative error code; nothing throws or aborts.
 *   - stream is a hipStream_t passed as void* (NULL = the default stream).  Calls are
 *     asynchronous on it unless stated otherwise.
 *   - All matrices are row-major; ld* is the distance in elements between consecutive rows.
 *   - 2 <= b <= 8: unpacked operands are stored as int8 for every b, or on request as 6-bit
 *     floating-point codes for b <= 4 (imunpack_plan_set_digits).
 */
#ifndef IMUNPACK_H
#define IMUNPACK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void *imunpack_stream_t;
typedef struct imunpack_plan imunpack_plan_t;
typedef struct imunpack_batch imunpack_batch_t;

enum { IMUNPACK_ROW = 0, IMUNPACK_COL = 1, IMUNPACK_BOTH = 2 };

enum {
    IMUNPACK_OK = 0,
    IMUNPACK_EINVAL = -1, /* null pointer, b outside [2,8], unknown strategy, bad sizes or strides */
    IMUNPACK_ERANGE = -2, /* a value or an accumulator bound does not fit (see each call)           */
    IMUNPACK_ENOMEM = -3, /* device or host allocation failed                                       */
    IMUNPACK_EHIP = -4,   /* a HIP call failed; see imunpack_last_hip_error()                       */
    IMUNPACK_ESMALL = -5  /* a caller buffer or workspace is too small                              */
};

/* Heavy-hitter statistics of one integer operand (device pointers, lengths rows / cols):
 * OB count and largest magnitude per row and per column.  (Sec. 4: the IB/OB predicate;
 * Alg. 1 line 3, Alg. 2 line 3, Alg. 4 line 3 consume them.)
 * Optionally also the list of the OB entries themselves, which UnpackBoth (Alg. 4) works on:
 * ob holds 3 * ob_cap int32 laid out as [rows | cols | values], *ob_count (device) the number of
 * OB entries found -- if that exceeds ob_cap the list is incomplete and the planner scans the
 * operand itself.  ob == NULL (ob_cap == 0) skips the list. */
typedef struct {
    int32_t *rowcnt;
    int32_t *colcnt;
    int32_t *rowmax;
    int32_t *colmax;
    int32_t *ob;
    int64_t ob_cap;
    int32_t *ob_count;
} imunpack_stats_t;

/* ---- (0) the range estimate that sets the RTN step ----------------------------------------------
 * Sec. 2, the sentence after Eq. (quantized_A): alpha_p(A), the p-th percentile of the magnitudes of
 * A: the smallest magnitude a such that at least p % of the entries lie in [-a, a], i.e. the k-th
 * smallest |x| with k = ceil(p * rows * cols / 100) (an entry of A, no interpolation).  With beta
 * integers to cover [-alpha_p, alpha_p], Eq. (quantized_A) is imunpack_quantize with
 * scale = alpha_p / (0.5 * beta).
 * X: device, element (r, c) at X[r*sx_r + c*sx_c], strides > 0.  0 < p <= 100; rows * cols < 2^32.
 * alpha: device, one float, written when the stream gets there.  status_flag: device, may be NULL;
 * set to 1 if X holds a NaN (alpha is then meaningless), else 0.  workspace: device,
 * IMUNPACK_PERCENTILE_WORKSPACE_BYTES, contents irrelevant before and after.  Errors: EINVAL. */
#define IMUNPACK_PERCENTILE_WORKSPACE_BYTES 16384
int imunpack_percentile(const float *X, int64_t rows, int64_t cols, int64_t sx_r, int64_t sx_c,
                        double p, float *alpha, int32_t *status_flag, void *workspace,
                        imunpack_stream_t stream);

/* The RTN step of Eq. (quantized_A) itself, formed on the device: beta integers are to cover
 * [-alpha_p, alpha_p], so one step is alpha_p / (0.5 beta) (one binary32 division; Sec. 2, the sentence
 * after Eq. (quantized_A) defines alpha_p).  A matrix whose p-th percentile is 0 (mostly zeros) falls back
 * to its largest magnitude, an all-zero one to the step 1.  Arguments as imunpack_percentile; step:
 * device, one float, written when the stream gets there (imunpack_gemm_batched hands such steps from
 * kernel to kernel without the host reading them).  Errors: EINVAL (also beta not a positive finite number). */
int imunpack_rtn_step(const float *X, int64_t rows, int64_t cols, int64_t sx_r, int64_t sx_c, double p,
                      float beta, float *step, int32_t *status_flag, void *workspace,
                      imunpack_stream_t stream);

/* The same range estimate for callers that cannot allocate device memory or bring a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the counters and the
 * selection state live in a fixed array of IMUNPACK_PERCENTILE_WORKSPACE_BYTES of device memory that the
 * library's code object carries, one copy per GPU, held until the process ends.  The call itself
 * allocates and frees nothing.  Arguments, result and errors as imunpack_percentile without the
 * workspace, except that more than IMUNPACK_PERCENTILE_STATIC_MAX_ENTRIES entries (what the array's
 * 32-bit counters can count) return ERANGE.  The array is cleared at the start of every call; all calls
 * on one GPU share it, so two calls that overlap on one GPU (different streams or threads) race: issue
 * them on one stream, or order them with events. */
#define IMUNPACK_PERCENTILE_STATIC_MAX_ENTRIES 4294967295ll
int imunpack_percentile_static(const float *X, int64_t rows, int64_t cols, int64_t sx_r, int64_t sx_c,
                               double p, float *alpha, int32_t *status_flag, imunpack_stream_t stream);

/* ---- (1)+(2) RTN quantisation fused with the heavy-hitter scan --------------------------------
 * Sec. 2, Eq. (quantized_A) with the step supplied by the caller:
 *     Q[r*ldq + c] = rint(X[r*sx_r + c*sx_c] / scale)      (int32, no clipping)
 * The paper prints the scaling as a multiplication by 0.5 beta / alpha_p; the reading taken here is a
 * binary32 division by the step scale = alpha_p / (0.5 beta) (the two can differ in the last bit of
 * the quotient, and so at rounding ties; the oracle the library is checked against divides too).
 * and, in the same pass, the statistics of Q for bit width b (any of the four stats pointers, or
 * stats itself, may be NULL to skip it).  X, Q, stats, status: device.  X may be any strided view
 * with sx_r, sx_c >= 1 (sx_c == 1 and sx_r == 1 have fast paths); Q is written row-major.
 * status (device int32, may be NULL) is set to 0, then to 1 if any input is NaN/Inf or any
 * quotient has magnitude >= 2^31 (such outputs are written as 0); the call itself still returns
 * IMUNPACK_OK -- read status when convenient.
 * Errors: EINVAL (null X/Q, rows/cols < 0, a stride < 1, ldq < cols, scale not finite or <= 0,
 * b outside [2,8]). */
int imunpack_quantize(const float *X, int64_t rows, int64_t cols, int64_t sx_r, int64_t sx_c,
                      float scale, int b, int32_t *Q, int64_t ldq,
                      const imunpack_stats_t *stats, int32_t *status, imunpack_stream_t stream);

/* The same for both operands of one product A B^T (A: n x d, B: h x d, Sec. 2 Eq. (quantized_A) applied to
 * each with its own step): results as two imunpack_quantize calls, issued as one clearing launch and,
 * when both operands take the unit-column-stride fast path, one launch over the rows of both (fewer
 * launches, and the shorter operand fills the tail of the longer one).  status (device, may be NULL):
 * two int32, status[0] for A and status[1] for B.  Errors: as imunpack_quantize. */
int imunpack_quantize_pair(const float *A, int64_t n, int64_t sa_r, int64_t sa_c, float scale_A, int32_t *QA,
                           int64_t ldqa, const imunpack_stats_t *stats_A, const float *B, int64_t h,
                           int64_t sb_r, int64_t sb_c, float scale_B, int32_t *QB, int64_t ldqb,
                           const imunpack_stats_t *stats_B, int64_t d, int b, int32_t *status,
                           imunpack_stream_t stream);

/* ---- (2) stand-alone scan of an integer operand (Sec. 4, IB/OB definition) -------------------- */
int imunpack_scan(const int32_t *Q, int64_t rows, int64_t cols, int64_t ldq, int b,
                  const imunpack_stats_t *stats, imunpack_stream_t stream);

/* ---- strategy choice (Sec. 4.2, unpack ratio r = n'd'h' / (ndh); the "Mix" rows of its tables) -
 * Prices the four pairs of the one-axis strategies from the scan statistics alone, without
 * unpacking: UnpackRow / UnpackColumn append one slot per further digit of the largest magnitude of
 * a row / column, so n', d', h' follow from rowmax / colmax (for UnpackColumn on both operands a
 * column k of A with LA digits meets LB digits of column k of B: LA * LB columns).
 * stats_A, stats_B: device, rowmax and colmax required.  workspace: device, 8-byte aligned,
 * IMUNPACK_PRICE_WORKSPACE_BYTES, contents irrelevant before and after (the call allocates nothing).
 * dims_out (host, may be NULL): [pair][3] = n', d', h' for the pairs (strategy_A, strategy_B) =
 * (ROW,ROW), (ROW,COL), (COL,ROW), (COL,COL); ratio_out (host, may be NULL): their r.  best_A / best_B
 * (host, may be NULL): the pair with the smallest r (first in that order on ties).  UnpackBoth is
 * priced by planning with it (imunpack_plan + imunpack_plan_dims).  Synchronises the stream.
 * Errors: EINVAL, ERANGE (a size does not fit int64), EHIP. */
#define IMUNPACK_PRICE_WORKSPACE_BYTES 64
int imunpack_price(const imunpack_stats_t *stats_A, int64_t n, const imunpack_stats_t *stats_B,
                   int64_t h, int64_t d, int b, void *workspace, int64_t *dims_out, double *ratio_out,
                   int *best_A, int *best_B, imunpack_stream_t stream);

/* ---- (3) unpack plan (Alg. 1, 2, 4, 5 and the two-operand composition of Sec. 4) -------------
 * Decides every row / column split for A (with B as partner) and then for B (with A_u as partner
 * and S_u carried over) without moving the operands.  A: n x d, B: h x d, int32, device.
 * stats_A / stats_B: statistics of A / B for this b as written by imunpack_quantize or
 * imunpack_scan; NULL lets the call scan the operand itself.  For an UnpackBoth operand the OB
 * entry list of its statistics is used if it is complete, and copied: nothing of stats_A / stats_B
 * is read after the call returns.
 * *plan == NULL creates a plan object; a non-NULL *plan is re-planned in place and its device
 * buffers are reused (they only grow), so that steady-state calls allocate nothing.
 * Synchronises the stream (the sizes n', d', h' are needed on the host).
 * Errors: EINVAL; ERANGE if an exponent group is too long for int32 accumulation or a weight
 * s^k would not fit 62 bits; ENOMEM; EHIP. */
int imunpack_plan(const int32_t *A, int64_t n, int64_t d, int64_t lda,
                  const int32_t *B, int64_t h, int64_t ldb,
                  int b, int strategy_A, int strategy_B,
                  const imunpack_stats_t *stats_A, const imunpack_stats_t *stats_B,
                  imunpack_plan_t **plan, imunpack_stream_t stream);

/* Sizes of the unpacked problem (host outputs; any may be NULL): n', d', h' of Sec. 4.2 and the
 * number of distinct diagonal entries of S_uu (the GEMM groups of Alg. 3). */
int imunpack_plan_dims(const imunpack_plan_t *plan, int64_t *n_u, int64_t *d_u, int64_t *h_u,
                       int32_t *n_groups);

/* The plan in the order the paper's algorithms produce it (host buffers sized from
 * imunpack_plan_dims; any may be NULL).  Pi_A column R is s^rowA_exp[R] at row rowA_src[R]; Pi_B
 * likewise; S_uu[c,c] = s^col_exp[c]; col_src[c] is the original column that unpacked column c
 * descends from; col_parent[c] is the column that column c was appended for (the one whose
 * floor(. / s) it took and whose copy the partner received: Alg. 2 lines 4-7, Alg. 4 lines 11-14),
 * -1 for the d original columns.  ops (3 * (n' - n + h' - h + d' - d) int32, that count also written
 * to *n_ops) lists every split in the order the paper's algorithms make them, as triples
 * (0 = first / 1 = second Unpack call of Sec. 4 "Combining everything", 0 = row split / 1 = column
 * split, index of the split row or column at that moment).
 * Synchronises the stream used by imunpack_plan. */
int imunpack_plan_export(imunpack_plan_t *plan,
                         int32_t *rowA_src, int32_t *rowA_exp,                   /* n' */
                         int32_t *rowB_src, int32_t *rowB_exp,                   /* h' */
                         int32_t *col_src, int32_t *col_exp, int32_t *col_parent, /* d' */
                         int32_t *ops, int64_t *n_ops);

int imunpack_plan_destroy(imunpack_plan_t *plan);

/* ---- weights that stay resident (Sec. 4.2: weights are unpacked once, when they are loaded) -----
 * The unpacking of the second operand, Unpack(B_e, A_u, S_u, b, strategy_B), depends on the first operand
 * only through the column slots of A's unpacking (which columns B_e repeats, and their exponents).
 * keep != 0 is the caller's promise that from now on B, its statistics and its OB list are the same in
 * every imunpack_plan on this plan object: a plan call then compares, on the device, the column slots of
 * A's unpacking with those of the call before and, if they are the same, takes the second operand's
 * unpacking (for UnpackBoth: without running Alg. 4 on it again) and the layouts of B's rows and of the
 * columns over as they stand (no extra host wait; the result is the same plan either way); the first
 * imunpack_unpack after such a plan call writes only the A store if it is given the B_eu buffer that the
 * unpack before wrote (same address, same digit format): B_eu and its row norms are already what they
 * would become.  Otherwise, and in the first call after keep was set, B is unpacked as usual.
 * imunpack_plan_weights_reused tells which of the two the last plan call did.  keep == 0 (the default)
 * ends the promise.  Errors: EINVAL (null plan). */
int imunpack_plan_keep_weights(imunpack_plan_t *plan, int keep);
int imunpack_plan_weights_reused(const imunpack_plan_t *plan);

/* ---- digit storage format of the unpacked operands ---------------------------------------------
 * Sec. 4.2 ("arbitrarily low" bit widths): for b <= 4 every digit lies in [-7, 7] and is exactly
 * representable in the 6-bit floating-point format e2m3 (1 sign, 2 exponent, 3 mantissa bits), which the
 * matrix cores multiply at twice the int8 rate and which takes three quarters of the bytes.  The
 * products and their sums are integers below 2^24 in binary32 accumulators, hence exact (the call
 * checks the bound, as it does for int32); results are bit-identical to the int8 path.
 * IMUNPACK_DIGITS_INT8 (default): one int8 per digit.  IMUNPACK_DIGITS_FP6: 96 bytes per 128 columns; a
 * group of 64 columns takes 48 bytes: the 32 columns of each half form a 192-bit string (column j at
 * bits 6j .. 6j+5), stored as the first 16 bytes of both strings followed by the last 8 bytes of both
 * (those two in the other order in physical rows whose index has bit 4 set).  The request stays with the plan object
 * across re-planning and is in effect whenever the plan's b <= 4 (a plan with b > 4 keeps int8);
 * imunpack_plan_digits returns the format in effect.  Call after imunpack_plan and before
 * imunpack_unpacked_bytes / imunpack_unpack: the format changes the sizes and the row pitches.
 * Errors: EINVAL (no valid plan, unknown format, FP6 on a plan with b > 4). */
enum { IMUNPACK_DIGITS_INT8 = 0, IMUNPACK_DIGITS_FP6 = 1 };
int imunpack_plan_set_digits(imunpack_plan_t *plan, int format);
int imunpack_plan_digits(const imunpack_plan_t *plan);

/* ---- (4) digit scatter (Eq. (mod); Alg. 1 l.4-5, Alg. 2 l.4-6, Alg. 4 l.7-8, 11-13) -----------
 * Writes the unpacked operands as int8 in the plan's *physical* layout: rows grouped by source row (all
 * digit levels of a row of A inside one 64-row chunk of a GEMM tile, of a row of B inside one tile),
 * both padded to tile multiples.  B_eu is stored in full, its columns grouped by diagonal entry of S_uu
 * in whole k-tiles of 128.  Of A_ue only the columns of A_u are stored, each once ("A store"): where
 * column unpacking of the partner repeats a column (Alg. 2 line 6 / Alg. 4 line 13) the GEMM reads the
 * stored one again, so the copies cost neither memory nor traffic.
 * imunpack_unpacked_bytes gives the buffer sizes and the workspace an un-fused GEMM needs.
 * A, B: the int32 operands the plan was made from.  A_ue, B_eu: device, caller-allocated.
 * imunpack_unpack does not wait for the device: the accumulator bounds that select the GEMM path
 * reach the host later, and imunpack_gemm / imunpack_plan_fusable wait for them. */
int imunpack_unpacked_bytes(const imunpack_plan_t *plan, size_t *bytes_A, size_t *bytes_B,
                            size_t *bytes_workspace);
/* The shape of the two buffers (host output, six values): physical rows, stored columns and bytes from
 * one row to the next, of the A store and then of B_eu.  bytes_A = rows * pitch.  The bytes of a row
 * behind its stored columns are neither written nor read. */
int imunpack_plan_layout(const imunpack_plan_t *plan, int64_t *shape);
int imunpack_unpack(imunpack_plan_t *plan, const int32_t *A, int64_t lda,
                    const int32_t *B, int64_t ldb, int8_t *A_ue, int8_t *B_eu,
                    imunpack_stream_t stream);

/* Test aid: re-orders the physical operands into the paper's order, dense n' x d' and h' x d'. */
int imunpack_unpack_canonical(imunpack_plan_t *plan, const int8_t *A_ue, const int8_t *B_eu,
                              int8_t *A_canon, int8_t *B_canon, imunpack_stream_t stream);

/* ---- (5) int8 MFMA GEMM (Alg. 3) ---------------------------------------------------------------
 * Runs C_g = A_ue[:, I_g] B_eu[:, I_g]^T for every group g of equal diagonal entry with int32
 * accumulation on v_mfma_i32_*_i8 and combines the groups by shifts (six-bit digits: binary32
 * accumulation of integers below 2^24 on v_mfma_f32_32x32x64_f8f6f4, the bound below is 2^24 then).
 * fuse != 0: one launch; the recombination (6) and the dequantisation run in the epilogue and
 *   C_int (n x h int64, device, may be NULL) and/or C_fp (n x h fp32, device, may be NULL) are
 *   written directly.  This needs the shifted sum of all groups to fit int32 for this plan's
 *   operands (bound measured by imunpack_unpack); if it does not, the call falls back to the
 *   un-fused path when workspace != NULL and returns ERANGE otherwise.
 * fuse == 0: writes the unpacked product C_u = A_ue S_uu B_eu^T as int64 into workspace
 *   (imunpack_unpacked_bytes) for imunpack_recombine; C_int / C_fp are ignored.
 * ldc: row stride of C_int and C_fp in elements (>= h).  scale_A, scale_B: the RTN steps. */
int imunpack_gemm(imunpack_plan_t *plan, const int8_t *A_ue, const int8_t *B_eu,
                  void *workspace, int64_t *C_int, float *C_fp, int64_t ldc,
                  float scale_A, float scale_B, int fuse, imunpack_stream_t stream);

/* ---- the whole path over a strided batch of products (Sec. 1 "Notations": the GEMMs of a Transformer) -
 * C_i = step_A,i * step_B,i * (RTN(A_i / step_A,i) RTN(B_i / step_B,i)^T), i = 0 .. batch-1, the integer
 * product evaluated exactly with b-bit digits (Sec. 4), as fp32.  Every item is a GEMM of its own: its own
 * percentile steps alpha_p / (0.5 beta) (Eq. (quantized_A)), its own unpack plan.  A_i: n x d at
 * A + i * sa_b, element (r, c) at offset r * sa_r + c * sa_c (so transposed operands are views, nothing is
 * copied); B_i: h x d likewise; C_i: n x h row-major at C + i * sc_b with row stride ldc.  All device, fp32.
 * *ctx == NULL creates a context; passing it again reuses its buffers (Q_A, Q_B, statistics, the unpacked
 * operands, a plan: they only grow), so steady-state calls allocate nothing.  The library owns the context;
 * release it with imunpack_batch_destroy.  The steps never leave the device; per item the host waits once,
 * inside the plan call, for the sizes of the unpacked problem.  Synchronises the stream before returning.
 * Errors: EINVAL; ERANGE if any operand held a NaN or Inf or a quotient beyond 32 bits (the outputs of
 * that item are then undefined); ENOMEM; EHIP.
 * For b <= 4 the digits are stored as six-bit floating-point codes (imunpack_plan_set_digits); the
 * results are the same bits either way. */
int imunpack_gemm_batched(const float *A, int64_t sa_b, int64_t sa_r, int64_t sa_c,
                          const float *B, int64_t sb_b, int64_t sb_r, int64_t sb_c,
                          int64_t batch, int64_t n, int64_t d, int64_t h,
                          double p, float beta_A, float beta_B, int b, int strategy_A, int strategy_B,
                          float *C, int64_t sc_b, int64_t ldc, imunpack_batch_t **ctx,
                          imunpack_stream_t stream);
int imunpack_batch_destroy(imunpack_batch_t *ctx);

/* ---- (6) recombination and dequantisation (Sec. 4 "Reconstructing A"; Eq. (quantized_gemm)) ---
 * C_int = Pi_A C_u Pi_B^T by shift-and-add in int64 from the workspace of an un-fused
 * imunpack_gemm, and C_fp = scale_A * scale_B * C_int (one rounding to fp32).  Either output may
 * be NULL. */
int imunpack_recombine(const imunpack_plan_t *plan, const void *workspace,
                       float scale_A, float scale_B, int64_t *C_int, float *C_fp, int64_t ldc,
                       imunpack_stream_t stream);

/* ---- diagnostics ------------------------------------------------------------------------------- */
/* Per-kernel device time of the last call of each stage on this plan is not kept; callers time
 * with events.  These two describe errors. */
const char *imunpack_strerror(int code);
int imunpack_last_hip_error(void);

/* Which GEMM path the plan's last imunpack_unpack selected: 1 = single fused launch is exact,
 * 0 = the shifted group sum may exceed int32 and the un-fused path is required.  Waits for that
 * unpack to finish on the device. */
int imunpack_plan_fusable(imunpack_plan_t *plan);

/* The two numbers that decision rests on, as the plan's last imunpack_unpack measured them:
 * bound[0] = max over the rows R of A_ue of sum_c s^e(c) |A_ue[R, c]|, bound[1] the same for B_eu,
 * e(c) the exponent of column c's diagonal entry of S_uu (Alg. 3).  Every entry of the other operand
 * is at most s - 1 in magnitude, so |sum_c s^e(c) a_c b_c| <= (s - 1) * min(bound[0], bound[1]), and
 * the fused launch is exact when that stays below 2^31.  Values of 2^44 and more are reported
 * saturated (at least 2^44).  bound: host, two elements.  Waits like imunpack_plan_fusable. */
int imunpack_plan_bounds(imunpack_plan_t *plan, uint64_t *bound);

/* Measured matrix-core peak (benchmark reporting only, not part of the method): launches
 * `workgroups` workgroups of 4 waves that each issue 8 * iters register-resident
 * v_mfma_i32_32x32x32_i8 with no memory traffic, and writes the number of integer operations
 * (2 per multiply-add) the launch performs to *ops.  The caller times the stream. */
int imunpack_diag_mfma_peak(int workgroups, int iters, int64_t *ops, imunpack_stream_t stream);

/* Measured HBM rate (benchmark reporting only): copies `bytes` (a multiple of 1 MiB, at most 65535 MiB)
 * from src to dst (device, 16-byte aligned, not overlapping) in the access pattern of the quantize pass,
 * with non-temporal loads and stores.  The caller times the stream; the traffic is 2 * bytes. */
int imunpack_diag_copy(const void *src, void *dst, int64_t bytes, imunpack_stream_t stream);

/* Shader clock under the GEMM's own load (benchmark reporting only).  While `ticks` (device, two
 * elements, owned by the caller) is set, every fused imunpack_gemm launch of this process has its
 * first workgroup write ticks[0] = shader clock cycles and ticks[1] = ticks of the constant 100 MHz
 * clock that its loop over K took; ticks[0] / ticks[1] * 100 is the clock in MHz the matrix cores ran
 * at, which the power limit holds below the 2400 MHz the published peak assumes.  NULL switches the
 * probe off (the default).  Not thread safe; set it while no GEMM is in flight. */
int imunpack_diag_clock_probe(uint64_t *ticks);

#ifdef __cplusplus
}
#endif
#endif /* IMUNPACK_H */
