/*
 * IM-Unpack CPU oracle  --  TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct implementation of the exact low-bit integer
 * GEMM of "IM-Unpack: Training and Inference with Arbitrarily Low Precision
 * Integers" (arXiv 2403.07339).  Only tests/, the smoke check and the
 * cpu_baseline leg of bench.py may call it.  It shares no code, header, table or
 * helper with the HIP library, and is never tuned for speed.
 *
 * What follows the paper literally (dense matrices that really grow):
 *   orc_rtn_quantize      Sec. 2, Eq. (quantized_A): A_q = round(c * A), all entries, no clipping
 *   orc_int_gemm          Sec. 1, Eq. (gemm): C = A B^T on the integers, int64
 *   orc_dequantize        Sec. 2, Eq. (quantized_gemm): undo the two scalings
 *   orc_digit             Sec. 4, Eq. (mod): m(v, s, i)
 *   unpack_row            Alg. 1  UnpackRow(A, b)
 *   unpack_column         Alg. 2  UnpackColumn(A, B, S, b)
 *   orc_scaled_matmul     Alg. 3  ScaledMatMul(A, B, S)
 *   unpack_both           Alg. 4  UnpackBoth(A, B, S, b)
 *   unpack_dispatch       Alg. 5  Unpack(A, B, S, b, strategy)
 *   orc_unpack_pair       Sec. 4 "Combining everything": A first, then B with A_u, S_u
 *   orc_apply_pi          Sec. 4 "Reconstructing A": Pi applied as an index-add
 *
 * Readings of the paper adopted here (the paper leaves them open):
 *   - floor / mod act on magnitudes (C's truncating '/' and '%'), so that every
 *     digit lies in the symmetric interval [-(s-1), s-1] the paper states and the
 *     digit sum of Eq. (vecter_unpack) reproduces negative entries too.
 *   - round = IEEE-754 binary32 division followed by round-half-to-even.
 *   - UnpackBoth ties: rows win over columns when c0 >= c1 (as printed); among
 *     rows (columns) with the same top count the lowest current index wins.
 *   - UnpackBoth starts with Pi = I (its printed signature has no Pi input).
 *   - OB counts in UnpackBoth are those of the current, growing matrix.
 *
 * Pi is held as one (source row, weight) pair per column, which is exactly the
 * structure the paper states for it (each column has a single non-zero); S is
 * held as its diagonal.  Both hold the literal values s^k as int64.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_ROW 0
#define ORC_COL 1
#define ORC_BOTH 2

/* ------------------------------------------------------------------ */
/* Sec. 2: RTN quantisation, integer GEMM, dequantisation              */
/* ------------------------------------------------------------------ */

/* q = round(x / scale).  Returns 0, or 1 if any input is non-finite or the
 * quotient does not fit int32 (those outputs are written as 0). */
int orc_rtn_quantize(const float *x, int64_t count, float scale, int32_t *q)
{
    int bad = 0;
    for (int64_t t = 0; t < count; ++t) {
        volatile float quo = x[t] / scale; /* one correctly rounded binary32 division */
        float r = rintf(quo);              /* round half to even (default rounding mode) */
        if (!isfinite(r) || fabsf(r) >= 2147483648.0f) {
            bad = 1;
            q[t] = 0;
        } else {
            q[t] = (int32_t)r;
        }
    }
    return bad;
}

/* C[i,j] = sum_k A[i,k] * B[j,k]   (A: n x d, B: h x d, C: n x h, all row-major) */
void orc_int_gemm(const int32_t *A, int64_t n, int64_t d, const int32_t *B, int64_t h, int64_t *C)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t j = 0; j < h; ++j) {
            int64_t acc = 0;
            for (int64_t k = 0; k < d; ++k)
                acc += (int64_t)A[i * d + k] * (int64_t)B[j * d + k];
            C[i * h + j] = acc;
        }
    }
}

/* Same dot products, but only at the listed output positions (for full-size checks). */
void orc_int_gemm_at(const int32_t *A, int64_t d, const int32_t *B,
                     const int64_t *rows, const int64_t *cols, int64_t count, int64_t *out)
{
    for (int64_t t = 0; t < count; ++t) {
        const int32_t *a = A + rows[t] * d, *b = B + cols[t] * d;
        int64_t acc = 0;
        for (int64_t k = 0; k < d; ++k)
            acc += (int64_t)a[k] * (int64_t)b[k];
        out[t] = acc;
    }
}

/* C_fp[t] = scale_A * scale_B * C_int[t]  in binary64 */
void orc_dequantize(const int64_t *C, int64_t count, float scale_a, float scale_b, double *out)
{
    for (int64_t t = 0; t < count; ++t)
        out[t] = (double)scale_a * (double)scale_b * (double)C[t];
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Sec. 4: digits                                                      */
/* ------------------------------------------------------------------ */

static int32_t div_s(int32_t v, int32_t s) { return v / s; } /* "floor(v / s)" on the magnitude */
static int32_t mod_s(int32_t v, int32_t s) { return v % s; } /* "v mod s", sign follows v       */
static int is_ob(int32_t v, int32_t s) { return v >= s || v <= -s; }

/* m(v, s, i) = floor(v / s^i) mod s */
int32_t orc_digit(int32_t v, int32_t s, int i)
{
    while (i-- > 0)
        v = div_s(v, s);
    return mod_s(v, s);
}

/* ------------------------------------------------------------------ */
/* dense matrices that grow by rows and by columns                     */
/* ------------------------------------------------------------------ */

typedef struct {
    int64_t rows, cols, rcap, ccap;
    int32_t *v; /* v[r * ccap + c] */
} mat_t;

static void mat_reserve(mat_t *m, int64_t rcap, int64_t ccap)
{
    if (rcap <= m->rcap && ccap <= m->ccap)
        return;
    if (rcap < m->rcap) rcap = m->rcap;
    if (ccap < m->ccap) ccap = m->ccap;
    int32_t *nv = (int32_t *)calloc((size_t)(rcap * ccap > 0 ? rcap * ccap : 1), sizeof(int32_t));
    for (int64_t r = 0; r < m->rows; ++r)
        memcpy(nv + r * ccap, m->v + r * m->ccap, (size_t)m->cols * sizeof(int32_t));
    free(m->v);
    m->v = nv;
    m->rcap = rcap;
    m->ccap = ccap;
}

static mat_t mat_from(const int32_t *src, int64_t rows, int64_t cols)
{
    mat_t m = {0, 0, 0, 0, NULL};
    mat_reserve(&m, rows > 0 ? rows : 1, cols > 0 ? cols : 1);
    m.rows = rows;
    m.cols = cols;
    for (int64_t r = 0; r < rows; ++r)
        memcpy(m.v + r * m.ccap, src + r * cols, (size_t)cols * sizeof(int32_t));
    return m;
}

static int32_t *mat_at(mat_t *m, int64_t r, int64_t c) { return m->v + r * m->ccap + c; }

static int64_t mat_append_row(mat_t *m) /* new zero row, returns its index */
{
    if (m->rows == m->rcap)
        mat_reserve(m, m->rcap * 2, m->ccap);
    memset(m->v + m->rows * m->ccap, 0, (size_t)m->ccap * sizeof(int32_t));
    return m->rows++;
}

static int64_t mat_append_col(mat_t *m) /* new zero column, returns its index */
{
    if (m->cols == m->ccap)
        mat_reserve(m, m->rcap, m->ccap * 2);
    for (int64_t r = 0; r < m->rows; ++r)
        *mat_at(m, r, m->cols) = 0;
    return m->cols++;
}

/* a growable int64 vector (Pi weights, Pi sources, S diagonal) */
typedef struct {
    int64_t len, cap;
    int64_t *v;
} vec_t;

static vec_t vec_new(int64_t len)
{
    vec_t x;
    x.len = len;
    x.cap = len > 4 ? len : 4;
    x.v = (int64_t *)calloc((size_t)x.cap, sizeof(int64_t));
    return x;
}

static void vec_push(vec_t *x, int64_t val)
{
    if (x->len == x->cap) {
        x->cap *= 2;
        x->v = (int64_t *)realloc(x->v, (size_t)x->cap * sizeof(int64_t));
    }
    x->v[x->len++] = val;
}

/* A record of what the algorithms did, kept beside their outputs (bookkeeping, no arithmetic):
 * col_parent[c] = the column that column c was appended for (Alg. 2 line 4 / Alg. 4 line 11:
 * the column it took floor(. / s) of, and whose copy the partner received), -1 for the columns
 * the first Unpack call started from; ops = one triple per split, in the order the splits were
 * made: (which Unpack call of Sec. 4 "Combining everything": 0 or 1, 0 = row split / 1 = column
 * split, index of the split row or column at that moment). */
typedef struct {
    vec_t col_parent;
    vec_t ops;
    int call;
} trace_t;

/* ------------------------------------------------------------------ */
/* the single split steps the three algorithms share by definition     */
/* ------------------------------------------------------------------ */

static int row_has_ob(mat_t *A, int64_t i, int32_t s)
{
    for (int64_t c = 0; c < A->cols; ++c)
        if (is_ob(*mat_at(A, i, c), s)) return 1;
    return 0;
}

static int col_has_ob(mat_t *A, int64_t j, int32_t s)
{
    for (int64_t r = 0; r < A->rows; ++r)
        if (is_ob(*mat_at(A, r, j), s)) return 1;
    return 0;
}

/* Alg. 1 lines 4-6 (= Alg. 4 lines 7-9): split row i of A, extend Pi. */
static void split_row(mat_t *A, int64_t i, int32_t s, vec_t *pi_src, vec_t *pi_w, trace_t *tr)
{
    vec_push(&tr->ops, tr->call); vec_push(&tr->ops, 0); vec_push(&tr->ops, i);
    int64_t nr = mat_append_row(A);
    for (int64_t c = 0; c < A->cols; ++c) {
        int32_t v = *mat_at(A, i, c);
        *mat_at(A, nr, c) = div_s(v, s); /* append floor(A[i,:] / s) */
        *mat_at(A, i, c) = mod_s(v, s);  /* A[i,:] <- A[i,:] mod s   */
    }
    vec_push(pi_src, pi_src->v[i]);      /* append s * Pi[:, i]      */
    vec_push(pi_w, (int64_t)s * pi_w->v[i]);
}

/* Alg. 2 lines 4-7 (= Alg. 4 lines 11-14): split column j of A, duplicate column j of B, extend S. */
static void split_col(mat_t *A, mat_t *B, int64_t j, int32_t s, vec_t *S, trace_t *tr)
{
    vec_push(&tr->ops, tr->call); vec_push(&tr->ops, 1); vec_push(&tr->ops, j);
    vec_push(&tr->col_parent, j);
    int64_t nc = mat_append_col(A);
    for (int64_t r = 0; r < A->rows; ++r) {
        int32_t v = *mat_at(A, r, j);
        *mat_at(A, r, nc) = div_s(v, s);
        *mat_at(A, r, j) = mod_s(v, s);
    }
    int64_t nb = mat_append_col(B);
    for (int64_t r = 0; r < B->rows; ++r)
        *mat_at(B, r, nb) = *mat_at(B, r, j);
    vec_push(S, (int64_t)s * S->v[j]);
}

/* Alg. 1 */
static void unpack_row(mat_t *A, int b, vec_t *pi_src, vec_t *pi_w, trace_t *tr)
{
    int32_t s = (int32_t)1 << (b - 1);
    int64_t i = 0;
    while (i < A->rows) {
        if (row_has_ob(A, i, s))
            split_row(A, i, s, pi_src, pi_w, tr);
        ++i;
    }
}

/* Alg. 2 */
static void unpack_column(mat_t *A, mat_t *B, vec_t *S, int b, trace_t *tr)
{
    int32_t s = (int32_t)1 << (b - 1);
    int64_t i = 0;
    while (i < A->cols) {
        if (col_has_ob(A, i, s))
            split_col(A, B, i, s, S, tr);
        ++i;
    }
}

/* Alg. 4.  recount != 0 recomputes every OB count from the matrix at every
 * step instead of updating the counts after each split (bookkeeping only:
 * tests check that both give the same result). */
static void unpack_both(mat_t *A, mat_t *B, vec_t *S, int b, vec_t *pi_src, vec_t *pi_w, int recount,
                        trace_t *tr)
{
    int32_t s = (int32_t)1 << (b - 1);
    vec_t rc = vec_new(0), cc = vec_new(0);
    for (int64_t r = 0; r < A->rows; ++r) vec_push(&rc, 0);
    for (int64_t c = 0; c < A->cols; ++c) vec_push(&cc, 0);
    for (int64_t r = 0; r < A->rows; ++r)
        for (int64_t c = 0; c < A->cols; ++c)
            if (is_ob(*mat_at(A, r, c), s)) { rc.v[r]++; cc.v[c]++; }

    for (;;) {
        if (recount) {
            for (int64_t r = 0; r < A->rows; ++r) rc.v[r] = 0;
            for (int64_t c = 0; c < A->cols; ++c) cc.v[c] = 0;
            for (int64_t r = 0; r < A->rows; ++r)
                for (int64_t c = 0; c < A->cols; ++c)
                    if (is_ob(*mat_at(A, r, c), s)) { rc.v[r]++; cc.v[c]++; }
        }
        /* top OB count over rows and over columns; first (lowest) index among equals */
        int64_t c0 = 0, i = 0, c1 = 0, j = 0;
        for (int64_t r = 0; r < A->rows; ++r)
            if (rc.v[r] > c0) { c0 = rc.v[r]; i = r; }
        for (int64_t c = 0; c < A->cols; ++c)
            if (cc.v[c] > c1) { c1 = cc.v[c]; j = c; }
        if (c0 == 0 && c1 == 0)
            break;
        if (c0 >= c1) {
            /* counts after the split: row i becomes all-IB; the new row keeps the entries still OB */
            int64_t newcount = 0;
            for (int64_t c = 0; c < A->cols; ++c) {
                int32_t v = *mat_at(A, i, c);
                if (is_ob(v, s)) {
                    if (is_ob(div_s(v, s), s)) newcount++;
                    else cc.v[c]--;
                }
            }
            split_row(A, i, s, pi_src, pi_w, tr);
            rc.v[i] = 0;
            vec_push(&rc, newcount);
        } else {
            int64_t newcount = 0;
            for (int64_t r = 0; r < A->rows; ++r) {
                int32_t v = *mat_at(A, r, j);
                if (is_ob(v, s)) {
                    if (is_ob(div_s(v, s), s)) newcount++;
                    else rc.v[r]--;
                }
            }
            split_col(A, B, j, s, S, tr);
            cc.v[j] = 0;
            vec_push(&cc, newcount);
        }
    }
    free(rc.v);
    free(cc.v);
}

/* Alg. 5: Pi starts as I for every strategy; S and B pass through for UnpackRow. */
static void unpack_dispatch(mat_t *A, mat_t *B, vec_t *S, int b, int strategy,
                            vec_t *pi_src, vec_t *pi_w, int recount, trace_t *tr)
{
    if (strategy == ORC_ROW)
        unpack_row(A, b, pi_src, pi_w, tr);
    else if (strategy == ORC_COL)
        unpack_column(A, B, S, b, tr);
    else
        unpack_both(A, B, S, b, pi_src, pi_w, recount, tr);
}

/* ------------------------------------------------------------------ */
/* results handed to Python                                            */
/* ------------------------------------------------------------------ */

typedef struct {
    mat_t A, B;               /* A_ue (n' x d'), B_eu (h' x d') */
    vec_t S;                  /* diagonal of S_uu, length d'    */
    vec_t piA_src, piA_w;     /* Pi_A: column t has weight piA_w[t] at row piA_src[t] */
    vec_t piB_src, piB_w;     /* Pi_B likewise                  */
    trace_t tr;               /* column parents and the sequence of splits */
} orc_result_t;

static vec_t identity_src(int64_t n)
{
    vec_t x = vec_new(0);
    for (int64_t i = 0; i < n; ++i) vec_push(&x, i);
    return x;
}

static vec_t ones(int64_t n)
{
    vec_t x = vec_new(0);
    for (int64_t i = 0; i < n; ++i) vec_push(&x, 1);
    return x;
}

/* One application of Alg. 5 to (A, B, S): A is unpacked, B is the partner.
 * S_in == NULL means S = I.  The result's Pi_B is the identity. */
orc_result_t *orc_unpack(const int32_t *A, int64_t n, int64_t d, const int32_t *B, int64_t h,
                         const int64_t *S_in, int b, int strategy, int recount)
{
    orc_result_t *R = (orc_result_t *)calloc(1, sizeof(orc_result_t));
    R->A = mat_from(A, n, d);
    R->B = mat_from(B, h, d);
    R->S = vec_new(0);
    for (int64_t c = 0; c < d; ++c) vec_push(&R->S, S_in ? S_in[c] : 1);
    R->piA_src = identity_src(n);
    R->piA_w = ones(n);
    R->piB_src = identity_src(h);
    R->piB_w = ones(h);
    R->tr.col_parent = vec_new(0);
    for (int64_t c = 0; c < d; ++c) vec_push(&R->tr.col_parent, -1);
    R->tr.ops = vec_new(0);
    R->tr.call = 0;
    unpack_dispatch(&R->A, &R->B, &R->S, b, strategy, &R->piA_src, &R->piA_w, recount, &R->tr);
    return R;
}

/* Sec. 4 "Combining everything":
 *   A_u, B_e, S_u, Pi_A     = Unpack(A,   B,   I,   b, strategy_a)
 *   B_eu, A_ue, S_uu, Pi_B  = Unpack(B_e, A_u, S_u, b, strategy_b)            */
orc_result_t *orc_unpack_pair(const int32_t *A, int64_t n, int64_t d, const int32_t *B, int64_t h,
                              int b, int strategy_a, int strategy_b, int recount)
{
    orc_result_t *R = orc_unpack(A, n, d, B, h, NULL, b, strategy_a, recount);
    R->tr.call = 1;
    unpack_dispatch(&R->B, &R->A, &R->S, b, strategy_b, &R->piB_src, &R->piB_w, recount, &R->tr);
    return R;
}

void orc_result_dims(const orc_result_t *R, int64_t *n_u, int64_t *d_u, int64_t *h_u)
{
    *n_u = R->A.rows;
    *d_u = R->A.cols;
    *h_u = R->B.rows;
}

/* copies out dense row-major A_ue (n' x d'), B_eu (h' x d'), diag S (d'), Pi_A (n'), Pi_B (h') */
void orc_result_copy(orc_result_t *R, int32_t *A_ue, int32_t *B_eu, int64_t *S,
                     int64_t *piA_src, int64_t *piA_w, int64_t *piB_src, int64_t *piB_w)
{
    for (int64_t r = 0; r < R->A.rows; ++r)
        memcpy(A_ue + r * R->A.cols, mat_at(&R->A, r, 0), (size_t)R->A.cols * sizeof(int32_t));
    for (int64_t r = 0; r < R->B.rows; ++r)
        memcpy(B_eu + r * R->B.cols, mat_at(&R->B, r, 0), (size_t)R->B.cols * sizeof(int32_t));
    memcpy(S, R->S.v, (size_t)R->S.len * sizeof(int64_t));
    memcpy(piA_src, R->piA_src.v, (size_t)R->piA_src.len * sizeof(int64_t));
    memcpy(piA_w, R->piA_w.v, (size_t)R->piA_w.len * sizeof(int64_t));
    memcpy(piB_src, R->piB_src.v, (size_t)R->piB_src.len * sizeof(int64_t));
    memcpy(piB_w, R->piB_w.v, (size_t)R->piB_w.len * sizeof(int64_t));
}

void orc_result_free(orc_result_t *R)
{
    if (!R) return;
    free(R->A.v); free(R->B.v); free(R->S.v);
    free(R->piA_src.v); free(R->piA_w.v); free(R->piB_src.v); free(R->piB_w.v);
    free(R->tr.col_parent.v); free(R->tr.ops.v);
    free(R);
}

/* ------------------------------------------------------------------ */
/* Alg. 3 and the application of Pi                                    */
/* ------------------------------------------------------------------ */

/* C = sum over distinct diagonal values t of  t * A[:, I_t] B[:, I_t]^T
 * A: n x d, B: h x d (row-major), S: diagonal (d), C: n x h int64. */
void orc_scaled_matmul(const int32_t *A, int64_t n, int64_t d, const int32_t *B, int64_t h,
                       const int64_t *S, int64_t *C)
{
    for (int64_t t = 0; t < n * h; ++t) C[t] = 0;
    char *done = (char *)calloc((size_t)(d > 0 ? d : 1), 1);
    for (int64_t first = 0; first < d; ++first) {
        if (done[first]) continue;
        int64_t val = S[first]; /* a distinct diagonal entry; its index set is {k : S[k] == val} */
        for (int64_t k = first; k < d; ++k)
            if (S[k] == val) done[k] = 2;
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < n; ++i)
            for (int64_t j = 0; j < h; ++j) {
                int64_t acc = 0;
                for (int64_t k = first; k < d; ++k)
                    if (done[k] == 2)
                        acc += (int64_t)A[i * d + k] * (int64_t)B[j * d + k];
                C[i * h + j] += val * acc;
            }
        for (int64_t k = first; k < d; ++k)
            if (done[k] == 2) done[k] = 1;
    }
    free(done);
}

/* C_out (n x h) = Pi_A * C_u (n' x h') * Pi_B^T, each Pi applied as an index-add:
 * C_out[piA_src[R], piB_src[Q]] += piA_w[R] * piB_w[Q] * C_u[R, Q]. */
void orc_apply_pi(const int64_t *C_u, int64_t n_u, int64_t h_u,
                  const int64_t *piA_src, const int64_t *piA_w,
                  const int64_t *piB_src, const int64_t *piB_w,
                  int64_t n, int64_t h, int64_t *C_out)
{
    for (int64_t t = 0; t < n * h; ++t) C_out[t] = 0;
    for (int64_t R = 0; R < n_u; ++R)
        for (int64_t Q = 0; Q < h_u; ++Q)
            C_out[piA_src[R] * h + piB_src[Q]] += piA_w[R] * piB_w[Q] * C_u[R * h_u + Q];
}

/* The product identity at single output positions, from the unpacked operands:
 * out[t] = sum over R with piA_src[R]==rows[t], Q with piB_src[Q]==cols[t], c of
 *          piA_w[R] * piB_w[Q] * S[c] * A_ue[R,c] * B_eu[Q,c].                   */
void orc_unpacked_product_at(const orc_result_t *R, const int64_t *rows, const int64_t *cols,
                             int64_t count, int64_t *out)
{
    const mat_t *A = &R->A, *B = &R->B;
    for (int64_t t = 0; t < count; ++t) {
        int64_t acc = 0;
        for (int64_t r = 0; r < A->rows; ++r) {
            if (R->piA_src.v[r] != rows[t]) continue;
            for (int64_t q = 0; q < B->rows; ++q) {
                if (R->piB_src.v[q] != cols[t]) continue;
                int64_t w = R->piA_w.v[r] * R->piB_w.v[q];
                for (int64_t c = 0; c < A->cols; ++c)
                    acc += w * R->S.v[c] * (int64_t)A->v[r * A->ccap + c] * (int64_t)B->v[q * B->ccap + c];
            }
        }
        out[t] = acc;
    }
}

/* max |entry| over both unpacked operands (range check without copying them out) */
int32_t orc_result_max_abs(const orc_result_t *R)
{
    int32_t m = 0;
    const mat_t *ms[2] = {&R->A, &R->B};
    for (int w = 0; w < 2; ++w)
        for (int64_t r = 0; r < ms[w]->rows; ++r)
            for (int64_t c = 0; c < ms[w]->cols; ++c) {
                int32_t v = ms[w]->v[r * ms[w]->ccap + c];
                if (v < 0) v = -v;
                if (v > m) m = v;
            }
    return m;
}

/* copy out as int8 (callers check the range first); used for operand parity on the big configs */
void orc_result_copy_i8(orc_result_t *R, int8_t *A_ue, int8_t *B_eu)
{
    for (int64_t r = 0; r < R->A.rows; ++r)
        for (int64_t c = 0; c < R->A.cols; ++c)
            A_ue[r * R->A.cols + c] = (int8_t)*mat_at(&R->A, r, c);
    for (int64_t r = 0; r < R->B.rows; ++r)
        for (int64_t c = 0; c < R->B.cols; ++c)
            B_eu[r * R->B.cols + c] = (int8_t)*mat_at(&R->B, r, c);
}

void orc_result_copy_meta(orc_result_t *R, int64_t *S,
                          int64_t *piA_src, int64_t *piA_w, int64_t *piB_src, int64_t *piB_w)
{
    memcpy(S, R->S.v, (size_t)R->S.len * sizeof(int64_t));
    memcpy(piA_src, R->piA_src.v, (size_t)R->piA_src.len * sizeof(int64_t));
    memcpy(piA_w, R->piA_w.v, (size_t)R->piA_w.len * sizeof(int64_t));
    memcpy(piB_src, R->piB_src.v, (size_t)R->piB_src.len * sizeof(int64_t));
    memcpy(piB_w, R->piB_w.v, (size_t)R->piB_w.len * sizeof(int64_t));
}

/* the record of the splits: number of splits, then (into caller buffers) col_parent (d') and the
 * triples (3 per split) */
int64_t orc_result_num_ops(const orc_result_t *R) { return R->tr.ops.len / 3; }

void orc_result_copy_trace(const orc_result_t *R, int64_t *col_parent, int64_t *ops)
{
    memcpy(col_parent, R->tr.col_parent.v, (size_t)R->tr.col_parent.len * sizeof(int64_t));
    memcpy(ops, R->tr.ops.v, (size_t)R->tr.ops.len * sizeof(int64_t));
}
