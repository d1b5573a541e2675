/* Host-side sanitizer run of the CPU oracle: compiled together with oracle/imunpack_oracle.c under
 * -fsanitize=address,undefined by tests/test_sanitizers.py.  Walks every exported routine over small
 * seeded inputs (all nine strategy pairs, several bit widths, shapes that make the growing matrices
 * reallocate) and checks the product identity, so that an out-of-bounds access, a leak or signed
 * overflow inside the oracle stops the test run. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct orc_result orc_result_t;
int orc_rtn_quantize(const float *x, int64_t count, float scale, int32_t *q);
void orc_int_gemm(const int32_t *A, int64_t n, int64_t d, const int32_t *B, int64_t h, int64_t *C);
void orc_dequantize(const int64_t *C, int64_t count, float scale_a, float scale_b, double *out);
int32_t orc_digit(int32_t v, int32_t s, int i);
orc_result_t *orc_unpack_pair(const int32_t *A, int64_t n, int64_t d, const int32_t *B, int64_t h, int b,
                              int strategy_a, int strategy_b, int recount);
void orc_result_dims(const orc_result_t *R, int64_t *n_u, int64_t *d_u, int64_t *h_u);
void orc_result_copy(orc_result_t *R, int32_t *A_ue, int32_t *B_eu, int64_t *S, int64_t *piA_src, int64_t *piA_w,
                     int64_t *piB_src, int64_t *piB_w);
void orc_result_copy_i8(orc_result_t *R, int8_t *A_ue, int8_t *B_eu);
void orc_result_copy_meta(orc_result_t *R, int64_t *S, int64_t *piA_src, int64_t *piA_w, int64_t *piB_src, int64_t *piB_w);
int64_t orc_result_num_ops(const orc_result_t *R);
void orc_result_copy_trace(const orc_result_t *R, int64_t *col_parent, int64_t *ops);
int32_t orc_result_max_abs(const orc_result_t *R);
void orc_unpacked_product_at(const orc_result_t *R, const int64_t *rows, const int64_t *cols, int64_t count, int64_t *out);
void orc_scaled_matmul(const int32_t *A, int64_t n, int64_t d, const int32_t *B, int64_t h, const int64_t *S, int64_t *C);
void orc_apply_pi(const int64_t *C_u, int64_t n_u, int64_t h_u, const int64_t *piA_src, const int64_t *piA_w,
                  const int64_t *piB_src, const int64_t *piB_w, int64_t n, int64_t h, int64_t *C_out);
void orc_result_free(orc_result_t *R);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void) {
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 32);
}

int main(void) {
    int failures = 0;
    for (int b = 2; b <= 8; b += 3) {
        const int32_t s = 1 << (b - 1);
        for (int sa = 0; sa < 3; ++sa)
            for (int sb = 0; sb < 3; ++sb) {
                const int64_t n = 5 + rnd() % 4, d = 9 + rnd() % 5, h = 3 + rnd() % 4;
                float *xf = malloc(sizeof(float) * n * d);
                int32_t *A = malloc(sizeof(int32_t) * n * d), *B = malloc(sizeof(int32_t) * h * d);
                for (int64_t t = 0; t < n * d; ++t) xf[t] = ((int)(rnd() % 2001) - 1000) * 0.37f * ((rnd() % 7 == 0) ? (float)(s * s) : 1.0f);
                if (orc_rtn_quantize(xf, n * d, 40.0f, A)) ++failures;
                for (int64_t t = 0; t < h * d; ++t) {
                    B[t] = (int32_t)(rnd() % (2 * s - 1)) - (s - 1);
                    if (rnd() % 5 == 0) B[t] *= s * (int32_t)(1 + rnd() % (uint32_t)s);
                }
                int64_t *want = malloc(sizeof(int64_t) * n * h);
                orc_int_gemm(A, n, d, B, h, want);
                orc_result_t *R = orc_unpack_pair(A, n, d, B, h, b, sa, sb, (int)(rnd() & 1));
                int64_t nu, du, hu;
                orc_result_dims(R, &nu, &du, &hu);
                int32_t *Au = malloc(sizeof(int32_t) * nu * du), *Bu = malloc(sizeof(int32_t) * hu * du);
                int8_t *A8 = malloc((size_t)(nu * du)), *B8 = malloc((size_t)(hu * du));
                int64_t *S = malloc(sizeof(int64_t) * du), *pas = malloc(sizeof(int64_t) * nu), *paw = malloc(sizeof(int64_t) * nu),
                        *pbs = malloc(sizeof(int64_t) * hu), *pbw = malloc(sizeof(int64_t) * hu);
                orc_result_copy(R, Au, Bu, S, pas, paw, pbs, pbw);
                orc_result_copy_i8(R, A8, B8);
                orc_result_copy_meta(R, S, pas, paw, pbs, pbw);
                int64_t nops = orc_result_num_ops(R);
                int64_t *par = malloc(sizeof(int64_t) * du), *ops = malloc(sizeof(int64_t) * 3 * (nops > 0 ? nops : 1));
                orc_result_copy_trace(R, par, ops);
                if (orc_result_max_abs(R) > s - 1) ++failures;
                if (nops != (nu - n) + (hu - h) + (du - d)) ++failures;
                int64_t *Cu = malloc(sizeof(int64_t) * nu * hu), *got = malloc(sizeof(int64_t) * n * h);
                orc_scaled_matmul(Au, nu, du, Bu, hu, S, Cu);
                orc_apply_pi(Cu, nu, hu, pas, paw, pbs, pbw, n, h, got);
                for (int64_t t = 0; t < n * h; ++t) failures += got[t] != want[t];
                int64_t rows[2] = {0, n - 1}, cols[2] = {h - 1, 0}, at[2];
                orc_unpacked_product_at(R, rows, cols, 2, at);
                failures += at[0] != want[0 * h + h - 1] || at[1] != want[(n - 1) * h];
                double *deq = malloc(sizeof(double) * n * h);
                orc_dequantize(want, n * h, 0.5f, 0.25f, deq);
                failures += deq[0] != 0.125 * (double)want[0];
                for (int i = 0; i < 5; ++i) failures += abs(orc_digit((int32_t)rnd(), s, i)) > s - 1;
                orc_result_free(R);
                free(xf); free(A); free(B); free(want); free(Au); free(Bu); free(A8); free(B8); free(S); free(pas);
                free(paw); free(pbs); free(pbw); free(par); free(ops); free(Cu); free(got); free(deq);
            }
    }
    printf("oracle sanitizer walk: %d failures\n", failures);
    return failures != 0;
}
