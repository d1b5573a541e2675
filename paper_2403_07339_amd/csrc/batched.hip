// Strided-batched exact integer GEMMs: the products of a Transformer come in batches of equal shape
// (Sec. 1 "Notations": P = Q K^T and O = M V and their gradients once per sequence and head; a linear
// layer is the batch of one).  Each item runs the whole path -- the RTN step alpha_p / (0.5 beta) of
// Eq. (quantized_A) from the item's own percentile, quantize + scan of both operands, unpack plan,
// digit scatter, int8 GEMM with the recombination and the dequantisation of Eq. (quantized_gemm) in
// its epilogue -- with the steps kept in device memory from the kernel that forms them to the kernels
// that divide and multiply by them, so that the host reads nothing back between the stages but the
// sizes of the unpacked problem (once per item, inside the plan call).  The item loop runs here, on
// the host, over one context object whose buffers are reused from item to item and call to call.
#include "common.h"

#include <algorithm>
#include <cstring>
#include <new>

namespace imu {
int quantize_pair(const float *A, int64_t n, int64_t sa_r, int64_t sa_c, float scale_A, const float *scale_A_dev,
                  int32_t *QA, int64_t ldqa, const imunpack_stats_t *stA, const float *B, int64_t h, int64_t sb_r,
                  int64_t sb_c, float scale_B, const float *scale_B_dev, int32_t *QB, int64_t ldqb,
                  const imunpack_stats_t *stB, int64_t d, int b, int32_t *status, hipStream_t stream);
int gemm_impl(imunpack_plan_t *p, const int8_t *A_ue, const int8_t *B_eu, void *workspace, int64_t *C_int,
              float *C_fp, int64_t ldc, float scale_A, float scale_B, const float *scale_a_dev,
              const float *scale_b_dev, int fuse, imunpack_stream_t stream);

__global__ void clear_flag_kernel(int32_t *any) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *any = 0;
}

// status[item] |= what the two quantize passes and the two percentile passes of the item flagged
__global__ void gather_status_kernel(const int32_t *flags, int nflags, int32_t *any) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        int bad = 0;
        for (int i = 0; i < nflags; ++i) bad |= flags[i];
        if (bad) atomicOr(any, 1);
    }
}
}  // namespace imu

struct imunpack_batch {
    imunpack_plan_t *plan;
    char *arena;           // Q_A, Q_B, statistics, OB lists, steps, flags, percentile workspace
    size_t arena_bytes;
    int8_t *ue;            // A store and B_eu
    size_t ue_bytes;
    void *ws;              // int64 unpacked product for items that cannot take the fused launch
    size_t ws_bytes;
    int32_t *pin_any;      // pinned: whether any item flagged NaN / Inf / overflow
};

using namespace imu;

static int grow(void **ptr, size_t *have, size_t want) {
    if (*have >= want) return IMUNPACK_OK;
    if (*ptr) IMU_HIP(hipFree(*ptr));
    *ptr = nullptr;
    *have = 0;
    const size_t take = want + want / 4;
    if (hipMalloc(ptr, take) != hipSuccess) {
        (void)hipGetLastError();
        *ptr = nullptr;
        return IMUNPACK_ENOMEM;
    }
    *have = take;
    return IMUNPACK_OK;
}

extern "C" int imunpack_batch_destroy(imunpack_batch_t *c) {
    if (!c) return IMUNPACK_OK;
    int rc = IMUNPACK_OK;
    if (c->plan) rc = imunpack_plan_destroy(c->plan);
    if (c->arena) (void)hipFree(c->arena);
    if (c->ue) (void)hipFree(c->ue);
    if (c->ws) (void)hipFree(c->ws);
    if (c->pin_any) (void)hipHostFree(c->pin_any);
    delete c;
    return rc;
}

extern "C" int imunpack_gemm_batched(const float *A, int64_t sa_b, int64_t sa_r, int64_t sa_c,
                                     const float *B, int64_t sb_b, int64_t sb_r, int64_t sb_c,
                                     int64_t batch, int64_t n, int64_t d, int64_t h,
                                     double p, float beta_A, float beta_B, int b, int strategy_A, int strategy_B,
                                     float *C, int64_t sc_b, int64_t ldc, imunpack_batch_t **ctx,
                                     imunpack_stream_t stream) {
    if (!A || !B || !C || !ctx || batch < 0 || n <= 0 || d <= 0 || h <= 0 || ldc < h || sa_r < 1 || sa_c < 1 ||
        sb_r < 1 || sb_c < 1 || sa_b < 0 || sb_b < 0 || sc_b < 0 || b < 2 || b > 8 || strategy_A < 0 || strategy_A > 2 ||
        strategy_B < 0 || strategy_B > 2 || !(p > 0.0) || !(p <= 100.0) || !(beta_A > 0.0f) || !(beta_B > 0.0f))
        return IMUNPACK_EINVAL;
    if (n > (1 << 24) || d > (1 << 24) || h > (1 << 24) || n * d >= ((int64_t)1 << 32) || h * d >= ((int64_t)1 << 32))
        return IMUNPACK_EINVAL;
    if (batch == 0) return IMUNPACK_OK;
    hipStream_t st = (hipStream_t)stream;
    imunpack_batch_t *c = *ctx;
    if (!c) {
        c = new (std::nothrow) imunpack_batch();
        if (!c) return IMUNPACK_ENOMEM;
        memset(c, 0, sizeof(*c));
        if (hipHostMalloc((void **)&c->pin_any, sizeof(int32_t), hipHostMallocDefault) != hipSuccess) {
            (void)hipGetLastError();
            delete c;
            return IMUNPACK_ENOMEM;
        }
        *ctx = c;
    }
    // ---- one arena for everything whose size the shapes fix
    const int64_t capA = strategy_A == IMUNPACK_BOTH ? std::max<int64_t>(4096, n * d / 64) : 0;
    const int64_t capB = strategy_B == IMUNPACK_BOTH ? std::max<int64_t>(4096, h * d / 64) : 0;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off = (off + bytes + 255) & ~(size_t)255; return at; };
    const size_t oQa = take((size_t)n * d * 4), oQb = take((size_t)h * d * 4);
    const size_t oSa = take((size_t)2 * (n + d) * 4), oSb = take((size_t)2 * (h + d) * 4);
    const size_t oLa = take((size_t)3 * capA * 4), oLb = take((size_t)3 * capB * 4);
    const size_t oSmall = take(256);   // steps (2 floats), OB counts (2), flags (4), any (1)
    const size_t oWs = take(IMUNPACK_PERCENTILE_WORKSPACE_BYTES);
    IMU_TRY(grow((void **)&c->arena, &c->arena_bytes, off));
    int32_t *Qa = (int32_t *)(c->arena + oQa), *Qb = (int32_t *)(c->arena + oQb);
    int32_t *sA = (int32_t *)(c->arena + oSa), *sB = (int32_t *)(c->arena + oSb);
    float *steps = (float *)(c->arena + oSmall);
    int32_t *small = (int32_t *)(c->arena + oSmall);
    int32_t *obcnt = small + 2, *flags = small + 4, *any = small + 8;
    void *pws = c->arena + oWs;
    imunpack_stats_t stA = {sA, sA + n, sA + n + d, sA + 2 * n + d, capA ? (int32_t *)(c->arena + oLa) : nullptr, capA,
                            capA ? obcnt : nullptr};
    imunpack_stats_t stB = {sB, sB + h, sB + h + d, sB + 2 * h + d, capB ? (int32_t *)(c->arena + oLb) : nullptr, capB,
                            capB ? obcnt + 1 : nullptr};
    hipLaunchKernelGGL(clear_flag_kernel, dim3(1), dim3(64), 0, st, any);
    for (int64_t i = 0; i < batch; ++i) {
        const float *Ai = A + i * sa_b, *Bi = B + i * sb_b;
        // the steps stay on the device: percentile -> step -> division in the quantizer -> product in the epilogue
        IMU_TRY(imunpack_rtn_step(Ai, n, d, sa_r, sa_c, p, beta_A, steps, flags, pws, st));
        IMU_TRY(imunpack_rtn_step(Bi, h, d, sb_r, sb_c, p, beta_B, steps + 1, flags + 1, pws, st));
        IMU_TRY(quantize_pair(Ai, n, sa_r, sa_c, 1.0f, steps, Qa, d, &stA, Bi, h, sb_r, sb_c, 1.0f, steps + 1, Qb, d, &stB, d,
                              b, flags + 2, st));
        hipLaunchKernelGGL(gather_status_kernel, dim3(1), dim3(64), 0, st, flags, 4, any);
        IMU_TRY(imunpack_plan(Qa, n, d, d, Qb, h, d, b, strategy_A, strategy_B, &stA, &stB, &c->plan, st));
        // digits of at most three bits: six-bit floating-point codes on the f8f6f4 matrix instruction (the
        // request stays with the context's plan object)
        if (b <= 4 && imunpack_plan_digits(c->plan) != IMUNPACK_DIGITS_FP6)
            IMU_TRY(imunpack_plan_set_digits(c->plan, IMUNPACK_DIGITS_FP6));
        size_t ba = 0, bb = 0, bw = 0;
        IMU_TRY(imunpack_unpacked_bytes(c->plan, &ba, &bb, &bw));
        const size_t ba_pad = (ba + 255) & ~(size_t)255;
        IMU_TRY(grow((void **)&c->ue, &c->ue_bytes, ba_pad + bb));
        IMU_TRY(imunpack_unpack(c->plan, Qa, d, Qb, d, c->ue, c->ue + ba_pad, st));
        float *Ci = C + i * sc_b;
        int rc = gemm_impl(c->plan, c->ue, c->ue + ba_pad, c->ws_bytes >= bw ? c->ws : nullptr, nullptr, Ci, ldc, 1.0f, 1.0f,
                           steps, steps + 1, 1, st);
        if (rc == IMUNPACK_ERANGE && c->ws_bytes < bw) {  // the fused launch is not exact for this item: un-fused path
            IMU_HIP(hipStreamSynchronize(st));             // the buffer may still be in use by an earlier item
            IMU_TRY(grow(&c->ws, &c->ws_bytes, bw));
            rc = gemm_impl(c->plan, c->ue, c->ue + ba_pad, c->ws, nullptr, Ci, ldc, 1.0f, 1.0f, steps, steps + 1, 1, st);
        }
        IMU_TRY(rc);
    }
    IMU_HIP(hipMemcpyAsync(c->pin_any, any, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    IMU_HIP(hipStreamSynchronize(st));
    return *c->pin_any ? IMUNPACK_ERANGE : IMUNPACK_OK;
}
