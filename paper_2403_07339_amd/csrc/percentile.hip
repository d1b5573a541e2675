// alpha_p(A) of Sec. 2 (the sentence after Eq. (quantized_A)): the p-th percentile of the magnitudes
// of a matrix, i.e. the smallest magnitude a such that at least p % of the entries lie in [-a, a].
// That is an order statistic: the k-th smallest |x| with k = ceil(p N / 100).
//
// The magnitude of a binary32 number, read as a 31-bit unsigned integer, orders like the magnitude
// itself, so the k-th smallest is found by a radix select over those integers, most significant
// digit first: three passes over the matrix (11 + 10 + 10 bits).  A pass counts, per value of its
// digit, the entries that agree with the digits fixed so far (a histogram in LDS per workgroup, merged
// with one atomic per non-empty bin); a single workgroup then picks the digit value whose cumulative
// count reaches k, fixes it and lowers k by the count below it.  HBM-bound: 12 bytes read per entry,
// nothing written but 8 KiB of counters.  Everything stays on the stream; the caller reads *alpha
// when it needs the number.
#include "common.h"

#include <cmath>
#include <mutex>

namespace imu {

constexpr int kSelBins = 2048;      // bins of the widest pass
constexpr int kSelThreads = 256;
constexpr int kSelItems = 4;        // 16-byte pieces per thread and step, loaded side by side

struct SelState {
    unsigned prefix;           // digits fixed so far (in place)
    unsigned prefix_mask;      // which bits those are
    unsigned long long k;      // rank wanted among the entries that agree with the prefix (1-based)
    unsigned maxbits;          // largest magnitude seen (as its bit pattern), gathered by the first pass
    unsigned pad_;
};

// Workspace layout: kSelBins counters, then the state.
__device__ __forceinline__ unsigned *sel_hist(void *ws) { return reinterpret_cast<unsigned *>(ws); }
__device__ __forceinline__ SelState *sel_state(void *ws) {
    return reinterpret_cast<SelState *>(reinterpret_cast<unsigned *>(ws) + kSelBins);
}

__global__ void select_init_kernel(void *ws, unsigned long long k, int32_t *status) {
    unsigned *hist = sel_hist(ws);
    for (int i = threadIdx.x; i < kSelBins; i += blockDim.x) hist[i] = 0;
    if (threadIdx.x == 0) {
        SelState *st = sel_state(ws);
        st->prefix = 0;
        st->prefix_mask = 0;
        st->k = k;
        st->maxbits = 0;
        if (status) *status = 0;
    }
}

// The matrix as nslow lines of nfast entries: entry (l, f) at X[l * stride_slow + f * stride_fast].
// VEC: stride_fast == 1, nfast % 4 == 0, lines 16-byte aligned.
template <bool VEC>
__global__ __launch_bounds__(kSelThreads) void select_count_kernel(const float *__restrict__ X, int64_t nslow,
                                                                   int64_t nfast, int64_t stride_slow,
                                                                   int64_t stride_fast, void *ws, int shift,
                                                                   int nbins, int32_t *status) {
    __shared__ unsigned lh[kSelBins];
    for (int i = threadIdx.x; i < nbins; i += kSelThreads) lh[i] = 0;
    __syncthreads();
    const SelState st = *sel_state(ws);
    const unsigned bmask = (unsigned)nbins - 1u;
    bool nan = false;
    unsigned umax = 0;
    auto take = [&](float x) {
        const unsigned u = __float_as_uint(x) & 0x7fffffffu;
        nan = nan || u > 0x7f800000u;
        umax = max(umax, u);
        if ((u & st.prefix_mask) == st.prefix) atomicAdd(&lh[(u >> shift) & bmask], 1u);
    };
    const int64_t per_line = VEC ? nfast / 4 : nfast;
    const int64_t items = nslow * per_line;
    const int64_t stride = (int64_t)gridDim.x * kSelThreads;
    for (int64_t base = (int64_t)blockIdx.x * kSelThreads + threadIdx.x; base < items; base += stride * kSelItems) {
        if (VEC) {
            float4 v[kSelItems];
#pragma unroll
            for (int u = 0; u < kSelItems; ++u) {
                const int64_t it = base + u * stride;
                v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (it < items) {
                    const int64_t l = it / per_line, f = it - l * per_line;
                    v[u] = *reinterpret_cast<const float4 *>(X + l * stride_slow + 4 * f);
                }
            }
#pragma unroll
            for (int u = 0; u < kSelItems; ++u) {
                if (base + u * stride < items) {
                    take(v[u].x); take(v[u].y); take(v[u].z); take(v[u].w);
                }
            }
        } else {
            float v[kSelItems];
#pragma unroll
            for (int u = 0; u < kSelItems; ++u) {
                const int64_t it = base + u * stride;
                v[u] = 0.f;
                if (it < items) {
                    const int64_t l = it / per_line, f = it - l * per_line;
                    v[u] = X[l * stride_slow + f * stride_fast];
                }
            }
#pragma unroll
            for (int u = 0; u < kSelItems; ++u)
                if (base + u * stride < items) take(v[u]);
        }
    }
    __syncthreads();
    unsigned *hist = sel_hist(ws);
    for (int i = threadIdx.x; i < nbins; i += kSelThreads)
        if (lh[i]) atomicAdd(&hist[i], lh[i]);
    if (status && __ballot(nan) && (threadIdx.x & 63) == 0) atomicOr(status, 1);
    if (shift == 20) {  // first pass: the largest magnitude, for the step's fall-back
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) umax = max(umax, (unsigned)__shfl_xor((int)umax, off, 64));
        if ((threadIdx.x & 63) == 0 && umax) atomicMax(&sel_state(ws)->maxbits, umax);
    }
}

// The RTN step of Eq. (quantized_A): beta integers cover [-alpha_p, alpha_p], so one step is
// alpha_p / (0.5 beta), formed once in binary32.  A matrix whose p-th percentile is 0 (mostly zeros)
// falls back to its largest magnitude, an all-zero (or non-finite) one to 1.  *step holds alpha_p on
// entry (the selection's last pass wrote it there) and the step on exit.
__global__ void rtn_step_kernel(void *ws, float half_beta, float *step) {
    float a = *step;
    if (!(a > 0.0f)) a = __uint_as_float(sel_state(ws)->maxbits);
    *step = (a > 0.0f && a < __uint_as_float(0x7f800000u)) ? __fdiv_rn(a, half_beta) : 1.0f;
}

// One workgroup: the bin whose cumulative count reaches k becomes the next digit.
__global__ __launch_bounds__(1024) void select_pick_kernel(void *ws, int shift, int nbins, float *alpha) {
    __shared__ unsigned long long part[1024];
    __shared__ int s_bin;
    __shared__ unsigned long long s_below;
    unsigned *hist = sel_hist(ws);
    SelState *st = sel_state(ws);
    const unsigned long long k = st->k;
    // thread t owns bins [t * per, t * per + per)
    const int per = (nbins + 1023) / 1024;
    unsigned long long mine = 0;
    for (int j = 0; j < per; ++j) {
        const int b = threadIdx.x * per + j;
        if (b < nbins) mine += hist[b];
    }
    part[threadIdx.x] = mine;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {  // inclusive scan
        const unsigned long long add = threadIdx.x >= (unsigned)off ? part[threadIdx.x - off] : 0ull;
        __syncthreads();
        part[threadIdx.x] += add;
        __syncthreads();
    }
    const unsigned long long incl = part[threadIdx.x], excl = incl - mine;
    if (excl < k && k <= incl) {  // exactly one thread, as 1 <= k <= the total count
        unsigned long long run = excl;
        for (int j = 0; j < per; ++j) {
            const int b = threadIdx.x * per + j;
            if (b >= nbins) break;
            const unsigned c = hist[b];
            if (k <= run + c) {
                s_bin = b;
                s_below = run;
                break;
            }
            run += c;
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nbins; i += 1024) hist[i] = 0;  // ready for the next pass (and the next call)
    if (threadIdx.x == 0) {
        const unsigned prefix = st->prefix | ((unsigned)s_bin << shift);
        st->prefix = prefix;
        st->prefix_mask |= ((unsigned)nbins - 1u) << shift;
        st->k = k - s_below;
        if (shift == 0) *alpha = __uint_as_float(prefix);
    }
}

}  // namespace imu

using namespace imu;

static int run_percentile(const float *X, int64_t rows, int64_t cols, int64_t sx_r, int64_t sx_c, double p,
                          float *alpha, int32_t *status_flag, void *workspace, hipStream_t st) {
    static_assert(IMUNPACK_PERCENTILE_WORKSPACE_BYTES >= kSelBins * sizeof(unsigned) + sizeof(SelState), "workspace");
    const int64_t N = rows * cols;
    double kd = std::ceil(p * (double)N / 100.0);
    if (kd < 1.0) kd = 1.0;
    if (kd > (double)N) kd = (double)N;
    const unsigned long long k = (unsigned long long)kd;
    // the unit-stride axis, if there is one, runs fastest
    int64_t nslow = rows, nfast = cols, sslow = sx_r, sfast = sx_c;
    if (sx_c != 1 && sx_r == 1) { nslow = cols; nfast = rows; sslow = sx_c; sfast = 1; }
    const bool vec = sfast == 1 && (nfast % 4) == 0 && (sslow % 4) == 0 && ((uintptr_t)X % 16) == 0;
    const int64_t items = nslow * (vec ? nfast / 4 : nfast);
    int64_t blocks = (items + (int64_t)kSelThreads * kSelItems - 1) / ((int64_t)kSelThreads * kSelItems);
    if (blocks > 1024) blocks = 1024;  // four per CU: every workgroup merges its histogram with atomics on the same few counters
    if (blocks < 1) blocks = 1;
    // the init kernel clears the counters and the state: whatever an earlier call left in the workspace is gone
    hipLaunchKernelGGL(select_init_kernel, dim3(1), dim3(256), 0, st, workspace, k, status_flag);
    const int shifts[3] = {20, 10, 0}, bins[3] = {2048, 1024, 1024};
    for (int pass = 0; pass < 3; ++pass) {
        if (vec)
            hipLaunchKernelGGL(select_count_kernel<true>, dim3((unsigned)blocks), dim3(kSelThreads), 0, st, X, nslow, nfast,
                               sslow, sfast, workspace, shifts[pass], bins[pass], pass == 0 ? status_flag : nullptr);
        else
            hipLaunchKernelGGL(select_count_kernel<false>, dim3((unsigned)blocks), dim3(kSelThreads), 0, st, X, nslow, nfast,
                               sslow, sfast, workspace, shifts[pass], bins[pass], pass == 0 ? status_flag : nullptr);
        hipLaunchKernelGGL(select_pick_kernel, dim3(1), dim3(1024), 0, st, workspace, shifts[pass], bins[pass], alpha);
    }
    return launch_status();
}

extern "C" int imunpack_percentile(const float *X, int64_t rows, int64_t cols, int64_t sx_r, int64_t sx_c,
                                   double p, float *alpha, int32_t *status_flag, void *workspace,
                                   imunpack_stream_t stream) {
    if (!X || !alpha || !workspace || rows <= 0 || cols <= 0 || sx_r < 1 || sx_c < 1 || !(p > 0.0) || !(p <= 100.0))
        return IMUNPACK_EINVAL;
    if (rows > (int64_t)1 << 31 || cols > (int64_t)1 << 31 || rows * cols >= (int64_t)1 << 32) return IMUNPACK_EINVAL;
    return run_percentile(X, rows, cols, sx_r, sx_c, p, alpha, status_flag, workspace, (hipStream_t)stream);
}

extern "C" int imunpack_rtn_step(const float *X, int64_t rows, int64_t cols, int64_t sx_r, int64_t sx_c, double p,
                                 float beta, float *step, int32_t *status_flag, void *workspace,
                                 imunpack_stream_t stream) {
    if (!X || !step || !workspace || rows <= 0 || cols <= 0 || sx_r < 1 || sx_c < 1 || !(p > 0.0) || !(p <= 100.0) ||
        !(beta > 0.0f) || !(beta < 3.0e38f))
        return IMUNPACK_EINVAL;
    if (rows > (int64_t)1 << 31 || cols > (int64_t)1 << 31 || rows * cols >= (int64_t)1 << 32) return IMUNPACK_EINVAL;
    IMU_TRY(run_percentile(X, rows, cols, sx_r, sx_c, p, step, status_flag, workspace, (hipStream_t)stream));
    hipLaunchKernelGGL(rtn_step_kernel, dim3(1), dim3(1), 0, (hipStream_t)stream, workspace, (float)(0.5 * (double)beta), step);
    return launch_status();
}

// ---- the same selection for callers that cannot allocate ------------------------------------------
// The counters and the selection state live in a file-scope device array instead of a caller
// workspace.  Every GPU holds its own copy of the array at its own address, which the host learns
// once per device; host code only ever uses that address, never the array's name.
static __device__ __align__(256) unsigned char scratch[IMUNPACK_PERCENTILE_WORKSPACE_BYTES];
static constexpr int kMaxDevices = 64;
static std::mutex g_scratch_lock;
static void *g_scratch_ptr[kMaxDevices];  // per device, nullptr until that device's first call

extern "C" int imunpack_percentile_static(const float *X, int64_t rows, int64_t cols, int64_t sx_r, int64_t sx_c,
                                          double p, float *alpha, int32_t *status_flag,
                                          imunpack_stream_t stream) {
    if (!X || !alpha || rows <= 0 || cols <= 0 || sx_r < 1 || sx_c < 1 || !(p > 0.0) || !(p <= 100.0))
        return IMUNPACK_EINVAL;
    // the scratch array's counters are 32 bits wide: more entries than they can count are refused
    if (rows > (int64_t)1 << 31 || cols > (int64_t)1 << 31 || rows * cols > IMUNPACK_PERCENTILE_STATIC_MAX_ENTRIES)
        return IMUNPACK_ERANGE;
    int dev = -1;
    IMU_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return IMUNPACK_EINVAL;
    void *ws = nullptr;
    {
        std::lock_guard<std::mutex> hold(g_scratch_lock);
        if (!g_scratch_ptr[dev]) {
            void *ptr = nullptr;
            IMU_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));  // the current device's copy
            if (!ptr) return IMUNPACK_EHIP;
            g_scratch_ptr[dev] = ptr;
        }
        ws = g_scratch_ptr[dev];
    }
    return run_percentile(X, rows, cols, sx_r, sx_c, p, alpha, status_flag, ws, (hipStream_t)stream);
}
