// RTN quantisation (Sec. 2, Eq. quantized_A) fused with the heavy-hitter scan (Sec. 4, IB/OB
// definition): one pass reads fp32 (or int32 for the stand-alone scan), writes int32 and reduces
// the OB count and the largest magnitude of every row and every column.
//
// HBM-bound: 4 B read + 4 B written per element (4 B read for the stand-alone scan).
#include "common.h"

#include <algorithm>

namespace imu {

// The RTN step: a value of the call, or (callers that keep it on the device) read from memory.  A step
// that is not a positive finite number turns every quotient into a flagged 0.
__device__ __forceinline__ float step_of(float value, const float *ptr) {
    const float s = ptr ? *ptr : value;
    return (s > 0.0f && s < 3.0e38f) ? s : __uint_as_float(0x7fc00000u);
}

// q = rint(x / scale): correctly rounded binary32 division, then round half to even.
__device__ __forceinline__ int32_t rtn_one(float x, float scale, int &bad) {
    float r = rintf(__fdiv_rn(x, scale));
    if (!(fabsf(r) < 2147483648.0f)) {  // also catches NaN and Inf
        bad = 1;
        return 0;
    }
    return (int32_t)r;
}

// 16 bytes that are read exactly once
__device__ __forceinline__ int4 load_nt16(const int32_t *p) {
    typedef int v4i_nt __attribute__((ext_vector_type(4)));
    const v4i_nt t = __builtin_nontemporal_load(reinterpret_cast<const v4i_nt *>(p));
    return make_int4(t[0], t[1], t[2], t[3]);
}

__device__ __forceinline__ int iabs_sat(int32_t v) { return v < 0 ? (v == INT32_MIN ? INT32_MAX : -v) : v; }

// Column partials of one workgroup: wave w holds, per lane, the statistics of its own columns over
// the rows that wave visited; they are combined through LDS and one atomic per column is issued.
template <int COLS_PER_LANE>
__device__ __forceinline__ void flush_columns(int (&ccnt)[COLS_PER_LANE], int (&cmax)[COLS_PER_LANE],
                                              int64_t c_first, int64_t cols, int32_t *colcnt,
                                              int32_t *colmax, int *lds /* [2][4][64*CPL] */) {
    constexpr int W = 64 * COLS_PER_LANE;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int u = 0; u < COLS_PER_LANE; ++u) {
        lds[(0 * 4 + wave) * W + lane * COLS_PER_LANE + u] = ccnt[u];
        lds[(1 * 4 + wave) * W + lane * COLS_PER_LANE + u] = cmax[u];
    }
    __syncthreads();
    for (int c = threadIdx.x; c < W; c += 256) {
        int cnt = 0, mx = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            cnt += lds[(0 * 4 + w) * W + c];
            mx = max(mx, lds[(1 * 4 + w) * W + c]);
        }
        int64_t col = c_first + c;
        if (col < cols) {
            if (colcnt && cnt) atomicAdd(&colcnt[col], cnt);
            if (colmax && mx) atomicMax(&colmax[col], mx);
        }
    }
}


// OB entries found by a workgroup are staged in LDS and appended to the global list with a single
// atomic per workgroup (one atomic per wave-row would serialise on the list's counter).
constexpr int kObStage = 1024;
struct ObStage {
    int count;
    int base;
    int32_t row[kObStage], col[kObStage], val[kObStage];
};

__device__ __forceinline__ void ob_push(ObStage *sg, int pos, int32_t r, int32_t c, int32_t v, int32_t *ob,
                                        int ob_cap, int32_t *ob_count) {
    if (pos < kObStage) {
        sg->row[pos] = r;
        sg->col[pos] = c;
        sg->val[pos] = v;
    } else {  // stage full (an almost entirely OB tile): append directly
        const int g = atomicAdd(ob_count, 1);
        if (g < ob_cap) {
            ob[g] = r;
            ob[ob_cap + g] = c;
            ob[2 * ob_cap + g] = v;
        }
    }
}

__device__ __forceinline__ void ob_flush(ObStage *sg, int32_t *ob, int ob_cap, int32_t *ob_count) {
    __syncthreads();
    const int n = min(sg->count, kObStage);
    if (n == 0) return;  // uniform
    if (threadIdx.x == 0) sg->base = atomicAdd(ob_count, n);
    __syncthreads();
    const int base = sg->base;
    for (int t = threadIdx.x; t < n; t += blockDim.x) {
        const int g = base + t;
        if (g < ob_cap) {
            ob[g] = sg->row[t];
            ob[ob_cap + g] = sg->col[t];
            ob[2 * ob_cap + g] = sg->val[t];
        }
    }
}

// Fast path: unit column stride, 16-byte aligned rows.  Workgroup = rows_per_wg rows x 256 columns;
// a wave reads one 1 KiB row segment per instruction (float4 per lane).
struct VecOperand {
    const void *X;
    int64_t rows, ldx;
    float scale_val;
    const float *scale_ptr;
    int32_t *Q;
    int64_t ldq;
    int32_t *rowcnt, *colcnt, *rowmax, *colmax, *status, *ob;
    int ob_cap;
    int32_t *ob_count;
    int rows_per_wg;
    int row_blocks;  // workgroups along the rows
};

template <bool FROM_FLOAT>
__device__ __forceinline__ void qscan_vec_body(const VecOperand &a, int64_t cols, int s, int by, int *lds, ObStage &stage) {
    const void *__restrict__ Xv = a.X;
    int32_t *__restrict__ Q = a.Q;
    const int64_t rows = a.rows, ldx = a.ldx, ldq = a.ldq;
    int32_t *rowcnt = a.rowcnt, *colcnt = a.colcnt, *rowmax = a.rowmax, *colmax = a.colmax, *status = a.status;
    int32_t *ob = a.ob, *ob_count = a.ob_count;
    const int ob_cap = a.ob_cap, rows_per_wg = a.rows_per_wg;
    if (ob) {
        if (threadIdx.x == 0) stage.count = 0;
        __syncthreads();
    }
    const float scale = step_of(a.scale_val, a.scale_ptr);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    // Workgroup ids are dealt round-robin to the 8 XCDs; rotating the column block with the row block
    // lets every XCD touch every column block (and so every memory channel) while the workgroups that
    // run together still cover whole rows.
    const int cbx = (blockIdx.x + by) % gridDim.x;
    const int64_t c0 = (int64_t)cbx * 256 + lane * 4;
    const int64_t r_base = (int64_t)by * rows_per_wg;
    const int64_t r_end = min(rows, r_base + rows_per_wg);
    int ccnt[4] = {0, 0, 0, 0}, cmax[4] = {0, 0, 0, 0};
    int bad = 0;
    const bool in_cols = c0 < cols;  // cols % 4 == 0 on this path
    // four rows per step: their loads are issued together, before any of them is used (keeping the next
    // step's loads in flight as well was slower: 0.113 against 0.105 ms for both operands of the benchmark)
    for (int64_t rb = r_base + wave; rb < r_end; rb += 16) {  // uniform per wave
        int4 raw[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int64_t r = rb + 4 * v;
            raw[v] = make_int4(0, 0, 0, 0);
            if (in_cols && r < r_end)  // read once: non-temporal (0.125 -> 0.109 ms)
                raw[v] = load_nt16(reinterpret_cast<const int32_t *>(Xv) + r * ldx + c0);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int64_t r = rb + 4 * v;
            if (r >= r_end) break;  // uniform per wave
            int4 q = raw[v];
            if (FROM_FLOAT && in_cols) {
                q.x = rtn_one(__int_as_float(raw[v].x), scale, bad);
                q.y = rtn_one(__int_as_float(raw[v].y), scale, bad);
                q.z = rtn_one(__int_as_float(raw[v].z), scale, bad);
                q.w = rtn_one(__int_as_float(raw[v].w), scale, bad);
                *reinterpret_cast<int4 *>(Q + r * ldq + c0) = q;
            }
            const int a0 = iabs_sat(q.x), a1 = iabs_sat(q.y), a2 = iabs_sat(q.z), a3 = iabs_sat(q.w);
            const int o0 = a0 >= s, o1 = a1 >= s, o2 = a2 >= s, o3 = a3 >= s;
            ccnt[0] += o0; ccnt[1] += o1; ccnt[2] += o2; ccnt[3] += o3;
            cmax[0] = max(cmax[0], a0); cmax[1] = max(cmax[1], a1);
            cmax[2] = max(cmax[2], a2); cmax[3] = max(cmax[3], a3);
            // row statistics: popcount of the wave's ballots, wave-wide max
            const unsigned long long b0 = __ballot(o0), b1 = __ballot(o1), b2 = __ballot(o2), b3 = __ballot(o3);
            const int n0 = __popcll(b0), n1 = __popcll(b1), n2 = __popcll(b2), n3 = __popcll(b3);
            const int rc = n0 + n1 + n2 + n3;
            if (rowcnt || rowmax) {
                const int rm = wave_max_nonneg_lane63(max(max(a0, a1), max(a2, a3)));
                if (lane == 63) {
                    if (rowcnt && rc) atomicAdd(&rowcnt[r], rc);
                    if (rowmax && rm) atomicMax(&rowmax[r], rm);
                }
            }
            if (ob && rc) {  // uniform per wave, rare: append the OB entries (row, column, value) to the staged list
                int base = 0;
                if (lane == 0) base = atomicAdd(&stage.count, rc);
                base = __builtin_amdgcn_readfirstlane(base);
                const unsigned long long below = (1ull << lane) - 1ull;
                const int p0 = base + __popcll(b0 & below), p1 = base + n0 + __popcll(b1 & below),
                          p2 = base + n0 + n1 + __popcll(b2 & below), p3 = base + n0 + n1 + n2 + __popcll(b3 & below);
                if (o0) ob_push(&stage, p0, (int32_t)r, (int32_t)c0, q.x, ob, ob_cap, ob_count);
                if (o1) ob_push(&stage, p1, (int32_t)r, (int32_t)(c0 + 1), q.y, ob, ob_cap, ob_count);
                if (o2) ob_push(&stage, p2, (int32_t)r, (int32_t)(c0 + 2), q.z, ob, ob_cap, ob_count);
                if (o3) ob_push(&stage, p3, (int32_t)r, (int32_t)(c0 + 3), q.w, ob, ob_cap, ob_count);
            }
        }
    }
    if (ob) ob_flush(&stage, ob, ob_cap, ob_count);
    if (colcnt || colmax)
        flush_columns<4>(ccnt, cmax, (int64_t)cbx * 256, cols, colcnt, colmax, lds);
    if (FROM_FLOAT && status && __ballot(bad) && lane == 0) atomicOr(status, 1);
}

template <bool FROM_FLOAT>
__global__ __launch_bounds__(256) void qscan_vec_kernel(VecOperand a, int64_t cols, int s) {
    __shared__ int lds[2 * 4 * 256];
    __shared__ ObStage stage;
    qscan_vec_body<FROM_FLOAT>(a, cols, s, blockIdx.y, lds, stage);
}

// Both operands of a product (same inner dimension) in one launch: the row blocks of the second follow
// those of the first, so that the end of the one overlaps the start of the other.
__global__ __launch_bounds__(256) void qscan_vec_pair_kernel(VecOperand a, VecOperand b, int64_t cols, int s) {
    __shared__ int lds[2 * 4 * 256];
    __shared__ ObStage stage;
    const int by = blockIdx.y;
    if (by < a.row_blocks) qscan_vec_body<true>(a, cols, s, by, lds, stage);
    else qscan_vec_body<true>(b, cols, s, by - a.row_blocks, lds, stage);
}

// General path: any strides.  Workgroup = 64 x 64 tile staged through LDS so that reads follow the
// input's unit-stride axis (if it has one) and writes follow the rows of Q.
template <bool FROM_FLOAT>
__global__ __launch_bounds__(256) void qscan_tile_kernel(const void *__restrict__ Xv, int64_t rows,
                                                         int64_t cols, int64_t sx_r, int64_t sx_c,
                                                         float scale_val, const float *scale_ptr, int s,
                                                         int32_t *__restrict__ Q,
                                                         int64_t ldq, int32_t *rowcnt, int32_t *colcnt,
                                                         int32_t *rowmax, int32_t *colmax,
                                                         int32_t *status, int32_t *ob, int ob_cap,
                                                         int32_t *ob_count) {
    __shared__ int32_t tile[64][65];
    __shared__ int lds[2 * 4 * 64];
    __shared__ ObStage stage;
    const float scale = step_of(scale_val, scale_ptr);
    if (ob && threadIdx.x == 0) stage.count = 0;  // published by the barrier after the tile is filled
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
    int bad = 0;
    const bool along_rows = (sx_r == 1 && sx_c != 1);  // unit stride runs down the rows
    for (int it = 0; it < 16; ++it) {
        const int a = wave + 4 * it;  // slow index of this pass
        const int rr = along_rows ? lane : a;
        const int cc = along_rows ? a : lane;
        const int64_t r = r0 + rr, c = c0 + cc;
        int32_t q = 0;
        if (r < rows && c < cols) {
            if (FROM_FLOAT)
                q = rtn_one(reinterpret_cast<const float *>(Xv)[r * sx_r + c * sx_c], scale, bad);
            else
                q = reinterpret_cast<const int32_t *>(Xv)[r * sx_r + c * sx_c];
        }
        tile[rr][cc] = q;
    }
    __syncthreads();
    int ccnt[1] = {0}, cmax[1] = {0};
    for (int it = 0; it < 16; ++it) {
        const int rr = wave + 4 * it;
        const int64_t r = r0 + rr, c = c0 + lane;
        const bool ok = r < rows && c < cols;
        const int32_t q = tile[rr][lane];
        if (FROM_FLOAT && ok) Q[r * ldq + c] = q;
        const int a = iabs_sat(q);
        const int o = a >= s;
        ccnt[0] += o;
        cmax[0] = max(cmax[0], a);
        const unsigned long long bo = __ballot(o);
        const int rc = __popcll(bo);
        const int rm = wave_max_nonneg_lane63(a);
        if (lane == 63 && r < rows) {
            if (rowcnt && rc) atomicAdd(&rowcnt[r], rc);
            if (rowmax && rm) atomicMax(&rowmax[r], rm);
        }
        if (ob && rc) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&stage.count, rc);
            base = __builtin_amdgcn_readfirstlane(base);
            const int pos = base + __popcll(bo & ((1ull << lane) - 1ull));
            if (o) ob_push(&stage, pos, (int32_t)r, (int32_t)c, q, ob, ob_cap, ob_count);
        }
    }
    if (ob) ob_flush(&stage, ob, ob_cap, ob_count);
    if (colcnt || colmax) flush_columns<1>(ccnt, cmax, c0, cols, colcnt, colmax, lds);
    if (FROM_FLOAT && status && __ballot(bad) && lane == 0) atomicOr(status, 1);
}

// Transposed input (unit stride down the rows of the operand, as for a weight-gradient GEMM that
// contracts over tokens).  Workgroup = 128 x 128 tile: it is read along the input's contiguous axis
// (512 bytes per column and instruction), quantised, staged in LDS column-major, and then written
// and scanned row by row exactly as on the fast path (512 bytes of Q per row).
constexpr int kTrTile = 128, kTrPitch = kTrTile + 1;
constexpr int kTrThreads = 1024, kTrWaves = kTrThreads / 64;  // LDS admits two workgroups per CU: 32 waves keep the loads coming
constexpr int kTrPerWave = kTrTile / kTrWaves;               // columns (then rows) of the tile per wave, two per instruction

template <bool FROM_FLOAT>
__global__ __launch_bounds__(kTrThreads) void qscan_tr_kernel(const void *__restrict__ Xv, int64_t rows, int64_t cols,
                                                       int64_t sx_c, float scale_val, const float *scale_ptr,
                                                       int s, int32_t *__restrict__ Q, int64_t ldq, int32_t *rowcnt,
                                                       int32_t *colcnt, int32_t *rowmax, int32_t *colmax,
                                                       int32_t *status, int32_t *ob, int ob_cap,
                                                       int32_t *ob_count) {
    __shared__ int32_t tile[kTrTile * kTrPitch];  // [column][row]
    __shared__ ObStage stage;
    const float scale = step_of(scale_val, scale_ptr);
    if (ob && threadIdx.x == 0) stage.count = 0;  // published by the barrier after the tile is filled
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int half = lane >> 5, l32 = lane & 31;
    const int64_t r0 = (int64_t)blockIdx.x * kTrTile, c0 = (int64_t)blockIdx.y * kTrTile;
    int bad = 0;
    // ---- read: wave w takes kTrPerWave columns, two per instruction, four rows per lane
    const int64_t rl = r0 + 4 * l32;  // rows % 4 == 0 on this path
#pragma unroll
    for (int it = 0; it < kTrPerWave / 2; ++it) {
        const int cc = kTrPerWave * wave + 2 * it + half;
        const int64_t c = c0 + cc;
        int4 raw = make_int4(0, 0, 0, 0);
        const bool ok = c < cols && rl < rows;
        if (ok) raw = load_nt16(reinterpret_cast<const int32_t *>(Xv) + c * sx_c + rl);
        int q[4] = {raw.x, raw.y, raw.z, raw.w};
        if (FROM_FLOAT && ok) {
#pragma unroll
            for (int i = 0; i < 4; ++i) q[i] = rtn_one(__int_as_float(q[i]), scale, bad);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) tile[cc * kTrPitch + 4 * l32 + i] = q[i];
    }
    __syncthreads();
    // ---- write and scan: wave w takes kTrPerWave rows, two per instruction, four columns per lane
    int ccnt[4] = {0, 0, 0, 0}, cmax[4] = {0, 0, 0, 0};
    const int64_t cl = c0 + 4 * l32;  // cols % 4 == 0 on this path
    const unsigned long long mine = half ? 0xFFFFFFFF00000000ull : 0x00000000FFFFFFFFull;
    for (int it = 0; it < kTrPerWave / 2; ++it) {
        const int rr = kTrPerWave * wave + 2 * it + half;
        const int64_t r = r0 + rr;
        const bool ok = r < rows && cl < cols;
        int q[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) q[i] = tile[(4 * l32 + i) * kTrPitch + rr];
        if (FROM_FLOAT && ok) *reinterpret_cast<int4 *>(Q + r * ldq + cl) = make_int4(q[0], q[1], q[2], q[3]);
        int a[4], o[4];
        int rm = 0, any = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[i] = ok ? iabs_sat(q[i]) : 0;
            o[i] = a[i] >= s;
            ccnt[i] += o[i];
            cmax[i] = max(cmax[i], a[i]);
            rm = max(rm, a[i]);
            any |= o[i];
        }
        if (rowcnt || rowmax) {
            int rc = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) rc += __popcll(__ballot(o[i]) & mine);
            rm = half_wave_max_nonneg_last(rm);
            if (l32 == 31 && r < rows) {
                if (rowcnt && rc) atomicAdd(&rowcnt[r], rc);
                if (rowmax && rm) atomicMax(&rowmax[r], rm);
            }
        }
        if (ob && any) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (o[i])
                    ob_push(&stage, atomicAdd(&stage.count, 1), (int32_t)r, (int32_t)(cl + i), q[i], ob, ob_cap,
                            ob_count);
        }
    }
    if (ob) ob_flush(&stage, ob, ob_cap, ob_count);
    if (colcnt || colmax) {
        __syncthreads();  // the tile has been consumed: its memory takes the column partials
        constexpr int HW = 2 * kTrWaves;
        int32_t *part = tile;  // [2][HW half-waves][128 columns]
        static_assert(2 * HW * kTrTile <= kTrTile * kTrPitch, "the partials must fit the tile");
        const int hw = 2 * wave + half;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            part[(0 * HW + hw) * kTrTile + 4 * l32 + i] = ccnt[i];
            part[(1 * HW + hw) * kTrTile + 4 * l32 + i] = cmax[i];
        }
        __syncthreads();
        if (threadIdx.x < kTrTile) {
            int cnt = 0, mx = 0;
#pragma unroll
            for (int w8 = 0; w8 < HW; ++w8) {
                cnt += part[(0 * HW + w8) * kTrTile + threadIdx.x];
                mx = max(mx, part[(1 * HW + w8) * kTrTile + threadIdx.x]);
            }
            const int64_t col = c0 + threadIdx.x;
            if (col < cols) {
                if (colcnt && cnt) atomicAdd(&colcnt[col], cnt);
                if (colmax && mx) atomicMax(&colmax[col], mx);
            }
        }
    }
    if (FROM_FLOAT && status && __ballot(bad) && lane == 0) atomicOr(status, 1);
}

// Device-to-device copy in the access pattern of the fast quantize path (a workgroup moves 64 rows x
// 1 KiB of a matrix with 16 KiB rows, non-temporal loads and stores): the rate the memory system gives
// a kernel that does nothing else, for the measured-peak line of the benchmark.
__global__ __launch_bounds__(256) void stream_copy_kernel(const float4 *__restrict__ src, float4 *__restrict__ dst) {
    typedef float v4f __attribute__((ext_vector_type(4)));
    constexpr size_t kPitch = 1024;  // float4 per row
    const size_t cb = (blockIdx.x + blockIdx.y) % gridDim.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const size_t base = (size_t)blockIdx.y * 64 * kPitch + cb * 64 + lane;
    const v4f *s = reinterpret_cast<const v4f *>(src);
    v4f *d = reinterpret_cast<v4f *>(dst);
    for (int r0 = wave; r0 < 64; r0 += 16) {
        v4f v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(s + base + (size_t)(r0 + 4 * u) * kPitch);
#pragma unroll
        for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], d + base + (size_t)(r0 + 4 * u) * kPitch);
    }
}

// Clears up to twelve int32 arrays (the statistics of two operands) in one launch.
constexpr int kZeroArrays = 12;
struct ZeroList {
    int32_t *p[kZeroArrays];
    int64_t len[kZeroArrays];
};
__global__ void zero_lists_kernel(ZeroList z) {
#pragma unroll
    for (int i = 0; i < kZeroArrays; ++i) {
        int32_t *p = z.p[i];
        const int64_t len = z.len[i];
        if (!p) continue;
        for (int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; x < len; x += (int64_t)gridDim.x * blockDim.x)
            p[x] = 0;
    }
}

// adds the arrays of one operand's statistics to the list, from entry `at` on; returns the longest of them
static int64_t list_stats(ZeroList &z, int at, const imunpack_stats_t *st, int64_t rows, int64_t cols, int32_t *status) {
    int64_t longest = 0;
    for (int i = 0; i < 6; ++i) { z.p[at + i] = nullptr; z.len[at + i] = 0; }
    if (st) {
        int32_t *p[4] = {st->rowcnt, st->colcnt, st->rowmax, st->colmax};
        const int64_t len[4] = {rows, cols, rows, cols};
        for (int i = 0; i < 4; ++i)
            if (p[i] && len[i] > 0) { z.p[at + i] = p[i]; z.len[at + i] = len[i]; longest = len[i] > longest ? len[i] : longest; }
        if (st->ob && st->ob_count) { z.p[at + 4] = st->ob_count; z.len[at + 4] = 1; longest = longest > 1 ? longest : 1; }
    }
    if (status) { z.p[at + 5] = status; z.len[at + 5] = 1; longest = longest > 1 ? longest : 1; }
    return longest;
}

static int zero_listed(const ZeroList &z, int64_t longest, hipStream_t stream) {
    if (longest == 0) return IMUNPACK_OK;
    int blocks = (int)((longest + 255) / 256);
    if (blocks > 256) blocks = 256;
    hipLaunchKernelGGL(zero_lists_kernel, dim3(blocks), dim3(256), 0, stream, z);
    return launch_status();
}

static int zero_stats(const imunpack_stats_t *st, int64_t rows, int64_t cols, int32_t *status,
                      hipStream_t stream) {
    ZeroList z;
    for (int i = 0; i < kZeroArrays; ++i) { z.p[i] = nullptr; z.len[i] = 0; }
    return zero_listed(z, list_stats(z, 0, st, rows, cols, status), stream);
}

// The operand's description for the fast path, if it qualifies (unit column stride, rows and pointers
// aligned to 16 bytes).
template <bool FROM_FLOAT>
static bool vec_operand(VecOperand &o, const void *X, int64_t rows, int64_t cols, int64_t sx_r, int64_t sx_c, float scale,
                        const float *scale_dev, int32_t *Q, int64_t ldq, const imunpack_stats_t *st, int32_t *status) {
    const bool vec = sx_c == 1 && (cols % 4) == 0 && (sx_r % 4) == 0 && ((uintptr_t)X % 16) == 0 &&
                     (!FROM_FLOAT || ((ldq % 4) == 0 && ((uintptr_t)Q % 16) == 0));
    if (!vec) return false;
    int64_t rpw = 64;  // 16, 32 and 128 rows per workgroup were all slower
    if ((rows + rpw - 1) / rpw > 32767) rpw = ((rows + 32766) / 32767 + 3) / 4 * 4;
    int32_t *ob = (st && st->ob && st->ob_count && st->ob_cap > 0) ? st->ob : nullptr;
    o = VecOperand{X, rows, sx_r, scale, scale_dev, Q, ldq,
                   st ? st->rowcnt : nullptr, st ? st->colcnt : nullptr, st ? st->rowmax : nullptr, st ? st->colmax : nullptr,
                   status, ob, ob ? (int)st->ob_cap : 0, ob ? st->ob_count : nullptr, (int)rpw, (int)((rows + rpw - 1) / rpw)};
    return true;
}

template <bool FROM_FLOAT>
static int check_qscan_args(const void *X, int64_t rows, int64_t cols, int64_t sx_r, int64_t sx_c, float scale,
                            const float *scale_dev, int b, const int32_t *Q, int64_t ldq, const imunpack_stats_t *st) {
    if (!X || rows < 0 || cols < 0 || b < 2 || b > 8) return IMUNPACK_EINVAL;
    if (FROM_FLOAT && (!Q || ldq < cols || (!scale_dev && (!(scale > 0.0f) || !(scale < 3.0e38f))))) return IMUNPACK_EINVAL;
    if (sx_r < 1 || sx_c < 1) return IMUNPACK_EINVAL;
    if (st && st->ob_cap > 0x7fffffff / 3) return IMUNPACK_EINVAL;
    return IMUNPACK_OK;
}

template <bool FROM_FLOAT>
int run_qscan(const void *X, int64_t rows, int64_t cols, int64_t sx_r, int64_t sx_c, float scale,
              const float *scale_dev, int b, int32_t *Q, int64_t ldq, const imunpack_stats_t *st, int32_t *status,
              hipStream_t stream) {
    IMU_TRY(check_qscan_args<FROM_FLOAT>(X, rows, cols, sx_r, sx_c, scale, scale_dev, b, Q, ldq, st));
    IMU_TRY(zero_stats(st, rows, cols, FROM_FLOAT ? status : nullptr, stream));
    if (rows == 0 || cols == 0) return IMUNPACK_OK;
    const int s = 1 << (b - 1);
    int32_t *rowcnt = st ? st->rowcnt : nullptr, *colcnt = st ? st->colcnt : nullptr;
    int32_t *rowmax = st ? st->rowmax : nullptr, *colmax = st ? st->colmax : nullptr;
    int32_t *ob = (st && st->ob && st->ob_count && st->ob_cap > 0) ? st->ob : nullptr;
    int32_t *ob_count = ob ? st->ob_count : nullptr;
    const int ob_cap = ob ? (int)st->ob_cap : 0;
    if (!FROM_FLOAT && !rowcnt && !colcnt && !rowmax && !colmax && !ob) return IMUNPACK_OK;
    VecOperand vo;
    if (vec_operand<FROM_FLOAT>(vo, X, rows, cols, sx_r, sx_c, scale, scale_dev, Q, ldq, st, status)) {
        dim3 grid((unsigned)((cols + 255) / 256), (unsigned)vo.row_blocks);
        hipLaunchKernelGGL(qscan_vec_kernel<FROM_FLOAT>, grid, dim3(256), 0, stream, vo, cols, s);
    } else if (sx_r == 1 && (rows % 4) == 0 && (cols % 4) == 0 && (sx_c % 4) == 0 && ((uintptr_t)X % 16) == 0 &&
               (!FROM_FLOAT || ((ldq % 4) == 0 && ((uintptr_t)Q % 16) == 0)) && (cols + kTrTile - 1) / kTrTile <= 65535) {
        dim3 grid((unsigned)((rows + kTrTile - 1) / kTrTile), (unsigned)((cols + kTrTile - 1) / kTrTile));
        hipLaunchKernelGGL(qscan_tr_kernel<FROM_FLOAT>, grid, dim3(kTrThreads), 0, stream, X, rows, cols, sx_c, scale, scale_dev, s, Q,
                           ldq, rowcnt, colcnt, rowmax, colmax, status, ob, ob_cap, ob_count);
    } else {
        dim3 grid((unsigned)((cols + 63) / 64), (unsigned)((rows + 63) / 64));
        hipLaunchKernelGGL(qscan_tile_kernel<FROM_FLOAT>, grid, dim3(256), 0, stream, X, rows, cols, sx_r,
                           sx_c, scale, scale_dev, s, Q, ldq, rowcnt, colcnt, rowmax, colmax, status, ob, ob_cap, ob_count);
    }
    return launch_status();
}

// Both operands of one product: a single clearing launch and, when both take the fast path, a single
// quantise-and-scan launch; otherwise one call after the other.  A step is a value of the call or, when
// its device pointer is given (the batched call keeps the steps on the device), read from there.
int quantize_pair(const float *A, int64_t n, int64_t sa_r, int64_t sa_c, float scale_A, const float *scale_A_dev,
                  int32_t *QA, int64_t ldqa, const imunpack_stats_t *stA, const float *B, int64_t h, int64_t sb_r,
                  int64_t sb_c, float scale_B, const float *scale_B_dev, int32_t *QB, int64_t ldqb,
                  const imunpack_stats_t *stB, int64_t d, int b, int32_t *status, hipStream_t stream) {
    int32_t *stat_a = status, *stat_b = status ? status + 1 : nullptr;
    IMU_TRY(check_qscan_args<true>(A, n, d, sa_r, sa_c, scale_A, scale_A_dev, b, QA, ldqa, stA));
    IMU_TRY(check_qscan_args<true>(B, h, d, sb_r, sb_c, scale_B, scale_B_dev, b, QB, ldqb, stB));
    VecOperand va, vb;
    const bool paired = n > 0 && h > 0 && d > 0 &&
                        vec_operand<true>(va, A, n, d, sa_r, sa_c, scale_A, scale_A_dev, QA, ldqa, stA, stat_a) &&
                        vec_operand<true>(vb, B, h, d, sb_r, sb_c, scale_B, scale_B_dev, QB, ldqb, stB, stat_b);
    if (!paired) {
        IMU_TRY(run_qscan<true>(A, n, d, sa_r, sa_c, scale_A, scale_A_dev, b, QA, ldqa, stA, stat_a, stream));
        return run_qscan<true>(B, h, d, sb_r, sb_c, scale_B, scale_B_dev, b, QB, ldqb, stB, stat_b, stream);
    }
    ZeroList z;
    const int64_t la = list_stats(z, 0, stA, n, d, stat_a), lb = list_stats(z, 6, stB, h, d, stat_b);
    IMU_TRY(zero_listed(z, std::max(la, lb), stream));
    const bool b_first = vb.row_blocks > va.row_blocks;  // the longer operand first: the shorter one fills its tail
    const VecOperand &first = b_first ? vb : va, &second = b_first ? va : vb;
    dim3 grid((unsigned)((d + 255) / 256), (unsigned)(first.row_blocks + second.row_blocks));
    hipLaunchKernelGGL(qscan_vec_pair_kernel, grid, dim3(256), 0, stream, first, second, d, 1 << (b - 1));
    return launch_status();
}

int scan_i32(const int32_t *Q, int64_t rows, int64_t cols, int64_t ldq, int b,
             const imunpack_stats_t *st, hipStream_t stream) {
    return run_qscan<false>(Q, rows, cols, ldq, 1, 1.0f, nullptr, b, nullptr, 0, st, nullptr, stream);
}

}  // namespace imu

extern "C" int imunpack_quantize(const float *X, int64_t rows, int64_t cols, int64_t sx_r, int64_t sx_c,
                                 float scale, int b, int32_t *Q, int64_t ldq,
                                 const imunpack_stats_t *stats, int32_t *status,
                                 imunpack_stream_t stream) {
    return imu::run_qscan<true>(X, rows, cols, sx_r, sx_c, scale, nullptr, b, Q, ldq, stats, status,
                                (hipStream_t)stream);
}

extern "C" int imunpack_quantize_pair(const float *A, int64_t n, int64_t sa_r, int64_t sa_c, float scale_A, int32_t *QA,
                                      int64_t ldqa, const imunpack_stats_t *stats_A, const float *B, int64_t h,
                                      int64_t sb_r, int64_t sb_c, float scale_B, int32_t *QB, int64_t ldqb,
                                      const imunpack_stats_t *stats_B, int64_t d, int b, int32_t *status,
                                      imunpack_stream_t stream) {
    return imu::quantize_pair(A, n, sa_r, sa_c, scale_A, nullptr, QA, ldqa, stats_A, B, h, sb_r, sb_c, scale_B, nullptr, QB,
                              ldqb, stats_B, d, b, status, (hipStream_t)stream);
}

extern "C" int imunpack_scan(const int32_t *Q, int64_t rows, int64_t cols, int64_t ldq, int b,
                             const imunpack_stats_t *stats, imunpack_stream_t stream) {
    if (!Q || ldq < cols) return IMUNPACK_EINVAL;
    return imu::scan_i32(Q, rows, cols, ldq, b, stats, (hipStream_t)stream);
}

extern "C" int imunpack_diag_copy(const void *src, void *dst, int64_t bytes, imunpack_stream_t stream) {
    constexpr int64_t kBlock = 64 * 16384;  // one band of 64 rows of 16 KiB
    if (!src || !dst || bytes <= 0 || bytes % kBlock || bytes / kBlock > 65535 || (uintptr_t)src % 16 || (uintptr_t)dst % 16)
        return IMUNPACK_EINVAL;
    hipLaunchKernelGGL(imu::stream_copy_kernel, dim3(16, (unsigned)(bytes / kBlock)), dim3(256), 0, (hipStream_t)stream,
                       (const float4 *)src, (float4 *)dst);
    return imu::launch_status();
}
