// int8 MFMA GEMM over the unpacked operands (Alg. 3, ScaledMatMul) with the recombination
// (Sec. 4 "Reconstructing A": Pi applied as an index-add with power-of-two weights) and the
// dequantisation (Sec. 2, Eq. quantized_gemm) fused into the epilogue.
//
// Alg. 3 runs one GEMM per distinct diagonal entry s^e of S and adds them with weight s^e.  The
// physical column order puts the groups one after the other, highest exponent first, so a single
// pass over K evaluates  sum_e s^e C_e  by Horner's rule: the int32 accumulators are shifted left
// by (b-1) * (e_g - e_{g+1}) between group g and group g+1.  That is exact whenever the weighted
// sum fits int32, which imunpack_unpack checks for the actual operands; otherwise each group is
// launched on its own and accumulated in int64 (the un-fused path).
#include "common.h"

#include <cstring>

namespace imu {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = kTile, BN = kTile, BK = 64;   // bytes of K per stage = int8 elements
constexpr int kGemmThreads = 256;                // 4 waves, 2 x 2, each 128 x 128

struct GemmArgs {
    const int8_t *A, *B;      // [Mp][Kp], [Np][Kp]
    int Kp, mtiles, ntiles;
    int kt0, kt1;             // k-tile range of this launch
    int nbound;               // Horner boundaries inside the range
    int bound_kt[kMaxGroups]; // shift the accumulators after this k-tile ...
    int bound_sh[kMaxGroups]; // ... by this many bits
    // fused epilogue
    RowLayout layA, layB;
    const int32_t *flatA, *flatB;   // per tile: 1 if every source row of the tile has a single level
    int sh, final_shift;
    int64_t *C_int;
    float *C_fp;
    int64_t ldc;
    double scale;             // scale_A * scale_B
    // un-fused: C_u[p][q] (+)= acc << seg_shift
    int64_t *C_u;
    int Np;
    int seg_shift, seg_first;
};

// LDS tile: [rows][64 B]; the four 16-byte chunks of a row are XOR-swizzled with bits 2..3 of
// the row so that 16 consecutive rows at one k-chunk hit 16 different bank groups.
__device__ __forceinline__ int lds_off(int row, int kc) { return row * BK + ((kc ^ ((row >> 2) & 3)) << 4); }

// XCD-aware tile order: workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2,
// so ids that land on one XCD are given one contiguous run of tiles; inside a run the tiles walk
// bands of 4 tile-rows so that an XCD's resident workgroups share A and B panels.
__device__ __forceinline__ void tile_of(int wg, int mtiles, int ntiles, int &tm, int &tn) {
    const int total = mtiles * ntiles;
    const int xcd = wg & 7, idx = wg >> 3;
    const int per = total >> 3, rem = total & 7;
    const int logical = xcd * per + min(xcd, rem) + idx;
    constexpr int kBand = 4;
    const int band_sz = kBand * ntiles;
    const int band = logical / band_sz;
    const int first_m = band * kBand;
    const int rows_in_band = min(kBand, mtiles - first_m);
    const int in_band = logical - band * band_sz;
    tm = first_m + in_band % rows_in_band;
    tn = in_band / rows_in_band;
}

template <int MODE>  // 0: fused epilogue, 1: int64 segment into C_u
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_i8_kernel(const GemmArgs g) {
    __shared__ __attribute__((aligned(16))) int8_t smem[2 * 2 * BM * BK];  // [buf][A|B][256][64] = 64 KiB
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    int tm, tn;
    tile_of(blockIdx.x, g.mtiles, g.ntiles, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    // global -> register staging: 1024 chunks of 16 B per operand tile, 4 per thread
    const int8_t *gA[4], *gB[4];
    int soff[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int id = tid + u * kGemmThreads;
        const int row = id >> 2, kc = id & 3;
        gA[u] = g.A + (int64_t)(m0 + row) * g.Kp + kc * 16;
        gB[u] = g.B + (int64_t)(n0 + row) * g.Kp + kc * 16;
        soff[u] = lds_off(row, kc);
    }
    v4i ra[4], rb[4];
    auto gload = [&](int kt) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            ra[u] = *reinterpret_cast<const v4i *>(gA[u] + (int64_t)kt * BK);
            rb[u] = *reinterpret_cast<const v4i *>(gB[u] + (int64_t)kt * BK);
        }
    };
    auto swrite = [&](int buf) {
        int8_t *sa = smem + buf * (2 * BM * BK), *sb = sa + BM * BK;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            *reinterpret_cast<v4i *>(sa + soff[u]) = ra[u];
            *reinterpret_cast<v4i *>(sb + soff[u]) = rb[u];
        }
    };

    v16i acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    const int lrow = lane & 31, lhalf = lane >> 5;
    int nb = 0;
    int next_kt = g.nbound > 0 ? g.bound_kt[0] : -1;

    if (g.kt0 < g.kt1) {
        gload(g.kt0);
        swrite(0);
    }
    __syncthreads();
    for (int kt = g.kt0; kt < g.kt1; ++kt) {
        const int buf = (kt - g.kt0) & 1;
        const bool more = kt + 1 < g.kt1;
        if (more) gload(kt + 1);
        const int8_t *sa = smem + buf * (2 * BM * BK), *sb = sa + BM * BK;
#pragma unroll
        for (int ks = 0; ks < BK / 32; ++ks) {
            v4i fa[4], fb[4];
            const int kc = ks * 2 + lhalf;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                fa[i] = *reinterpret_cast<const v4i *>(sa + lds_off(wm * 128 + i * 32 + lrow, kc));
                fb[i] = *reinterpret_cast<const v4i *>(sb + lds_off(wn * 128 + i * 32 + lrow, kc));
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (kt == next_kt) {  // end of an exponent group: Horner step
            const int shv = g.bound_sh[nb];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] <<= shv;
            ++nb;
            next_kt = nb < g.nbound ? g.bound_kt[nb] : -1;
        }
        if (more) swrite(buf ^ 1);
        __syncthreads();
    }

    // accumulator element r of block (i, j): row 8*(r/4) + 4*(lane/32) + r%4, column lane%32
    if (MODE == 1) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int p = m0 + wm * 128 + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
                    const int q = n0 + wn * 128 + j * 32 + lrow;
                    int64_t *dst = g.C_u + (int64_t)p * g.Np + q;
                    const int64_t v = (int64_t)acc[i][j][r] << g.seg_shift;
                    *dst = g.seg_first ? v : *dst + v;
                }
        return;
    }

    const int isrc0 = g.layA.tile_src0[tm], nsrcA = g.layA.tile_src0[tm + 1] - isrc0;
    const int jsrc0 = g.layB.tile_src0[tn], nsrcB = g.layB.tile_src0[tn + 1] - jsrc0;
    if (g.flatA[tm] && g.flatB[tn]) {
        // no row of this tile was split on either side: physical = source order, store directly
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int pi = wm * 128 + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
                    const int qj = wn * 128 + j * 32 + lrow;
                    if (pi < nsrcA && qj < nsrcB) {
                        const int64_t v = (int64_t)acc[i][j][r] << g.final_shift;
                        const int64_t o = (int64_t)(isrc0 + pi) * g.ldc + (jsrc0 + qj);
                        if (g.C_int) g.C_int[o] = v;
                        if (g.C_fp) g.C_fp[o] = (float)((double)v * g.scale);
                    }
                }
        return;
    }

    // general tile: fold the digit levels of both operands through LDS, 64 physical rows at a time
    int32_t *fold = reinterpret_cast<int32_t *>(smem);  // [64][256] int32 = 64 KiB
    const int j = jsrc0 + tid;
    const bool have_col = tid < nsrcB;
    const int q0 = have_col ? g.layB.src_pstart[j] - n0 : 0;
    const int lj = have_col ? g.layB.src_nlev[j] : 0;
    int64_t run = 0;
    for (int c = 0; c < 4; ++c) {
        __syncthreads();
        if (wm == (c >> 1)) {
#pragma unroll
            for (int ii = 0; ii < 2; ++ii) {
                const int i = (c & 1) * 2 + ii;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int row = ii * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
                        const int col = wn * 128 + jj * 32 + lrow;
                        fold[row * 256 + (col ^ (((row >> 2) & 1) << 5))] = acc[i][jj][r];
                    }
            }
        }
        __syncthreads();
        for (int row = 0; row < 64; ++row) {
            const int p = m0 + c * 64 + row;
            const int i = g.layA.prow_src[p];
            if (i < 0) continue;  // padding row (uniform)
            const int lvl = g.layA.prow_exp[p];
            const bool last = lvl == g.layA.src_nlev[i] - 1;
            if (have_col) {
                int64_t v = 0;
                const int sw = ((row >> 2) & 1) << 5;
                for (int l = 0; l < lj; ++l) v += (int64_t)fold[row * 256 + ((q0 + l) ^ sw)] << (g.sh * l);
                run += v << (g.sh * lvl);
                if (last) {
                    const int64_t outv = run << g.final_shift;
                    const int64_t o = (int64_t)i * g.ldc + j;
                    if (g.C_int) g.C_int[o] = outv;
                    if (g.C_fp) g.C_fp[o] = (float)((double)outv * g.scale);
                    run = 0;
                }
            }
        }
    }
}

// C_int = Pi_A C_u Pi_B^T from the int64 unpacked product, then dequantise.
__global__ __launch_bounds__(256) void recombine_kernel(const int64_t *__restrict__ C_u, int Np, RowLayout layA,
                                                        RowLayout layB, int n, int h, int sh,
                                                        int64_t *C_int, float *C_fp, int64_t ldc,
                                                        double scale) {
    const int i = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (i >= n || j >= h) return;
    const int p0 = layA.src_pstart[i], li = layA.src_nlev[i];
    const int q0 = layB.src_pstart[j], lj = layB.src_nlev[j];
    int64_t acc = 0;
    for (int a = 0; a < li; ++a)
        for (int c = 0; c < lj; ++c) acc += C_u[(int64_t)(p0 + a) * Np + (q0 + c)] << (sh * (a + c));
    const int64_t o = (int64_t)i * ldc + j;
    if (C_int) C_int[o] = acc;
    if (C_fp) C_fp[o] = (float)((double)acc * scale);
}

}  // namespace imu

using namespace imu;

static int check_shifts(const Plan *p) {
    // every weight s^(levelA + levelB + e) applied in int64 must stay below 2^62
    const int maxexp = (p->hdr.lmaxA - 1) + (p->hdr.lmaxB - 1) + (p->hdr.ngroups ? p->hdr.grp_exp[0] : 0);
    return maxexp * p->sh <= 62 ? IMUNPACK_OK : IMUNPACK_ERANGE;
}

extern "C" int imunpack_recombine(const imunpack_plan_t *p, const void *workspace, float scale_A,
                                  float scale_B, int64_t *C_int, float *C_fp, int64_t ldc,
                                  imunpack_stream_t stream) {
    if (!p || !p->valid || !workspace || ldc < p->h) return IMUNPACK_EINVAL;
    if (!C_int && !C_fp) return IMUNPACK_OK;
    IMU_TRY(check_shifts(p));
    dim3 grid((unsigned)((p->h + 255) / 256), (unsigned)p->n);
    if (grid.y > 65535u) return IMUNPACK_EINVAL;
    hipLaunchKernelGGL(recombine_kernel, grid, dim3(256), 0, (hipStream_t)stream,
                       (const int64_t *)workspace, p->hdr.Np, p->layA, p->layB, (int)p->n, (int)p->h, p->sh,
                       C_int, C_fp, ldc, (double)scale_A * (double)scale_B);
    return launch_status();
}

extern "C" int imunpack_gemm(const imunpack_plan_t *p, const int8_t *A_ue, const int8_t *B_eu,
                             void *workspace, int64_t *C_int, float *C_fp, int64_t ldc, float scale_A,
                             float scale_B, int fuse, imunpack_stream_t stream) {
    if (!p || !p->valid || !p->unpacked || !A_ue || !B_eu) return IMUNPACK_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const PlanHeader &h = p->hdr;
    if (h.mtiles <= 0 || h.ntiles <= 0) return IMUNPACK_OK;
    IMU_TRY(check_shifts(p));
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.A = A_ue; g.B = B_eu;
    g.Kp = h.Kp; g.mtiles = h.mtiles; g.ntiles = h.ntiles;
    g.layA = p->layA; g.layB = p->layB;
    g.flatA = p->layA.tile_flat; g.flatB = p->layB.tile_flat;
    g.sh = p->sh;
    g.Np = h.Np;
    const int grid = h.mtiles * h.ntiles;
    bool fused = fuse != 0;
    if (fused && !p->fusable) {
        if (!workspace) return IMUNPACK_ERANGE;
        fused = false;
    }
    if (fused) {
        if ((!C_int && !C_fp) || ldc < p->h) return IMUNPACK_EINVAL;
        g.kt0 = 0; g.kt1 = h.Kp / BK;
        g.nbound = 0;
        for (int q = 0; q + 1 < h.ngroups; ++q) {
            g.bound_kt[g.nbound] = h.grp_k0[q + 1] / BK - 1;
            g.bound_sh[g.nbound] = p->sh * (h.grp_exp[q] - h.grp_exp[q + 1]);
            ++g.nbound;
        }
        g.final_shift = h.ngroups ? p->sh * h.grp_exp[h.ngroups - 1] : 0;
        g.C_int = C_int; g.C_fp = C_fp; g.ldc = ldc;
        g.scale = (double)scale_A * (double)scale_B;
        hipLaunchKernelGGL(gemm_i8_kernel<0>, dim3(grid), dim3(kGemmThreads), 0, st, g);
        return launch_status();
    }
    if (!workspace) return IMUNPACK_EINVAL;
    g.C_u = (int64_t *)workspace;
    for (int q = 0; q < h.ngroups; ++q) {
        g.kt0 = h.grp_k0[q] / BK;
        g.kt1 = g.kt0 + (h.grp_len[q] + BK - 1) / BK;
        g.nbound = 0;
        g.seg_shift = p->sh * h.grp_exp[q];
        g.seg_first = q == 0;
        hipLaunchKernelGGL(gemm_i8_kernel<1>, dim3(grid), dim3(kGemmThreads), 0, st, g);
    }
    IMU_TRY(launch_status());
    if (fuse != 0)  // the caller asked for final outputs: finish the job here
        return imunpack_recombine(p, workspace, scale_A, scale_B, C_int, C_fp, ldc, stream);
    return IMUNPACK_OK;
}
