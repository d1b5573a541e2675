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
constexpr int kStages = 4;                       // LDS ring of k-tiles filled by direct-to-LDS loads
constexpr int kStageBytes = (BM + BN) * BK;      // 32 KiB: A tile then B tile
constexpr int kGemmLds = kStages * kStageBytes;  // 128 KiB of the CU's 160 KiB
constexpr int kDmaPerStage = 8;                  // direct-to-LDS loads one wave issues per k-tile

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

// One direct-to-LDS load: every lane fetches 16 bytes from gbase + voff and the wave's 1 KiB lands
// contiguously at LDS byte address lds_addr (lane l at lds_addr + 16 l).  The LDS base travels in M0.
__device__ __forceinline__ void dma16(unsigned lds_addr, unsigned voff, const int8_t *gbase) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(gbase)
                 : "memory");
}

__device__ __forceinline__ const int8_t *uniform_ptr(const int8_t *p) {
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const int8_t *)(((uint64_t)hi << 32) | lo);
}

// LDS tile: [256 rows][64 B]; the four 16-byte chunks of a row are XOR-swizzled with bits 1..2 of
// the row, which makes the 64-lane ds_read_b128 of an MFMA operand (32 rows x 2 chunks)
// conflict-free.  Chunk kc of row r lives at r*64 + ((kc ^ ((r >> 1) & 3)) << 4).
template <int MODE>  // 0: fused epilogue, 1: int64 segment into C_u
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_i8_kernel(const GemmArgs g) {
    extern __shared__ __attribute__((aligned(1024))) int8_t smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    int tm, tn;
    tile_of(blockIdx.x, g.mtiles, g.ntiles, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const unsigned lds0 = (unsigned)(size_t)smem;

    // ---- global -> LDS: wave w fills rows [64w, 64w+64) of the A tile and of the B tile, 16 rows
    // (1 KiB) per load; lane l writes slot l&3 of row l>>2, so it fetches the chunk that belongs there
    unsigned voff[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int row = 64 * wave + 16 * u + (lane >> 2);
        const int kc = (lane & 3) ^ ((row >> 1) & 3);
        voff[u] = (unsigned)row * (unsigned)g.Kp + (unsigned)(kc * 16);
    }
    const int8_t *gA = g.A + (int64_t)m0 * g.Kp, *gB = g.B + (int64_t)n0 * g.Kp;
    auto issue = [&](int kt) {
        const int8_t *pa = uniform_ptr(gA + (int64_t)kt * BK), *pb = uniform_ptr(gB + (int64_t)kt * BK);
        const unsigned l = __builtin_amdgcn_readfirstlane(lds0 + (unsigned)((kt & (kStages - 1)) * kStageBytes) +
                                                          (unsigned)(wave * 4096));
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            dma16(l + u * 1024, voff[u], pa);
            dma16(l + BM * BK + u * 1024, voff[u], pb);
        }
    };

    // ---- LDS -> registers: operand fragments of v_mfma_i32_32x32x32_i8 (lane: row lane%32, 16 K-bytes
    // at chunk 2*ks + lane/32)
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int swz = (lrow >> 1) & 3;
    const unsigned fa_base = (unsigned)((wm * 128 + lrow) * BK);
    const unsigned fb_base = (unsigned)(BM * BK + (wn * 128 + lrow) * BK);
    const unsigned kc_off[2] = {(unsigned)(((0 + lhalf) ^ swz) << 4), (unsigned)(((2 + lhalf) ^ swz) << 4)};
    v4i fa[2][4], fb[2][4];
    auto load_frags = [&](int kt, int ks, v4i(&a)[4], v4i(&b)[4]) {
        const int8_t *st = smem + (kt & (kStages - 1)) * kStageBytes;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[i] = *reinterpret_cast<const v4i *>(st + fa_base + kc_off[ks] + i * 32 * BK);
            b[i] = *reinterpret_cast<const v4i *>(st + fb_base + kc_off[ks] + i * 32 * BK);
        }
    };

    v16i acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // ---- prologue: three k-tiles in flight, first one landed, its first fragments loaded
    const int kt0 = g.kt0, kt1 = g.kt1;
    for (int p = 0; p < kStages - 1; ++p)
        if (kt0 + p < kt1) issue(kt0 + p);
    if (kt0 + 2 < kt1) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    else if (kt0 + 1 < kt1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (kt0 < kt1) load_frags(kt0, 0, fa[0], fb[0]);

    int kt = kt0;
    for (int seg = 0; seg <= g.nbound; ++seg) {
        const int kend = seg < g.nbound ? g.bound_kt[seg] + 1 : kt1;
        for (; kt < kend; ++kt) {
            // k-tile kt+1 must be complete in LDS for every wave before anyone reads it below; the
            // same barrier retires k-tile kt-1, whose buffer the load of k-tile kt+3 then overwrites
            if (kt + 2 < kt1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            if (kt + 3 < kt1) issue(kt + 3);
            load_frags(kt, 1, fa[1], fb[1]);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[0][i], fb[0][j], acc[i][j], 0, 0, 0);
            if (kt + 1 < kt1) load_frags(kt + 1, 0, fa[0], fb[0]);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[1][i], fb[1][j], acc[i][j], 0, 0, 0);
        }
        if (seg < g.nbound) {  // end of an exponent group: Horner step
            const int shv = g.bound_sh[seg];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] <<= shv;
        }
    }
    __syncthreads();  // all fragment reads done: the ring may be reused by the epilogue

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
    int32_t *fold = reinterpret_cast<int32_t *>(smem);  // [64][256] int32 = 64 KiB of the ring
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

static int gemm_lds_opt_in() {
    static int done = 0;  // the kernels use 128 KiB of dynamic LDS, above the default limit
    if (!done) {
        IMU_HIP(hipFuncSetAttribute((const void *)gemm_i8_kernel<0>, hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds));
        IMU_HIP(hipFuncSetAttribute((const void *)gemm_i8_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds));
        done = 1;
    }
    return IMUNPACK_OK;
}

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
    IMU_TRY(gemm_lds_opt_in());
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
        hipLaunchKernelGGL(gemm_i8_kernel<0>, dim3(grid), dim3(kGemmThreads), kGemmLds, st, g);
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
        hipLaunchKernelGGL(gemm_i8_kernel<1>, dim3(grid), dim3(kGemmThreads), kGemmLds, st, g);
    }
    IMU_TRY(launch_status());
    if (fuse != 0)  // the caller asked for final outputs: finish the job here
        return imunpack_recombine(p, workspace, scale_A, scale_B, C_int, C_fp, ldc, stream);
    return IMUNPACK_OK;
}
