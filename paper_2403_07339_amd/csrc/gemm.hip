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

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <type_traits>

// first register of every aligned quad of the 256 accumulation registers
#define IMU_ACC_QUADS "0,4,8,12,16,20,24,28,32,36,40,44,48,52,56,60,64,68,72,76,80,84,88,92,96,100,104,108,112,116,120,124,128,132,136,140,144,148,152,156,160,164,168,172,176,180,184,188,192,196,200,204,208,212,216,220,224,228,232,236,240,244,248,252"

namespace imu {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef long v2l __attribute__((ext_vector_type(2)));
typedef float v4f_u __attribute__((ext_vector_type(4), aligned(4)));  // 16 bytes at any float boundary
typedef long v2l_u __attribute__((ext_vector_type(2), aligned(8)));

constexpr int BM = kTile, BN = kTile, BK = 128;  // bytes (= int8 elements) of K per LDS stage: one full 128-byte line per row
constexpr int kGemmThreads = 256;                // 4 waves, 2 x 2, each 128 x 128
constexpr int kHalfBytes = BM * BK;              // 32 KiB: the A tile or the B tile of one k-tile
constexpr int kRing = 5;                         // LDS ring of half-stages: A(k) in slot 2k mod 5, B(k) in slot 2k+1 mod 5
constexpr int kGemmLds = kRing * kHalfBytes;     // all 160 KiB of the CU's LDS

struct GemmArgs {
    const int8_t *A, *B;      // the A store [Mp][ldA] and B_eu [Np][ldB] (row pitches in bytes)
    int ldA, ldB, Kp, mtiles, ntiles;
    int kt0, kt1;             // k-tile range of this launch
    // The range is cut into segments at the k-tiles where the exponent group changes (Horner step) or
    // where the walk through the A store jumps: k-tile kt of segment i reads block kt + seg_delta[i].
    int nbound;               // boundaries inside the range
    int bound_kt[kMaxGroups]; // segment i ends with this k-tile ...
    int bound_sh[kMaxGroups]; // ... after which the accumulators are shifted by this many bits (0: same group)
    int seg_delta[kMaxGroups + 1];
    // fused epilogue
    RowLayout layA, layB;
    const int32_t *flatA, *flatB;   // per tile: 1 if every source row of the tile has a single level
    int sh, final_shift;
    int64_t *C_int;
    float *C_fp;
    int64_t ldc;
    double scale;             // scale_A * scale_B
    const float *scale_a_dev, *scale_b_dev;  // if set: the two RTN steps are read from device memory instead
    // un-fused: C_u[p][q] (+)= acc << seg_shift
    int64_t *C_u;
    int Np;
    int seg_shift, seg_first;
    // fused launch made before the host knows the accumulator bounds: the kernel checks them itself
    // and writes nothing if the shifted group sum could leave int32
    const unsigned long long *guard;
    int guard_mul;            // s - 1
    int fold_f64;             // no int64 output wanted and every sum over digit levels is exact in binary64
    // benchmark reporting: if set, workgroup 0 writes {shader clock ticks, 100 MHz wall ticks} of its K loop
    unsigned long long *clock_probe;
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

// LDS half-stage: [256 rows][128 B] of one operand; the eight 16-byte chunks of a row are XOR-swizzled
// with bits 1..3 of the row (chunk kc of row r lives at r*128 + ((kc ^ ((r >> 1) & 7)) << 4)), which
// makes the 64-lane ds_read_b128 of an MFMA operand (32 rows x 2 chunks) conflict-free.
//
// FP6 = true: the digits are 6-bit floating-point codes (b <= 4).  A k-tile is still 128 columns, now 96
// bytes of a row; LDS rows are 112 bytes apart (seven 16-byte slots, the seventh a repeat of the sixth:
// with 96 the rows that a wave reads together would share banks two by two); a lane's fragment of
// v_mfma_f32_32x32x64_f8f6f4 is one 16-byte and one 8-byte read (see fp6_dword); a k-tile is two k-steps
// of 16 matrix instructions; the accumulators are binary32 and hold integers below 2^24, exactly.
template <int MODE, bool FP6>  // MODE 0: fused epilogue, 1: int64 segment into C_u
__device__ __forceinline__ void gemm_body(const GemmArgs &g, int8_t *smem) {
    constexpr int kRowB = FP6 ? 96 : BK;           // bytes of a row of the operand per k-tile
    constexpr int kPitch = FP6 ? 112 : BK;         // bytes from row to row in LDS
    constexpr int kHalfBytes = BM * kPitch;        // the A tile or the B tile of one k-tile in LDS
    constexpr int kLoads = FP6 ? 7 : 8;            // direct-to-LDS loads per wave and half-stage
    constexpr int kWaveBytes = 64 * kPitch;        // a wave's 64 rows of a half-stage
    if (MODE == 0 && g.guard) {
        const unsigned long long b0 = g.guard[0], b1 = g.guard[1];
        const unsigned long long m = b0 < b1 ? b0 : b1;
        if (!(m < (1ull << 40) && m * (unsigned long long)g.guard_mul < (1ull << (FP6 ? 24 : 31)))) return;
    }
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    int tm, tn;
    tile_of(blockIdx.x, g.mtiles, g.ntiles, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const unsigned lds0 = (unsigned)(size_t)smem;

    // ---- global -> LDS: wave w fills rows [64w, 64w+64) of the A tile and of the B tile, 8 rows x 128 B
    // (1 KiB) per load; lane l writes slot l&7 of row l>>3, so it fetches the 16-byte chunk that
    // belongs there under the swizzle: chunk kc of row r lives at r*128 + ((kc ^ ((r >> 1) & 7)) << 4),
    // which makes the 64-lane ds_read_b128 of an MFMA operand (32 rows x 2 chunks) conflict-free.
    unsigned voffA[8], voffB[8];
#pragma unroll
    for (int u = 0; u < kLoads; ++u) {
        if (FP6) {  // slot u * 64 + lane of the wave's 64 x 7 slots: row slot / 7, piece slot % 7 (6 repeats 5)
            const int slot = u * 64 + lane;
            const int r = slot / 7, piece = min(slot - 7 * r, 5);
            const int row = 64 * wave + r;
            voffA[u] = (unsigned)row * (unsigned)g.ldA + (unsigned)(piece * 16);
            voffB[u] = (unsigned)row * (unsigned)g.ldB + (unsigned)(piece * 16);
        } else {
            const int row = 64 * wave + 8 * u + (lane >> 3);
            const int kc = (lane & 7) ^ ((row >> 1) & 7);
            voffA[u] = (unsigned)row * (unsigned)g.ldA + (unsigned)(kc * 16);
            voffB[u] = (unsigned)row * (unsigned)g.ldB + (unsigned)(kc * 16);
        }
    }
    const int8_t *gA = g.A + (int64_t)m0 * g.ldA, *gB = g.B + (int64_t)n0 * g.ldB;
    // Loads past the end of the range are clamped to the last k-tile: they land in a free slot and
    // are never read, which keeps the count of outstanding loads the same in every iteration.
    const int kt0 = g.kt0, kt1 = g.kt1;
    // The loads run two k-tiles ahead of the arithmetic and so cross into the next segment earlier: they
    // keep a segment pointer of their own.  Lane i holds the end and the block offset of segment i, so
    // that moving on to the next segment is two lane reads and no memory access inside the loop.
    const int v_end = lane < g.nbound ? g.bound_kt[lane] + 1 : kt1;
    const int v_delta = g.seg_delta[min(lane, g.nbound)];
    int la_seg = 0, la_end = __builtin_amdgcn_readlane(v_end, 0), la_delta = __builtin_amdgcn_readlane(v_delta, 0);
    auto ring = [](int slot, int k) { slot += k; return slot >= kRing ? slot - kRing : slot; };
    const int8_t *pg = nullptr;
    unsigned dl = 0;
    auto half_setup = [&](bool isA, int kt, int slot) {
        const int ktc = min(kt, kt1 - 1);
        int blk = ktc;
        if (isA) {
            // k-tiles are asked for in ascending order, one further per call: at most one segment ends
            la_seg += ktc >= la_end ? 1 : 0;
            la_end = __builtin_amdgcn_readlane(v_end, la_seg);
            la_delta = __builtin_amdgcn_readlane(v_delta, la_seg);
            blk = ktc + la_delta;
        }
        pg = uniform_ptr((isA ? gA : gB) + (int64_t)blk * kRowB);
        dl = __builtin_amdgcn_readfirstlane(lds0 + (unsigned)(slot * kHalfBytes) + (unsigned)(wave * kWaveBytes));
    };
    auto dma_one = [&](bool isA, int u) {  // u = 0..kLoads-1: the u-th KiB of the wave's rows of the half-stage set up last
        dma16(dl + u * 1024, isA ? voffA[u] : voffB[u], pg);
    };

    // ---- LDS -> registers: operand fragments of v_mfma_i32_32x32x32_i8 (lane: row lane%32, 16 K-bytes
    // at chunk 2*ks + lane/32 of the row)
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int swz = (lrow >> 1) & 7;
    const unsigned fa_base = (unsigned)((wm * 128 + lrow) * kPitch);
    const unsigned fb_base = (unsigned)((wn * 128 + lrow) * kPitch);
    unsigned kc_off[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) kc_off[ks] = FP6 ? (unsigned)(48 * ks + 16 * lhalf) : (unsigned)(((2 * ks + lhalf) ^ swz) << 4);
    using FragT = std::conditional_t<FP6, v8i, v4i>;
    using AccT = std::conditional_t<FP6, v16f, v16i>;
    FragT fa[2][4], fb[2][4];
    if (FP6) {
#pragma unroll
        for (int bq = 0; bq < 8; ++bq)
#pragma unroll
            for (int r = 0; r < (int)(sizeof(FragT) / 4); ++r) {
                fa[bq >> 2][bq & 3][r] = 0;
                fb[bq >> 2][bq & 3][r] = 0;
            }
    }
    // fragment q of a k-step in the order the MFMA sequence below first needs them: a0 b0 b1 a1 b2 b3 a2 a3
    auto load_frag = [&](const int8_t *sta, const int8_t *stb, int ks, int buf, int q) {
        constexpr int isA[8] = {1, 0, 0, 1, 0, 0, 1, 1};
        constexpr int idx[8] = {0, 0, 1, 1, 2, 3, 2, 3};
        const int8_t *src = isA[q] ? sta + fa_base + idx[q] * 32 * kPitch : stb + fb_base + idx[q] * 32 * kPitch;
        FragT &dst = isA[q] ? fa[buf][idx[q]] : fb[buf][idx[q]];
        if constexpr (FP6) {
            const v4i lo = *reinterpret_cast<const v4i *>(src + kc_off[ks]);
            const v2i hi = *reinterpret_cast<const v2i *>(src + 48 * ks + 32 + 8 * (lhalf ^ ((lrow >> 4) & 1)));
            dst[0] = lo[0]; dst[1] = lo[1]; dst[2] = lo[2]; dst[3] = lo[3];
            dst[4] = hi[0]; dst[5] = hi[1];
        } else {
            dst = *reinterpret_cast<const v4i *>(src + kc_off[ks]);
        }
    };
    auto mma = [&](const FragT &a, const FragT &b, AccT &c) {
        if constexpr (FP6) c = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 2, 2, 0, 0, 0, 0);  // e2m3 x e2m3, no scaling
        else c = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
    };

    AccT acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
    // MFMA order: 2 x 2 sub-blocks, so that the fragments of the next k-step can trickle in
    constexpr int mi[16] = {0, 0, 1, 1, 0, 0, 1, 1, 2, 2, 3, 3, 2, 2, 3, 3};
    constexpr int mj[16] = {0, 1, 0, 1, 2, 3, 2, 3, 0, 1, 0, 1, 2, 3, 2, 3};

    // One step = 16 MFMAs on the fragments in buffer `cur`, interleaved with the 8 fragment loads of
    // the next k-step into the other buffer and with `ndma` direct-to-LDS loads (starting at block
    // `dma0`) of the half-stage set up last.
    auto step = [&](int cur, const int8_t *sta, const int8_t *stb, int next_ks, bool isA, int dma0, int ndma) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            load_frag(sta, stb, next_ks, cur ^ 1, q);
            mma(fa[cur][mi[2 * q]], fb[cur][mj[2 * q]], acc[mi[2 * q]][mj[2 * q]]);
            if (q < ndma) dma_one(isA, dma0 + q);
            mma(fa[cur][mi[2 * q + 1]], fb[cur][mj[2 * q + 1]], acc[mi[2 * q + 1]][mj[2 * q + 1]]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    unsigned long long probe_c = 0, probe_w = 0;
    const bool probing = MODE == 0 && g.clock_probe != nullptr && blockIdx.x == 0;
    if (probing) {
        probe_c = __builtin_readcyclecounter();
        probe_w = wall_clock64();
    }
    // ---- prologue: k-tile kt0 landed, k-tile kt0+1 in flight, first fragments loaded
    int sa = 0;  // ring slot of A(kt); B(kt) is sa+1, A(kt+1) sa+2, B(kt+1) sa+3, A(kt+2) sa+4, B(kt+2) sa
    half_setup(true, kt0, 0);
#pragma unroll
    for (int u = 0; u < kLoads; ++u) dma_one(true, u);
    half_setup(false, kt0, 1);
#pragma unroll
    for (int u = 0; u < kLoads; ++u) dma_one(false, u);
    half_setup(true, kt0 + 1, 2);
#pragma unroll
    for (int u = 0; u < kLoads; ++u) dma_one(true, u);
    half_setup(false, kt0 + 1, 3);
#pragma unroll
    for (int u = 0; u < kLoads; ++u) dma_one(false, u);
    if (FP6) asm volatile("s_waitcnt vmcnt(14)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int q = 0; q < 8; ++q) load_frag(smem, smem + kHalfBytes, 0, 0, q);

    // ---- main loop, one 128-byte k-tile (4 k-steps, 64 MFMAs) and one barrier per iteration.
    // Steps 1-3 stream A(kt+2) into the spare slot.  After step 3 every fragment of k-tile kt has been
    // read (lgkmcnt(0)) and this wave's parts of A(kt+1), B(kt+1) have landed (all but the 8 newest
    // loads); past the barrier that holds for all waves, so step 4 may prefetch fragments of k-tile
    // kt+1 and stream B(kt+2) into the slot of A(kt).
    int kt = kt0;
    for (int seg = 0; seg <= g.nbound; ++seg) {
        if (seg > 0 && g.bound_sh[seg - 1] != 0) {  // start of the next exponent group: Horner step
            // The accumulators fill the whole accumulation register file (a0..a255), so shifting every
            // one of those registers shifts every accumulator, whichever block sits where.  Written
            // out by hand: left to the compiler, this step spills three blocks to scratch memory.
            const int shv = g.bound_sh[seg - 1];
            int t0, t1, t2, t3;
            if constexpr (FP6) {  // binary32 accumulators: times 2^shift, exact
                asm volatile(
                    "s_nop 15\n\ts_nop 7\n\t"
                    ".irp n," IMU_ACC_QUADS "\n\t"
                    "v_accvgpr_read_b32 %[t0], a[\\n]\n\t"
                    "v_accvgpr_read_b32 %[t1], a[\\n+1]\n\t"
                    "v_accvgpr_read_b32 %[t2], a[\\n+2]\n\t"
                    "v_accvgpr_read_b32 %[t3], a[\\n+3]\n\t"
                    "v_ldexp_f32 %[t0], %[t0], %[sh]\n\t"
                    "v_ldexp_f32 %[t1], %[t1], %[sh]\n\t"
                    "v_ldexp_f32 %[t2], %[t2], %[sh]\n\t"
                    "v_ldexp_f32 %[t3], %[t3], %[sh]\n\t"
                    "v_accvgpr_write_b32 a[\\n], %[t0]\n\t"
                    "v_accvgpr_write_b32 a[\\n+1], %[t1]\n\t"
                    "v_accvgpr_write_b32 a[\\n+2], %[t2]\n\t"
                    "v_accvgpr_write_b32 a[\\n+3], %[t3]\n\t"
                    ".endr\n\t"
                    "s_nop 7"
                    : [t0] "=&v"(t0), [t1] "=&v"(t1), [t2] "=&v"(t2), [t3] "=&v"(t3), "+a"(acc[0][0]), "+a"(acc[0][1]),
                      "+a"(acc[0][2]), "+a"(acc[0][3]), "+a"(acc[1][0]), "+a"(acc[1][1]), "+a"(acc[1][2]),
                      "+a"(acc[1][3]), "+a"(acc[2][0]), "+a"(acc[2][1]), "+a"(acc[2][2]), "+a"(acc[2][3]),
                      "+a"(acc[3][0]), "+a"(acc[3][1]), "+a"(acc[3][2]), "+a"(acc[3][3])
                    : [sh] "s"(shv));
            } else
            asm volatile(
                "s_nop 15\n\ts_nop 7\n\t"  // the last MFMA results must have landed
                ".irp n," IMU_ACC_QUADS "\n\t"
                "v_accvgpr_read_b32 %[t0], a[\\n]\n\t"
                "v_accvgpr_read_b32 %[t1], a[\\n+1]\n\t"
                "v_accvgpr_read_b32 %[t2], a[\\n+2]\n\t"
                "v_accvgpr_read_b32 %[t3], a[\\n+3]\n\t"
                "v_lshlrev_b32 %[t0], %[sh], %[t0]\n\t"
                "v_lshlrev_b32 %[t1], %[sh], %[t1]\n\t"
                "v_lshlrev_b32 %[t2], %[sh], %[t2]\n\t"
                "v_lshlrev_b32 %[t3], %[sh], %[t3]\n\t"
                "v_accvgpr_write_b32 a[\\n], %[t0]\n\t"
                "v_accvgpr_write_b32 a[\\n+1], %[t1]\n\t"
                "v_accvgpr_write_b32 a[\\n+2], %[t2]\n\t"
                "v_accvgpr_write_b32 a[\\n+3], %[t3]\n\t"
                ".endr\n\t"
                "s_nop 7"
                : [t0] "=&v"(t0), [t1] "=&v"(t1), [t2] "=&v"(t2), [t3] "=&v"(t3), "+a"(acc[0][0]), "+a"(acc[0][1]),
                  "+a"(acc[0][2]), "+a"(acc[0][3]), "+a"(acc[1][0]), "+a"(acc[1][1]), "+a"(acc[1][2]),
                  "+a"(acc[1][3]), "+a"(acc[2][0]), "+a"(acc[2][1]), "+a"(acc[2][2]), "+a"(acc[2][3]),
                  "+a"(acc[3][0]), "+a"(acc[3][1]), "+a"(acc[3][2]), "+a"(acc[3][3])
                : [sh] "s"(shv));
        }
        const int kend = seg < g.nbound ? g.bound_kt[seg] + 1 : kt1;
        for (; kt < kend; ++kt) {
            const int8_t *stA = smem + sa * kHalfBytes, *stB = smem + ring(sa, 1) * kHalfBytes;
            const int8_t *stA1 = smem + ring(sa, 2) * kHalfBytes, *stB1 = smem + ring(sa, 3) * kHalfBytes;
            half_setup(true, kt + 2, ring(sa, 4));
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (FP6) {  // two k-steps of 64 columns: the first streams A(kt+2), the second B(kt+2)
                step(0, stA, stB, 1, true, 0, 7);
                asm volatile("s_waitcnt vmcnt(7) lgkmcnt(0)" ::: "memory");
            } else {
                step(0, stA, stB, 1, true, 0, 3);
                step(1, stA, stB, 2, true, 3, 3);
                step(0, stA, stB, 3, true, 6, 2);
                asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
            }
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            half_setup(false, kt + 2, sa);
            __builtin_amdgcn_sched_barrier(0);
            step(1, stA1, stB1, 0, false, 0, kLoads);
            sa = ring(sa, 2);
        }
    }
    if (probing && tid == 0) {
        g.clock_probe[0] = __builtin_readcyclecounter() - probe_c;
        g.clock_probe[1] = wall_clock64() - probe_w;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // drain the clamped tail loads before LDS is reused
    __syncthreads();  // all fragment reads done: the buffers may be reused by the epilogue

    if (MODE == 1) {
        // un-fused: the int32 partial product of this exponent group goes, shifted, into the int64
        // unpacked product C_u (physical coordinates, padded to tiles: no bounds to check)
        constexpr int FLD1 = 260;
        int32_t *buf = reinterpret_cast<int32_t *>(smem);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            __syncthreads();
            if (wm == (c >> 1)) {
#pragma unroll
                for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            buf[(ii * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3)) * FLD1 + wn * 128 + jj * 32 + lrow] =
                                (int32_t)acc[(c & 1) * 2 + ii][jj][r];
            }
            __syncthreads();
            const int col4 = (tid & 63) * 4;
            for (int it = 0; it < 16; ++it) {
                const int row = (tid >> 6) + 4 * it;
                const v4i v = *reinterpret_cast<const v4i *>(buf + row * FLD1 + col4);
                int64_t *dst = g.C_u + (int64_t)(m0 + c * 64 + row) * g.Np + n0 + col4;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int64_t x = (int64_t)v[k] << g.seg_shift;
                    dst[k] = g.seg_first ? x : dst[k] + x;
                }
            }
        }
        return;
    }

    // ---- fused epilogue.  The accumulators leave the registers through LDS, one chunk of 64 physical
    // rows of the tile at a time ([64][256] int32, rows padded to 260), so that global stores are
    // row-contiguous and the digit levels of a source row (which the planner keeps inside one chunk)
    // and of a source column (inside one tile) can be added up:
    // C_int[i,j] = sum_{levels a of i, c of j} s^(a+c) * acc[row(i,a)][col(j,c)].
    const int jsrc0 = g.layB.tile_src0[tn], nsrcB = g.layB.tile_src0[tn + 1] - jsrc0;
    const bool flatA = g.flatA[tm] != 0, flatB = g.flatB[tn] != 0;
    constexpr int FLD = 260;
    int32_t *foldbuf = reinterpret_cast<int32_t *>(smem);  // two regions of [64][FLD]
    // behind the staging buffer: per source row of the tile its first physical row (relative to the
    // tile) | levels << 16; the same per source column; the first source row of each chunk
    int32_t *rowmeta = foldbuf + 2 * kChunk * FLD, *colmeta = rowmeta + kTile, *chunk0 = colmeta + kTile;
    // scale * 2^final_shift is exact: one multiplication in binary64, one rounding to fp32
    const double scale2 = (g.scale_a_dev ? (double)*g.scale_a_dev * (double)*g.scale_b_dev : g.scale) *
                          (double)(1ull << g.final_shift);
    {
        const int isrc0 = g.layA.tile_src0[tm], nsrcA = g.layA.tile_src0[tm + 1] - isrc0;
        if (!flatA && tid < nsrcA)
            rowmeta[tid] = (g.layA.src_pstart[isrc0 + tid] - m0) | (g.layA.src_nlev[isrc0 + tid] << 16);
        if (!flatB && tid < nsrcB)
            colmeta[tid] = (g.layB.src_pstart[jsrc0 + tid] - n0) | (g.layB.src_nlev[jsrc0 + tid] << 16);
        if (tid <= kTile / kChunk) chunk0[tid] = g.layA.chunk_src0[tm * (kTile / kChunk) + tid];
    }  // published by the first barrier below
    // Four results of one output row leave as 16 bytes of fp32 and / or 32 bytes of int64 (any element
    // boundary will do: a wave still writes a contiguous kilobyte), fewer than four at the ragged end of
    // a tile one by one.  v: the integer sums before the final shift.
    auto store4 = [&](int64_t o, int cols_left, auto v0, auto v1, auto v2, auto v3) {
        if constexpr (std::is_same<decltype(v0), double>::value) {  // exact integer sums held in binary64; no int64 output
            const float f[4] = {(float)(v0 * scale2), (float)(v1 * scale2), (float)(v2 * scale2), (float)(v3 * scale2)};
            if (cols_left >= 4) {
                v4f_u x;
                x[0] = f[0]; x[1] = f[1]; x[2] = f[2]; x[3] = f[3];
                __builtin_nontemporal_store(x, reinterpret_cast<v4f_u *>(g.C_fp + o));
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (k < cols_left) g.C_fp[o + k] = f[k];
            }
            return;
        }
        const int64_t w[4] = {(int64_t)v0, (int64_t)v1, (int64_t)v2, (int64_t)v3};
        float f[4];
        if (g.C_fp) {
            if constexpr (sizeof(v0) == 4) {
                f[0] = (float)((double)v0 * scale2); f[1] = (float)((double)v1 * scale2);
                f[2] = (float)((double)v2 * scale2); f[3] = (float)((double)v3 * scale2);
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) f[k] = (float)((double)w[k] * scale2);
            }
        }
        if (cols_left >= 4) {
            if (g.C_fp) {
                v4f_u x;
                x[0] = f[0]; x[1] = f[1]; x[2] = f[2]; x[3] = f[3];
                __builtin_nontemporal_store(x, reinterpret_cast<v4f_u *>(g.C_fp + o));
            }
            if (g.C_int) {
                v2l_u lo, hi;
                lo[0] = w[0] << g.final_shift; lo[1] = w[1] << g.final_shift;
                hi[0] = w[2] << g.final_shift; hi[1] = w[3] << g.final_shift;
                __builtin_nontemporal_store(lo, reinterpret_cast<v2l_u *>(g.C_int + o));
                __builtin_nontemporal_store(hi, reinterpret_cast<v2l_u *>(g.C_int + o + 2));
            }
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (k < cols_left) {
                    if (g.C_fp) g.C_fp[o + k] = f[k];
                    if (g.C_int) g.C_int[o + k] = w[k] << g.final_shift;
                }
        }
    };
    // two chunks per round: every wave parks 64 of its 128 rows (region wm of the staging buffer), then
    // all threads work the two chunks off
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        __syncthreads();
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    foldbuf[(wm * kChunk + ii * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3)) * FLD + wn * 128 + jj * 32 + lrow] =
                        (int32_t)acc[half * 2 + ii][jj][r];
        __syncthreads();
#pragma unroll 1
        for (int reg = 0; reg < 2; ++reg) {
            const int c = 2 * reg + half;  // chunk of the tile: rows [64 c, 64 c + 64)
            const int32_t *fold = foldbuf + reg * kChunk * FLD;
            // source rows of this chunk: cs0 .. cs0 + ns - 1; no source row straddles a chunk
            const int cs0 = chunk0[c], ns = chunk0[c + 1] - cs0;
            const int rs0 = cs0 - chunk0[0];  // index of the chunk's first source row in rowmeta
            if (flatB) {
                // source columns = physical columns: work items are (source row, four columns)
                const int col4 = (tid & 63) * 4;
                if (col4 < nsrcB && flatA) {  // physical order = source order inside the chunk
                    for (int r = tid >> 6; r < ns; r += kGemmThreads / 64) {
                        const v4i x = *reinterpret_cast<const v4i *>(fold + r * FLD + col4);
                        store4((int64_t)(cs0 + r) * g.ldc + jsrc0 + col4, nsrcB - col4, x[0], x[1], x[2], x[3]);
                    }
                } else if (col4 < nsrcB) {
                    // split rows: the digit levels of a source row are added up, four source rows at a time
                    // per thread so that their LDS reads are in flight together (a wave works on one row, so
                    // the level counts are uniform); in binary64 where every sum is exact in it
                    constexpr int RS = kGemmThreads / 64;
                    auto fold_rows = [&](auto zero) {
                        using T = decltype(zero);
                        for (int r0 = tid >> 6; r0 < ns; r0 += 4 * RS) {
                            int prel[4], nl[4];
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                const int m = r0 + u * RS < ns ? rowmeta[rs0 + r0 + u * RS] : 0;
                                prel[u] = (m & 0xFFFF) - c * kChunk;
                                nl[u] = m >> 16;  // 0 past the chunk's last source row
                            }
                            const int nlmax = max(max(nl[0], nl[1]), max(nl[2], nl[3]));
                            T v[4][4];
#pragma unroll
                            for (int u = 0; u < 4; ++u)
#pragma unroll
                                for (int k = 0; k < 4; ++k) v[u][k] = zero;
                            for (int l = 0; l < nlmax; ++l) {
                                v4i x[4];
#pragma unroll
                                for (int u = 0; u < 4; ++u)
                                    x[u] = l < nl[u] ? *reinterpret_cast<const v4i *>(fold + (prel[u] + l) * FLD + col4)
                                                     : v4i{0, 0, 0, 0};
                                if constexpr (std::is_same<T, double>::value) {
                                    const double wl = (double)(1ull << (g.sh * l));
#pragma unroll
                                    for (int u = 0; u < 4; ++u)
#pragma unroll
                                        for (int k = 0; k < 4; ++k) v[u][k] += (double)x[u][k] * wl;
                                } else {
#pragma unroll
                                    for (int u = 0; u < 4; ++u)
#pragma unroll
                                        for (int k = 0; k < 4; ++k) v[u][k] += (int64_t)x[u][k] << (g.sh * l);
                                }
                            }
#pragma unroll
                            for (int u = 0; u < 4; ++u)
                                if (r0 + u * RS < ns)
                                    store4((int64_t)(cs0 + r0 + u * RS) * g.ldc + jsrc0 + col4, nsrcB - col4, v[u][0],
                                           v[u][1], v[u][2], v[u][3]);
                        }
                    };
                    if (g.fold_f64) fold_rows(0.0);
                    else fold_rows((int64_t)0);
                }
            } else {
                // split source columns: lane l owns source columns 4l .. 4l+3 of the tile (where they sit in
                // the tile and how many digit levels each has is looked up once per chunk).  Four unsplit
                // columns side by side are the usual case and go the way of the flat tile (behind a split
                // column they no longer start at a multiple of four: four words rather than one vector).
                // A few other quads are then worked off one at a time with the wave's rows spread over its
                // lanes, so that their level loops run once per wave and quad, not once per row; if most
                // quads are of that kind, every lane works its own.
                const int j4 = (tid & 63) * 4;
                int q0[4], lj[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int cm = j4 + k < nsrcB ? colmeta[j4 + k] : 0;
                    q0[k] = cm & 0xFFFF;
                    lj[k] = cm >> 16;  // 0 past the last source column
                }
                const bool plain = lj[0] == 1 && lj[1] == 1 && lj[2] == 1 && lj[3] == 1 && q0[1] == q0[0] + 1 &&
                                   q0[2] == q0[0] + 2 && q0[3] == q0[0] + 3;
                const unsigned long long others = __ballot(j4 < nsrcB && !plain);
                auto row_levels = [&](int r, int &prel, int &nl) {
                    prel = r;
                    nl = 1;
                    if (!flatA) {
                        const int m = rowmeta[rs0 + r];
                        prel = (m & 0xFFFF) - c * kChunk;
                        nl = m >> 16;
                    }
                };
                if (plain) {
                    const bool aligned = (q0[0] & 3) == 0;
                    for (int r = tid >> 6; r < ns; r += kGemmThreads / 64) {
                        int prel, nl;
                        row_levels(r, prel, nl);
                        int64_t v[4] = {0, 0, 0, 0};
                        for (int a = 0; a < nl; ++a) {
                            const int32_t *row = fold + (prel + a) * FLD + q0[0];
                            v4i x;
                            if (aligned) {
                                x = *reinterpret_cast<const v4i *>(row);
                            } else {
                                x[0] = row[0]; x[1] = row[1]; x[2] = row[2]; x[3] = row[3];
                            }
#pragma unroll
                            for (int k = 0; k < 4; ++k) v[k] += (int64_t)x[k] << (g.sh * a);
                        }
                        store4((int64_t)(cs0 + r) * g.ldc + jsrc0 + j4, nsrcB - j4, v[0], v[1], v[2], v[3]);
                    }
                }
                const bool many = __popcll(others) > 8;  // mostly split columns: every lane works its own quad
                if (many && !plain && j4 < nsrcB) {
                    const int ljmax = max(max(lj[0], lj[1]), max(lj[2], lj[3]));
                    for (int r = tid >> 6; r < ns; r += kGemmThreads / 64) {
                        int prel, nl;
                        row_levels(r, prel, nl);
                        int64_t v[4] = {0, 0, 0, 0};
                        for (int a = 0; a < nl; ++a) {
                            const int32_t *row = fold + (prel + a) * FLD;
                            for (int l = 0; l < ljmax; ++l) {
                                int x[4];
#pragma unroll
                                for (int k = 0; k < 4; ++k) x[k] = l < lj[k] ? row[q0[k] + l] : 0;
#pragma unroll
                                for (int k = 0; k < 4; ++k) v[k] += (int64_t)x[k] << (g.sh * (a + l));
                            }
                        }
                        store4((int64_t)(cs0 + r) * g.ldc + jsrc0 + j4, nsrcB - j4, v[0], v[1], v[2], v[3]);
                    }
                }
                for (unsigned long long m = many ? 0ull : others; m; m &= m - 1) {
                    const int from = __builtin_ctzll(m);  // the lane that owns this quad
                    int Q0[4], LJ[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        Q0[k] = __builtin_amdgcn_readlane(q0[k], from);
                        LJ[k] = __builtin_amdgcn_readlane(lj[k], from);
                    }
                    const int ljmax = max(max(LJ[0], LJ[1]), max(LJ[2], LJ[3]));
                    const int r = (tid >> 6) + (kGemmThreads / 64) * (tid & 63);  // this wave's rows, one per lane
                    if (r < ns) {
                        int prel, nl;
                        row_levels(r, prel, nl);
                        int64_t v[4] = {0, 0, 0, 0};
                        for (int a = 0; a < nl; ++a) {
                            const int32_t *row = fold + (prel + a) * FLD;
                            for (int l = 0; l < ljmax; ++l) {
#pragma unroll
                                for (int k = 0; k < 4; ++k)
                                    if (l < LJ[k]) v[k] += (int64_t)row[Q0[k] + l] << (g.sh * (a + l));
                            }
                        }
                        store4((int64_t)(cs0 + r) * g.ldc + jsrc0 + 4 * from, nsrcB - 4 * from, v[0], v[1], v[2], v[3]);
                    }
                }
            }
        }
    }
}

template <int MODE>
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_i8_kernel(const GemmArgs g) {
    extern __shared__ __attribute__((aligned(1024))) int8_t smem[];
    gemm_body<MODE, false>(g, smem);
}

template <int MODE>
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_f6_kernel(const GemmArgs g) {
    extern __shared__ __attribute__((aligned(1024))) int8_t smem[];
    gemm_body<MODE, true>(g, smem);
}

// C_int = Pi_A C_u Pi_B^T from the int64 unpacked product, then dequantise.
__global__ __launch_bounds__(256) void recombine_kernel(const int64_t *__restrict__ C_u, int Np, RowLayout layA,
                                                        RowLayout layB, int n, int h, int sh,
                                                        int64_t *C_int, float *C_fp, int64_t ldc,
                                                        double scale_val, const float *scale_a_dev,
                                                        const float *scale_b_dev) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= h) return;
    const double scale = scale_a_dev ? (double)*scale_a_dev * (double)*scale_b_dev : scale_val;
    const int q0 = layB.src_pstart[j], lj = layB.src_nlev[j];
    for (int i = blockIdx.y; i < n; i += gridDim.y) {
        const int p0 = layA.src_pstart[i], li = layA.src_nlev[i];
        int64_t acc = 0;
        for (int a = 0; a < li; ++a)
            for (int c = 0; c < lj; ++c) acc += C_u[(int64_t)(p0 + a) * Np + (q0 + c)] << (sh * (a + c));
        const int64_t o = (int64_t)i * ldc + j;
        if (C_int) C_int[o] = acc;
        if (C_fp) C_fp[o] = (float)((double)acc * scale);
    }
}

// Register-resident back-to-back int8 MFMAs (no memory traffic): what the matrix cores sustain on
// this chip, for the measured-peak line of the benchmark.  Eight independent accumulators per wave.
__global__ __launch_bounds__(256) void mfma_peak_kernel(int iters, int *sink) {
    v4i a, b;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = (int)threadIdx.x + i;
        b[i] = (int)blockIdx.x + i;
    }
    v16i acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i], 0, 0, 0);
    }
    int x = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) x ^= acc[i][r];
    if (x == 0x7fffffff && sink) *sink = x;  // keeps the accumulators live
}

}  // namespace imu

using namespace imu;

// device memory of the caller, see imunpack_diag_clock_probe
static std::atomic<unsigned long long *> g_clock_probe{nullptr};

static int gemm_lds_opt_in() {
    // the kernels use all 160 KiB of a CU's LDS as dynamic shared memory, above the default limit; the
    // attribute is idempotent, so two threads racing through here both set the same value
    static std::atomic<int> done{0};
    if (!done.load(std::memory_order_acquire)) {
        IMU_HIP(hipFuncSetAttribute((const void *)gemm_i8_kernel<0>, hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds));
        IMU_HIP(hipFuncSetAttribute((const void *)gemm_i8_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds));
        IMU_HIP(hipFuncSetAttribute((const void *)gemm_f6_kernel<0>, hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds));
        IMU_HIP(hipFuncSetAttribute((const void *)gemm_f6_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds));
        done.store(1, std::memory_order_release);
    }
    return IMUNPACK_OK;
}

static int check_shifts(const Plan *p) {
    // every weight s^(levelA + levelB + e) applied in int64 must stay below 2^62
    const int maxexp = (p->hdr.lmaxA - 1) + (p->hdr.lmaxB - 1) + (p->hdr.ngroups ? p->hdr.grp_exp[0] : 0);
    return maxexp * p->sh <= 62 ? IMUNPACK_OK : IMUNPACK_ERANGE;
}

namespace imu {
int recombine_impl(const imunpack_plan_t *p, const void *workspace, float scale_A, float scale_B,
                   const float *scale_a_dev, const float *scale_b_dev, int64_t *C_int, float *C_fp, int64_t ldc,
                   hipStream_t stream) {
    if (!p || !p->valid || !workspace || ldc < p->h) return IMUNPACK_EINVAL;
    if (!C_int && !C_fp) return IMUNPACK_OK;
    IMU_TRY(check_shifts(p));
    dim3 grid((unsigned)((p->h + 255) / 256), (unsigned)std::min<int64_t>(p->n, 65535));
    hipLaunchKernelGGL(recombine_kernel, grid, dim3(256), 0, stream,
                       (const int64_t *)workspace, p->hdr.Np, p->layA, p->layB, (int)p->n, (int)p->h, p->sh,
                       C_int, C_fp, ldc, (double)scale_A * (double)scale_B, scale_a_dev, scale_b_dev);
    return launch_status();
}
}  // namespace imu

extern "C" int imunpack_recombine(const imunpack_plan_t *p, const void *workspace, float scale_A,
                                  float scale_B, int64_t *C_int, float *C_fp, int64_t ldc,
                                  imunpack_stream_t stream) {
    return recombine_impl(p, workspace, scale_A, scale_B, nullptr, nullptr, C_int, C_fp, ldc, (hipStream_t)stream);
}

namespace imu {
int gemm_impl(imunpack_plan_t *p, const int8_t *A_ue, const int8_t *B_eu, void *workspace, int64_t *C_int,
              float *C_fp, int64_t ldc, float scale_A, float scale_B, const float *scale_a_dev,
              const float *scale_b_dev, int fuse, imunpack_stream_t stream) {
    if (!p || !p->valid || !p->unpacked || !A_ue || !B_eu || (scale_a_dev == nullptr) != (scale_b_dev == nullptr))
        return IMUNPACK_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const PlanHeader &h = p->hdr;
    if (h.mtiles <= 0 || h.ntiles <= 0) return IMUNPACK_OK;
    IMU_TRY(check_shifts(p));
    IMU_TRY(gemm_lds_opt_in());
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.A = A_ue; g.B = B_eu;
    g.ldA = (int)store_pitch(p, 0); g.ldB = (int)store_pitch(p, 1); g.Kp = h.Kp; g.mtiles = h.mtiles; g.ntiles = h.ntiles;
    g.layA = p->layA; g.layB = p->layB;
    g.flatA = p->layA.tile_flat; g.flatB = p->layB.tile_flat;
    g.sh = p->sh;
    g.Np = h.Np;
    const int grid = h.mtiles * h.ntiles;
    bool fused = fuse != 0;
    const bool too_many_runs = h.nruns > 63;  // more segments than the lanes of a wave can hold the tables of
    // The bounds of the last imunpack_unpack may still be on their way to the host.  If the fused
    // launch was exact for this plan object the last time, it goes out now with a guard (the kernel
    // checks the bounds on the device and writes nothing if they are too large), and only then does
    // the host wait: the GPU does not idle while the answer travels.
    if (fused && too_many_runs) {
        if (!workspace) return IMUNPACK_ERANGE;
        fused = false;
    }
    const bool speculate = fused && p->bound_pending && p->guess_fusable;
    if (!speculate) {
        IMU_TRY(resolve_bound(p));
        if (fused && !p->fusable) {
            if (!workspace) return IMUNPACK_ERANGE;
            fused = false;
        }
    }
    if (fused) {
        if ((!C_int && !C_fp) || ldc < p->h) return IMUNPACK_EINVAL;
        g.guard = speculate ? p->d_hdr->bound : nullptr;
        g.guard_mul = p->s - 1;
        g.kt0 = 0; g.kt1 = h.Kp / BK;
        g.nbound = 0;
        for (int r = 0; r < h.nruns; ++r) {
            g.seg_delta[r] = h.run_blk0[r] - h.run_kt0[r];
            if (r + 1 < h.nruns) {
                g.bound_kt[g.nbound] = h.run_kt0[r + 1] - 1;
                g.bound_sh[g.nbound] = p->sh * (h.grp_exp[h.run_grp[r]] - h.grp_exp[h.run_grp[r + 1]]);
                ++g.nbound;
            }
        }
        g.final_shift = h.ngroups ? p->sh * h.grp_exp[h.ngroups - 1] : 0;
        g.C_int = C_int; g.C_fp = C_fp; g.ldc = ldc;
        g.scale = (double)scale_A * (double)scale_B;
        g.scale_a_dev = scale_a_dev; g.scale_b_dev = scale_b_dev;
        g.clock_probe = g_clock_probe.load(std::memory_order_relaxed);
        // |accumulator| < 2^31, weights up to s^(levels of a row - 1 + levels of a column - 1)
        g.fold_f64 = !C_int && 31 + p->sh * ((h.lmaxA - 1) + (h.lmaxB - 1)) <= 52;
        if (p->fp6) hipLaunchKernelGGL(gemm_f6_kernel<0>, dim3(grid), dim3(kGemmThreads), kGemmLds, st, g);
        else hipLaunchKernelGGL(gemm_i8_kernel<0>, dim3(grid), dim3(kGemmThreads), kGemmLds, st, g);
        IMU_TRY(launch_status());
        if (!speculate) return IMUNPACK_OK;
        IMU_TRY(resolve_bound(p));
        if (p->fusable) return IMUNPACK_OK;
        if (!workspace) return IMUNPACK_ERANGE;  // the guarded launch wrote nothing
        g.guard = nullptr;
    }
    if (!workspace) return IMUNPACK_EINVAL;
    g.C_u = (int64_t *)workspace;
    for (int r = 0; r < h.nruns; ++r) {  // one launch per stretch of consecutive blocks of the A store
        g.kt0 = h.run_kt0[r];
        g.kt1 = r + 1 < h.nruns ? h.run_kt0[r + 1] : h.Kp / BK;
        g.nbound = 0;
        g.seg_delta[0] = h.run_blk0[r] - h.run_kt0[r];
        g.seg_shift = p->sh * h.grp_exp[h.run_grp[r]];
        g.seg_first = r == 0;
        if (p->fp6) hipLaunchKernelGGL(gemm_f6_kernel<1>, dim3(grid), dim3(kGemmThreads), kGemmLds, st, g);
        else hipLaunchKernelGGL(gemm_i8_kernel<1>, dim3(grid), dim3(kGemmThreads), kGemmLds, st, g);
    }
    IMU_TRY(launch_status());
    if (fuse != 0)  // the caller asked for final outputs: finish the job here
        return recombine_impl(p, workspace, scale_A, scale_B, scale_a_dev, scale_b_dev, C_int, C_fp, ldc, st);
    return IMUNPACK_OK;
}
}  // namespace imu

extern "C" int imunpack_gemm(imunpack_plan_t *p, const int8_t *A_ue, const int8_t *B_eu,
                             void *workspace, int64_t *C_int, float *C_fp, int64_t ldc, float scale_A,
                             float scale_B, int fuse, imunpack_stream_t stream) {
    return gemm_impl(p, A_ue, B_eu, workspace, C_int, C_fp, ldc, scale_A, scale_B, nullptr, nullptr, fuse, stream);
}

extern "C" int imunpack_diag_clock_probe(uint64_t *ticks) {
    g_clock_probe.store(reinterpret_cast<unsigned long long *>(ticks), std::memory_order_relaxed);
    return IMUNPACK_OK;
}

extern "C" int imunpack_diag_mfma_peak(int workgroups, int iters, int64_t *ops, imunpack_stream_t stream) {
    if (workgroups <= 0 || workgroups > 65535 || iters <= 0 || iters > (1 << 24)) return IMUNPACK_EINVAL;
    hipLaunchKernelGGL(mfma_peak_kernel, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, iters, (int *)nullptr);
    // 4 waves per workgroup, 8 MFMAs per iteration, 2 * 32 * 32 * 32 operations each
    if (ops) *ops = (int64_t)workgroups * 4 * (int64_t)iters * 8 * 65536;
    return launch_status();
}
