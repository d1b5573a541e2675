// Digit scatter (Sec. 4, Eq. (mod); Alg. 1 l.4-5, Alg. 2 l.4-6, Alg. 4 l.7-8 and 11-13): writes the
// unpacked int8 operands in the plan's physical layout, gathering from the int32 operands: B_eu in
// full, and of A_ue every column of A_u once (the copies that column unpacking of the partner asks
// for, Alg. 2 line 6 / Alg. 4 line 13, are not stored: the GEMM reads a stored column wherever a copy
// of it stands).  HBM-bound: 4 B read per source element, 1 B written per stored element.
//
// Where an entry's digits go.  A split of a row (column) keeps digit 0 of every entry of that row
// (column) in place and moves floor(v / s) to the appended row (column); a row or column is split
// at most once.  So the digits of the original entry (i, k) lie on a chain of positions: the
// remainder sitting at (R, C) moves to the child of R if R was split before C, to the child of C
// otherwise, and every other descendant position holds 0.
//   - An operand unpacked by UnpackRow or UnpackColumn splits along one axis only: position (R, C)
//     with row level eR and column level eC holds digit eR + eC of its entry.  scatter_kernel<true>
//     writes all of it.
//   - An operand unpacked by UnpackBoth holds digit 0 at the level-(0, 0) position of every entry and
//     0 elsewhere, except along the chains of its OB entries.  scatter_kernel<false> writes the
//     former, fixup_kernel then places the higher digits of the listed OB entries.
#include "common.h"

namespace imu { int poll_ready(Plan *p); }

#include <algorithm>
#include <cstddef>
#include <cstring>

namespace imu {

// A wave writes kBandRows physical rows of one window of 64 output units (1024 stored columns): lane l
// owns unit l of the window.  Per row a lane reads the 16 source values of its unit (64 contiguous
// bytes when the unit copies 16 consecutive source columns, which the column layout makes the rule)
// and writes the unit's 16 bytes; the wave also leaves  sum_c w(c) |digit|  of what it wrote, its part
// of the row's weighted L1 norm.  The launch has exactly one wave per (band, window) of either
// operand, no empty workgroups, no staging and no barriers.  Short waves are what the memory system
// wants here: with two rows per wave (eight 16-byte loads per lane in flight, then out) the pass
// takes 0.10 ms on the benchmark workload, with 16 rows per wave (the unit's description decoded once
// for all of them) 0.17 ms, with 64 rows 0.42 ms; four rows at a time or one changed nothing.
constexpr int kScatterThreads = 256;
constexpr int kScatterWaves = kScatterThreads / 64;
constexpr int kBandRows = 2;  // divides kTile: the padded row counts are multiples of it

struct ScatterArgs {
    const int32_t *M;            // the int32 operand, row-major
    int64_t ldm;
    const int32_t *prow_slot, *prow_src, *prow_exp;  // per physical row
    const int32_t *col_k;        // per stored column: source column, -1 = none
    const int32_t *col_e;        // per stored column: digit level along this operand's column axis
    const unsigned long long *col_w;   // per stored column: weight in the row norm (nullptr: s^exponent of the unit)
    const int4 *unit;            // per 16 stored columns, see ColLayout
    const unsigned long long *unit_w;  // per unit: the weight its columns share (nullptr: s^exponent of the unit)
    int rows, W, ld, s, sh;      // physical rows, stored columns, bytes from one row of `out` to the next
    int nwin;                    // windows of 1024 stored columns
    int fp6;                     // store 6-bit floating-point codes (12 bytes per unit) instead of int8 digits
    int items;                   // waves that serve this operand: (rows / kBandRows) * nwin
    int8_t *out;
    unsigned long long *wavesum; // [rows][nwin]: every wave leaves its part of the row norm
};

typedef int v4i_u __attribute__((ext_vector_type(4), aligned(4)));  // 16 bytes at any int boundary

// Sign-magnitude digit at bit offset sft (`bits` wide) of four values, one per byte; mag += the four
// magnitudes.
__device__ __forceinline__ int digits4(const int (&x)[4], unsigned sft, int bits, unsigned &mag) {
    int dg[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int sx = x[i] >> 31;
        const unsigned av = (unsigned)((x[i] ^ sx) - sx);
        const int m = (int)__builtin_amdgcn_ubfe(av, sft, (unsigned)bits);
        mag += (unsigned)m;
        dg[i] = (m ^ sx) - sx;
    }
    return (int)(__builtin_amdgcn_perm((unsigned)dg[1], (unsigned)dg[0], 0x0c0c0400u) |
                 __builtin_amdgcn_perm((unsigned)dg[3], (unsigned)dg[2], 0x04000c0cu));
}

// Digit 0 of four values, on the four bytes at once.  With v = x mod s (the low bits of the two's
// complement), the sign-magnitude digit is v for x >= 0 and, for x < 0, 0 if v = 0 and v - s
// otherwise, which as a byte is v with the bits above the digit set.  mask4 = (s - 1) in every byte.
__device__ __forceinline__ int digit0x4(const int (&x)[4], unsigned mask4, unsigned &mag) {
    const unsigned l01 = __builtin_amdgcn_perm((unsigned)x[1], (unsigned)x[0], 0x07030400u);  // lo0 lo1 hi0 hi1
    const unsigned l23 = __builtin_amdgcn_perm((unsigned)x[3], (unsigned)x[2], 0x07030400u);
    const unsigned lo = __builtin_amdgcn_perm(l23, l01, 0x05040100u);  // the four low bytes
    const unsigned hi = __builtin_amdgcn_perm(l23, l01, 0x07060302u);  // the four high bytes (sign in bit 7)
    const unsigned v = lo & mask4;
    const unsigned nz = (v + 0x7f7f7f7fu) & 0x80808080u;              // bit 7: v != 0
    const unsigned t = hi & nz;                                        // bit 7: negative and v != 0
    const unsigned full = (t - (t >> 7)) | t;                          // 0xff in those bytes
    const unsigned r = v | (full & ~mask4);
    mag = __builtin_amdgcn_sad_u8(r ^ 0x80808080u, 0x80808080u, mag);  // sum of |int8|
    return (int)r;
}

// Four int8 digits in [-7, 7] (one per byte) -> their four e2m3 codes (one per byte): magnitudes 0..7 are
// 0, 1, 2, 1.5*2, 4, 1.25*4, 1.5*4, 1.75*4, i.e. the codes 0, 8, 16, 20, 24, 26, 28, 30; bit 5 is the sign.
__device__ __forceinline__ unsigned fp6_codes4(unsigned w) {
    const unsigned n = (w >> 7) & 0x01010101u;   // 1 in the negative bytes
    const unsigned s = (n << 8) - n;             // 0xff in the negative bytes
    const unsigned mag = (w ^ s) + n;            // |digit| per byte (no carries: every byte stays below 8)
    return __builtin_amdgcn_perm(0x1e1c1a18u, 0x14100800u, mag) | (n << 5);
}
// ... and squeezed to 24 bits, the first code lowest
__device__ __forceinline__ unsigned fp6_pack4(unsigned w) {
    const unsigned c = fp6_codes4(w);
    return (c & 0x3fu) | ((c >> 2) & 0xfc0u) | ((c >> 4) & 0x3f000u) | ((c >> 6) & 0xfc0000u);
}
typedef int v3i_u __attribute__((ext_vector_type(3), aligned(4)));
typedef int v2i_u __attribute__((ext_vector_type(2), aligned(4)));

__device__ __forceinline__ unsigned long long sat44(unsigned long long m, unsigned long long w) {
    if (m == 0) return 0;
    if (w >= (1ull << 44) || m >= (1ull << 20)) return 1ull << 44;
    const unsigned long long t = m * w;
    return t < (1ull << 44) ? t : (1ull << 44);
}

// Two operands in one launch when they take the same variant: waves below a0.items serve a0, the rest a1.
template <bool DENSE>
__global__ __launch_bounds__(kScatterThreads) void scatter_kernel(ScatterArgs a0, ScatterArgs a1) {
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63);
    int item = (int)blockIdx.x * kScatterWaves + wave;
    const bool second = item >= a0.items;
    const ScatterArgs &a = second ? a1 : a0;
    if (second) item -= a0.items;
    if (item >= a.items) return;  // uniform per wave; no barriers anywhere
    const int band = item / a.nwin, win = item - band * a.nwin;
    const int nunits = a.W >> 4;
    const int upos = win * 64 + lane;
    const bool inside = upos < nunits;
    const int4 ud = inside ? a.unit[upos] : make_int4(-1, -1, 7, 0);
    const int q0 = upos * 16;
    const int kmin = ud.x, kmax = ud.y;
    const bool run = (ud.z & 1) != 0, uniform = (ud.z & 2) != 0, onew = (ud.z & 4) != 0;
    const int ecu = ud.w & 0xFF;
    // what an entry of this unit weighs in the row norm: s^(exponent of S) for B_eu, the sum of those
    // over the column slots that read the stored column for A
    unsigned long long wgt = 0;
    if (inside && kmax >= 0)
        wgt = a.unit_w ? a.unit_w[upos] : ((ud.w >> 16) * a.sh >= 44 ? (1ull << 44) : (1ull << ((ud.w >> 16) * a.sh)));
    const unsigned mask4 = (unsigned)(a.s - 1) * 0x01010101u;
    const int p_first = band * kBandRows;
    constexpr int RS = 2;  // rows per step
    for (int r0 = 0; r0 < kBandRows; r0 += RS) {
        int si[RS], er[RS];
        bool live[RS];
        int v[RS][4][4];
        // ---- both rows' loads first
#pragma unroll
        for (int h = 0; h < RS; ++h) {
            const int p = __builtin_amdgcn_readfirstlane(p_first + r0 + h);
            const int slot = a.prow_slot[p];
            er[h] = a.prow_exp[p];
            si[h] = max(a.prow_src[p], 0);
            // padding row, padding unit, or (UnpackBoth operands hold digit 0 at level (0, 0) only; every
            // operand: no digit that high) a unit that holds nothing in this row
            const unsigned usft = (unsigned)(a.sh * (er[h] + ecu));
            live[h] = inside && slot >= 0 && kmax >= 0 && !(uniform && (DENSE ? usft >= 32u : er[h] + ecu != 0));

            if (live[h]) {
                const int32_t *src = a.M + (int64_t)si[h] * a.ldm;
                if (run) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const v4i_u x = *reinterpret_cast<const v4i_u *>(src + kmin + 4 * j);
                        v[h][j][0] = x.x; v[h][j][1] = x.y; v[h][j][2] = x.z; v[h][j][3] = x.w;
                    }
                } else {  // gather through the column table
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int4 kk = *reinterpret_cast<const int4 *>(a.col_k + q0 + 4 * j);
                        v[h][j][0] = kk.x >= 0 ? src[kk.x] : 0;
                        v[h][j][1] = kk.y >= 0 ? src[kk.y] : 0;
                        v[h][j][2] = kk.z >= 0 ? src[kk.z] : 0;
                        v[h][j][3] = kk.w >= 0 ? src[kk.w] : 0;
                    }
                }
            }
        }
        // ---- digits, store, norm
#pragma unroll
        for (int h = 0; h < RS; ++h) {
            const int p = p_first + r0 + h;
            unsigned mag = 0;               // sum of |digit| over the unit (columns that share the weight wgt)
            unsigned long long wsum = 0;    // weighted sum, for units whose columns weigh differently
            int4 o = make_int4(0, 0, 0, 0);
            if (live[h]) {
                int pk[4];
                const unsigned usft = (unsigned)(a.sh * (er[h] + ecu));
                if (uniform && onew) {
                    if (!DENSE || usft == 0u) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) pk[j] = digit0x4(v[h][j], mask4, mag);
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) pk[j] = digits4(v[h][j], usft, a.sh, mag);
                    }
                } else {  // a digit level and / or a weight per column
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int4 ee = *reinterpret_cast<const int4 *>(a.col_e + q0 + 4 * j);
                        const int ec[4] = {ee.x, ee.y, ee.z, ee.w};
                        int dg[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int t = er[h] + ec[i];
                            const unsigned sft = (unsigned)(a.sh * t);
                            const int one[4] = {v[h][j][i], 0, 0, 0};
                            unsigned m1 = 0;
                            const bool holds = DENSE ? sft < 32u : t == 0;
                            dg[i] = holds ? (digits4(one, sft, a.sh, m1) & 0xFF) : 0;
                            if (holds && m1) {
                                if (onew) mag += m1;
                                else wsum += sat44(m1, a.col_w[q0 + 4 * j + i]);
                            }
                        }
                        pk[j] = dg[0] | (dg[1] << 8) | (dg[2] << 16) | (dg[3] << 24);
                    }
                }
                o = make_int4(pk[0], pk[1], pk[2], pk[3]);
            }
            if (inside) {
                if (a.fp6) {  // uniform: 16 digits -> 96 bits
                    const unsigned t0 = fp6_pack4((unsigned)o.x), t1 = fp6_pack4((unsigned)o.y), t2 = fp6_pack4((unsigned)o.z),
                                   t3 = fp6_pack4((unsigned)o.w);
                    // the unit is the lower or the upper half of a 32-column fragment (see fp6_dword in common.h)
                    const int d0 = (int)(t0 | (t1 << 24)), d1 = (int)((t1 >> 8) | (t2 << 16)), d2 = (int)((t2 >> 16) | (t3 << 8));
                    int8_t *row = a.out + (int64_t)p * a.ld;
                    const int grp = upos >> 2, frag = (upos >> 1) & 1;
                    if ((upos & 1) == 0) {
                        v3i_u w3;
                        w3.x = d0; w3.y = d1; w3.z = d2;
                        *reinterpret_cast<v3i_u *>(row + 4 * fp6_dword(p, grp, frag, 0)) = w3;
                    } else {
                        *reinterpret_cast<int *>(row + 4 * fp6_dword(p, grp, frag, 3)) = d0;
                        v2i_u w2;
                        w2.x = d1; w2.y = d2;
                        *reinterpret_cast<v2i_u *>(row + 4 * fp6_dword(p, grp, frag, 4)) = w2;
                    }
                } else {
                    *reinterpret_cast<int4 *>(a.out + (int64_t)p * a.ld + q0) = o;
                }
            }
            // ---- the wave's part of the row norm
            const unsigned long long nz = __ballot(mag != 0 || wsum != 0);
            unsigned long long total = 0;
            if (nz != 0) {
                const int first = __builtin_ctzll(nz);
                const unsigned wlo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)wgt, first);
                const unsigned whi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(wgt >> 32), first);
                const unsigned long long w1 = ((unsigned long long)whi << 32) | wlo;
                if (__all(wsum == 0 && (mag == 0 || wgt == w1))) {  // one weight: add the magnitudes, weigh once
                    total = sat44(wave_sum_lane63(mag), w1);  // lane 63 holds the sum
                } else {
                    total = wsum + sat44(mag, wgt);
#pragma unroll
                    for (int off = 32; off > 0; off >>= 1) total += (unsigned long long)__shfl_xor((long long)total, off, 64);
                    if (total > (1ull << 44)) total = 1ull << 44;  // every lane holds the sum
                }
            }
            if (lane == 63) a.wavesum[(int64_t)p * a.nwin + win] = total;
        }
    }
}

// Places the digits above digit 0 of the listed OB entries of an operand unpacked by UnpackBoth.
// The remainder floor(|v| / s) of an entry at (R, C) moves to the child of whichever of R and C was
// split first (Alg. 4 lines 7-9 / 11-14) and leaves its own digit 0 there.
//   second == 0 (A): the entry's column chain lives in the column slots of A's unpacking; A_ue then
//     repeats column r of A_u in every column slot of the second unpacking that descends from r
//     (Alg. 2 line 6 / Alg. 4 line 13): the digit is stored wherever such a slot reads its column of A
//     (mostly one and the same stored column), and counts in the row norm once per such slot.
//   second == 1 (B): B_e holds a copy of column k of B in every column slot r of A's unpacking that
//     descends from k, and each copy is unpacked on its own.
struct FixupArgs {
    const int32_t *ob;          // [3][ob_cap] rows | columns | values
    int ob_cap;
    const int32_t *ob_count;
    int second;
    SlotSet rows, cset;         // the operand's row slots and the column slots of its own unpacking
    const int32_t *c1_child;    // second == 1: child links among the column slots of A's unpacking
    const int32_t *c2_child;    // second == 0: child links among the column slots of the second unpacking
    const int32_t *row_phys;
    const int32_t *out_col;     // per column slot of the second unpacking: the stored column that holds it
    const int32_t *col_phys, *col_sexp;  // its column of B_eu, and per such column the exponent of S
    int W, s, sh;               // bytes from one row of `out` to the next
    int fp6;                    // `out` holds 6-bit floating-point codes
    int8_t *out;
    unsigned long long *rowsum; // per physical row: what the digits placed here add to the row norm
};

// The whole norm of physical row p as far as it is known: the scatter kernel's parts plus `placed`.
__device__ __forceinline__ unsigned long long row_norm(const unsigned long long *wavesum, int wpr, int p,
                                                       unsigned long long placed) {
    unsigned long long t = placed;
    for (int w = 0; w < wpr; ++w) t += wavesum[(int64_t)p * wpr + w];
    return t < (1ull << 60) ? t : (1ull << 60);
}

// rowsum[p] += term for every lane that gets here together.  Atomics on one address are served one
// after the other, and the OB entries of a heavy row sit side by side in the list: in two rounds, the
// lanes that name the same row as the first lane still waiting are added up and share one atomic; the
// lanes left after that issue their own.
__device__ __forceinline__ void add_to_row(unsigned long long *rowsum, int p, unsigned long long term) {
    const int lane = threadIdx.x & 63;
    const int lo = (int)(unsigned)term, hi = (int)(unsigned)(term >> 32);
    unsigned long long pending = __ballot(1), sum = term;
    bool mine = true;  // this lane still has to issue its own atomic
    for (int round = 0; round < 2 && pending; ++round) {
        const int lead = __builtin_ctzll(pending);
        const int pl = __builtin_amdgcn_readlane(p, lead);
        const unsigned long long same = __ballot(mine && p == pl);
        if (same != (1ull << lead)) {  // uniform
            unsigned long long t = 0;
            for (unsigned long long m = same; m; m &= m - 1) {
                const int from = __builtin_ctzll(m);
                t += ((unsigned long long)(unsigned)__builtin_amdgcn_readlane(hi, from) << 32) |
                     (unsigned long long)(unsigned)__builtin_amdgcn_readlane(lo, from);
            }
            if (lane == lead) sum = t;
            else if (mine && p == pl) mine = false;  // carried by the leading lane
        }
        pending &= ~same;
    }
    if (mine) atomicAdd(&rowsum[p], sum);
}

// Both operands in one launch: blocks [0, blocks_a) serve fa, the next blocks_b serve fb.  What a digit
// placed here adds to its row's norm goes to rowsum; bound_kernel, launched behind this one, takes the
// largest norm (a wait for the sum inside this kernel, to keep the bound current entry by entry, was
// half its run time).
__global__ void fixup_kernel(FixupArgs fa, FixupArgs fb, int blocks_a, int blocks_b) {
    const bool first = (int)blockIdx.x < blocks_a;
    const FixupArgs &f = first ? fa : fb;
    const int block = first ? blockIdx.x : blockIdx.x - blocks_a;
    const int nblocks = first ? blocks_a : blocks_b;
    const int n = min(*f.ob_count, f.ob_cap);
    const unsigned mask = (unsigned)(f.s - 1);
    for (int t = block * blockDim.x + threadIdx.x; t < n; t += nblocks * blockDim.x) {
        const int i = f.ob[t], k = f.ob[f.ob_cap + t], v = f.ob[2 * (size_t)f.ob_cap + t];
        const unsigned av = v < 0 ? 0u - (unsigned)v : (unsigned)v;
        for (int croot = k, copies = 0; croot >= 0 && copies < 64; croot = f.second ? f.c1_child[croot] : -1, ++copies) {
            int R = i, C = croot;
            unsigned rem = av;
            for (int step = 0; step < 40; ++step) {
                rem >>= f.sh;
                if (rem == 0) break;
                const uint32_t tr = f.rows.time[R], tc = f.cset.time[C];
                if (tr < tc) R = f.rows.child[R];
                else if (tc != kNever) C = f.cset.child[C];
                else break;  // an OB remainder nothing splits: not a complete plan
                if (R < 0 || C < 0) break;
                const int m = (int)(rem & mask);
                if (m == 0) continue;
                const int p = f.row_phys[R];
                const int8_t dg = (int8_t)(v < 0 ? -m : m);
                for (int c = C, hops = 0; c >= 0 && hops < 4096; c = f.second ? -1 : f.c2_child[c], ++hops) {
                    if (f.fp6) {  // the position holds 0 (the scatter wrote it): OR the code in, 6 bits at bit 6 * column
                        const unsigned code = (fp6_codes4((unsigned)(uint8_t)dg) & 0x3fu);
                        const int col = f.out_col[c];
                        const unsigned bit = 6u * (unsigned)(col & 31);  // inside the 32-column fragment
                        unsigned *row = reinterpret_cast<unsigned *>(f.out + (int64_t)p * f.W);
                        const int grp = col >> 6, frag = (col >> 5) & 1, i = (int)(bit >> 5);
                        atomicOr(row + fp6_dword(p, grp, frag, i), code << (bit & 31u));
                        if ((bit & 31u) > 26u) atomicOr(row + fp6_dword(p, grp, frag, i + 1), code >> (32u - (bit & 31u)));
                    } else {
                        f.out[(int64_t)p * f.W + f.out_col[c]] = dg;
                    }
                    const unsigned nsft = (unsigned)(f.sh * f.col_sexp[f.col_phys[c]]);
                    const unsigned long long term = nsft >= 40u ? (1ull << 44) : ((unsigned long long)m << nsft);
                    add_to_row(f.rowsum, p, term);
                }
            }
        }
    }
}

// The accumulator bounds: the largest row norm of either operand (the scatter kernel's parts per wave
// plus what the fix-up pass placed).
__global__ void bound_kernel(const unsigned long long *rowsum_a, const unsigned long long *wavesum_a, int rows_a,
                             unsigned long long *bound_a, const unsigned long long *rowsum_b,
                             const unsigned long long *wavesum_b, int rows_b, unsigned long long *bound_b, int wpr_a,
                             int wpr_b) {
    unsigned long long ma = 0, mb = 0;
    for (int t = blockIdx.x * blockDim.x + threadIdx.x; t < rows_a + rows_b; t += gridDim.x * blockDim.x) {
        if (t < rows_a) ma = max(ma, row_norm(wavesum_a, wpr_a, t, rowsum_a[t]));
        else mb = max(mb, row_norm(wavesum_b, wpr_b, t - rows_a, rowsum_b[t - rows_a]));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        ma = max(ma, (unsigned long long)__shfl_xor((long long)ma, off, 64));
        mb = max(mb, (unsigned long long)__shfl_xor((long long)mb, off, 64));
    }
    if ((threadIdx.x & 63) == 0) {  // the bound only grows: a plain (possibly stale) read filters most of the updates
        if (ma > __hip_atomic_load(bound_a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(bound_a, ma);
        if (mb > __hip_atomic_load(bound_b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(bound_b, mb);
    }
}

// A repeated unpack of one plan: clears what the planner left cleared for the first.
__global__ void reset_bound_kernel(PlanHeader *hdr, unsigned long long *rowsum_a, int rows_a,
                                   unsigned long long *rowsum_b, int rows_b) {
    const int t0 = blockIdx.x * blockDim.x + threadIdx.x, stride = gridDim.x * blockDim.x;
    if (t0 == 0) hdr->bound[0] = hdr->bound[1] = 0;
    for (int t = t0; t < rows_a; t += stride) rowsum_a[t] = 0;
    for (int t = t0; t < rows_b; t += stride) rowsum_b[t] = 0;
}

// canon[R][c] = phys[row_phys[R]][col_phys[c]]; Kp: stored columns per physical row
__global__ void canonical_kernel(const int8_t *__restrict__ phys, int Kp, const int32_t *row_phys,
                                 const int32_t *col_phys, int nrows, int ncols, int8_t *__restrict__ canon, int fp6) {
    const int R = blockIdx.x;
    if (R >= nrows) return;
    const int8_t *src = phys + (int64_t)row_phys[R] * Kp;
    for (int c = threadIdx.x; c < ncols; c += blockDim.x) {
        int8_t v;
        if (fp6) {  // e2m3 code at bit 6 * column -> the integer it stands for (digits are integers)
            const int col = col_phys[c];
            const unsigned bit = 6u * (unsigned)(col & 31);
            const unsigned *row = reinterpret_cast<const unsigned *>(src);
            const int grp = col >> 6, frag = (col >> 5) & 1, i = (int)(bit >> 5);
            const int pr = row_phys[R];
            unsigned long long two = row[fp6_dword(pr, grp, frag, i)];
            if ((bit & 31u) > 26u) two |= (unsigned long long)row[fp6_dword(pr, grp, frag, i + 1)] << 32;
            const unsigned code = (unsigned)(two >> (bit & 31u)) & 0x3fu;
            const unsigned e = (code >> 3) & 3u, m = code & 7u;
            const unsigned eighths = e == 0 ? m : ((8u + m) << (e - 1));   // value * 8
            const int mag = (int)(eighths >> 3);
            v = (int8_t)((code & 32u) ? -mag : mag);
        } else {
            v = src[col_phys[c]];
        }
        canon[(int64_t)R * ncols + c] = v;
    }
}

}  // namespace imu

using namespace imu;

extern "C" int imunpack_unpacked_bytes(const imunpack_plan_t *p, size_t *bytes_A, size_t *bytes_B,
                                       size_t *bytes_workspace) {
    if (!p || !p->valid) return IMUNPACK_EINVAL;
    if (bytes_A) *bytes_A = (size_t)p->hdr.Mp * (size_t)store_pitch(p, 0);
    if (bytes_B) *bytes_B = (size_t)p->hdr.Np * (size_t)store_pitch(p, 1);
    if (bytes_workspace) *bytes_workspace = (size_t)p->hdr.Mp * p->hdr.Np * sizeof(int64_t);
    return IMUNPACK_OK;
}

extern "C" int imunpack_plan_set_digits(imunpack_plan_t *p, int format) {
    if (!p || !p->valid || (format != IMUNPACK_DIGITS_INT8 && format != IMUNPACK_DIGITS_FP6)) return IMUNPACK_EINVAL;
    if (format == IMUNPACK_DIGITS_FP6 && p->b > 4) return IMUNPACK_EINVAL;
    if (p->bound_pending) IMU_TRY(resolve_bound(p));  // of an unpack in the other format
    p->digits_req = format;
    p->fp6 = format == IMUNPACK_DIGITS_FP6;
    p->kept_Beu = nullptr;
    return IMUNPACK_OK;
}

extern "C" int imunpack_plan_digits(const imunpack_plan_t *p) {
    return (p && p->valid && p->fp6) ? IMUNPACK_DIGITS_FP6 : IMUNPACK_DIGITS_INT8;
}

extern "C" int imunpack_plan_layout(const imunpack_plan_t *p, int64_t *shape) {
    if (!p || !p->valid || !shape) return IMUNPACK_EINVAL;
    const int64_t v[6] = {p->hdr.Mp, p->hdr.KA, store_pitch(p, 0), p->hdr.Np, p->hdr.Kp, store_pitch(p, 1)};
    memcpy(shape, v, sizeof(v));
    return IMUNPACK_OK;
}

extern "C" int imunpack_unpack(imunpack_plan_t *p, const int32_t *A, int64_t lda, const int32_t *B,
                               int64_t ldb, int8_t *A_ue, int8_t *B_eu, imunpack_stream_t stream) {
    if (!p || !p->valid || !A || !B || !A_ue || !B_eu || lda < p->d || ldb < p->d) return IMUNPACK_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const PlanHeader &h = p->hdr;
    if (p->bound_pending) IMU_TRY(resolve_bound(p));  // of an earlier unpack of this plan
    // the planner leaves the bounds and the row norms cleared; a repeated unpack of the same plan clears them again
    if (p->unpacked)
        hipLaunchKernelGGL(reset_bound_kernel, dim3(64), dim3(256), 0, st, p->d_hdr, p->layA.rowsum, h.Mp,
                           p->layB.rowsum, h.Np);
    FixupArgs fx[2] = {};
    int fblocks[2] = {0, 0};
    ScatterArgs sc[2];
    memset(sc, 0, sizeof(sc));
    bool launch[2] = {false, false}, dense[2] = {false, false};
    // keep-weights mode: the plan took the second operand's unpacking over, and the caller's buffer still holds
    // what the unpack before wrote for exactly that unpacking (same buffer, same format, row norms in place)
    const bool keepB = p->keep_B && h.reusedB && !p->unpacked && p->kept_Beu == B_eu && p->kept_Beu_fp6 == p->fp6;
    for (int op = 0; op < 2; ++op) {
        const int rowsP = op ? h.Np : h.Mp;
        const int W = op ? h.Kp : h.KA;
        if (rowsP <= 0 || W <= 0) continue;
        const RowLayout &lay = op ? p->layB : p->layA;
        const bool both = (op ? p->sB : p->sA) == IMUNPACK_BOTH;
        ScatterArgs &a = sc[op];
        a.M = op ? B : A; a.ldm = op ? ldb : lda;
        a.prow_slot = lay.prow_slot; a.prow_src = lay.prow_src; a.prow_exp = lay.prow_exp;
        a.col_k = op ? p->cols.colB_k : p->cols.colA_k;
        a.col_e = op ? p->cols.colB_e : p->cols.colA_e;
        a.col_w = op ? nullptr : p->cols.colA_w;
        a.unit = op ? p->cols.unitB : p->cols.unitA;
        a.unit_w = op ? nullptr : p->cols.unitA_w;
        a.rows = rowsP; a.W = W; a.ld = (int)store_pitch(p, op); a.s = p->s; a.sh = p->sh; a.fp6 = p->fp6;
        a.nwin = (W + 1023) / 1024;
        a.items = (rowsP / kBandRows) * a.nwin;
        a.out = op ? B_eu : A_ue;
        a.wavesum = lay.wavesum;
        launch[op] = !(op == 1 && keepB);
        dense[op] = !both;
        const int nob = op ? h.nobB : h.nobA;
        if (both && nob > 0 && launch[op]) {
            FixupArgs &f = fx[op];
            f.ob = op ? p->obcopyB : p->obcopyA;
            f.ob_cap = p->cap[op ? CAP_EDGEB : CAP_EDGEA];
            f.ob_count = op ? &p->d_hdr->nobB : &p->d_hdr->nobA;
            f.second = op;
            f.rows = op ? p->rowB : p->rowA;
            f.cset = op ? p->c2 : p->c1;
            f.c1_child = p->c1.child;
            f.c2_child = p->c2.child;
            f.row_phys = lay.row_phys;
            f.out_col = op ? p->cols.col_phys : p->cols.acol_phys;
            f.col_phys = p->cols.col_phys; f.col_sexp = p->cols.col_sexp;
            f.W = (int)store_pitch(p, op); f.s = p->s; f.sh = p->sh; f.fp6 = p->fp6;
            f.out = a.out; f.rowsum = lay.rowsum;
            fblocks[op] = (nob + 255) / 256;
        }
    }
    auto scatter = [&](const ScatterArgs &x, const ScatterArgs &y, int items, bool dns) {
        const dim3 grid((unsigned)((items + kScatterWaves - 1) / kScatterWaves));
        if (dns) hipLaunchKernelGGL(scatter_kernel<true>, grid, dim3(kScatterThreads), 0, st, x, y);
        else hipLaunchKernelGGL(scatter_kernel<false>, grid, dim3(kScatterThreads), 0, st, x, y);
    };
    ScatterArgs none;
    memset(&none, 0, sizeof(none));
    if (launch[0] && launch[1] && dense[0] == dense[1]) {  // one launch: the tail of A overlaps the head of B
        scatter(sc[0], sc[1], sc[0].items + sc[1].items, dense[0]);
    } else {
        for (int op = 0; op < 2; ++op)
            if (launch[op]) scatter(sc[op], none, sc[op].items, dense[op]);
    }
    if (h.Kp > 0 && h.Mp + h.Np > 0) {
        // after both scatters: the fix-up overwrites zeros they wrote; then the bounds from the row norms
        if (fblocks[0] + fblocks[1] > 0) {
            if (!fblocks[0]) fx[0] = fx[1];  // never dereferenced, but keep the argument well-formed
            if (!fblocks[1]) fx[1] = fx[0];
            hipLaunchKernelGGL(fixup_kernel, dim3(fblocks[0] + fblocks[1]), dim3(256), 0, st, fx[0], fx[1], fblocks[0],
                               fblocks[1]);
        }
        const int nscan = std::min(256, (h.Mp + h.Np + 255) / 256);
        hipLaunchKernelGGL(bound_kernel, dim3(nscan), dim3(256), 0, st, p->layA.rowsum, p->layA.wavesum, h.Mp,
                           &p->d_hdr->bound[0], p->layB.rowsum, p->layB.wavesum, h.Np, &p->d_hdr->bound[1],
                           sc[0].nwin, sc[1].nwin);
    }
    IMU_TRY(launch_status());
    // The bounds travel to the host on the plan's side stream, behind the scatter: the caller's stream is
    // free to take the GEMM at once (imunpack_gemm launches it guarded and then waits for the bounds).
    IMU_HIP(hipEventRecord(p->scattered, st));
    IMU_HIP(hipStreamWaitEvent(p->side, p->scattered, 0));
    IMU_HIP(hipMemcpyAsync(reinterpret_cast<char *>(p->pin_hdr) + offsetof(PlanHeader, bound),
                           reinterpret_cast<const char *>(p->d_hdr) + offsetof(PlanHeader, bound),
                           sizeof(p->hdr.bound), hipMemcpyDeviceToHost, p->side));
    IMU_HIP(hipEventRecord(p->ready, p->side));
    p->bound_pending = 1;
    p->unpacked = 1;
    p->kept_Beu = p->keep_B ? B_eu : nullptr;
    p->kept_Beu_fp6 = p->fp6;
    return IMUNPACK_OK;
}

namespace imu {
int resolve_bound(Plan *p) {
    if (!p->bound_pending) return IMUNPACK_OK;
    p->bound_pending = 0;
    IMU_TRY(poll_ready(p));
    memcpy(p->hdr.bound, p->pin_hdr->bound, sizeof(p->hdr.bound));
    // |sum_c s^e(c) a_c b_c| <= (s - 1) * min(bound_A, bound_B): the shifted sum of all groups
    // fits int32 iff that is below 2^31.
    const unsigned long long m = p->hdr.bound[0] < p->hdr.bound[1] ? p->hdr.bound[0] : p->hdr.bound[1];
    // (6-bit floating-point digits accumulate in binary32: exact below 2^24)
    p->fusable = (m < (1ull << 40)) && (m * (unsigned long long)(p->s - 1) < (1ull << (p->fp6 ? 24 : 31)));
    p->guess_fusable = p->fusable;
    return IMUNPACK_OK;
}
}  // namespace imu

extern "C" int imunpack_plan_fusable(imunpack_plan_t *p) {
    if (!p || !p->valid || !p->unpacked) return 0;
    if (resolve_bound(p) != IMUNPACK_OK) return 0;
    return p->fusable;
}

extern "C" int imunpack_plan_bounds(imunpack_plan_t *p, uint64_t *bound) {
    if (!p || !p->valid || !p->unpacked || !bound) return IMUNPACK_EINVAL;
    IMU_TRY(resolve_bound(p));
    bound[0] = p->hdr.bound[0];
    bound[1] = p->hdr.bound[1];
    return IMUNPACK_OK;
}

namespace imu { int ensure_canonical(Plan *p); }

extern "C" int imunpack_unpack_canonical(imunpack_plan_t *p, const int8_t *A_ue, const int8_t *B_eu,
                                         int8_t *A_canon, int8_t *B_canon, imunpack_stream_t stream) {
    if (!p || !p->valid) return IMUNPACK_EINVAL;
    IMU_TRY(ensure_canonical(p));  // host-side renumbering into the paper's order (synchronises)
    hipStream_t st = (hipStream_t)stream;
    const PlanHeader &h = p->hdr;
    if (A_ue && A_canon && h.n_u > 0)
        hipLaunchKernelGGL(canonical_kernel, dim3(h.n_u), dim3(256), 0, st, A_ue, (int)store_pitch(p, 0), p->canon_rowphysA,
                           p->canon_acolphys, h.n_u, h.d_u, A_canon, p->fp6);
    if (B_eu && B_canon && h.h_u > 0)
        hipLaunchKernelGGL(canonical_kernel, dim3(h.h_u), dim3(256), 0, st, B_eu, (int)store_pitch(p, 1), p->canon_rowphysB,
                           p->canon_colphys, h.h_u, h.d_u, B_canon, p->fp6);
    return launch_status();
}
