// Digit scatter (Sec. 4, Eq. (mod); Alg. 1 l.4-5, Alg. 2 l.4-6, Alg. 4 l.7-8 and 11-13): writes the
// unpacked int8 operands A_ue and B_eu in the plan's physical layout, gathering from the int32
// operands.  HBM-bound: 4 B read per source element, 1 B written per unpacked element.
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

#include <cstddef>
#include <cstring>

namespace imu {

// One workgroup handles kScatterRows consecutive physical rows and walks the source in windows of
// kScatterWin columns.  A window of the block's source rows (all digit levels of a source row are
// adjacent, so the block has few distinct ones) is staged in LDS once; every 16-column output unit
// whose first column copies a source column of the window is then produced from LDS -- the columns of
// a group are ordered by source column, so the units of every group advance with the window and
// each source element is read from HBM once.  A column that copies a source column outside the
// window (the tail of a unit that straddles two windows, or a sparse group) is read from global
// memory instead.  Stores are 16 bytes wide.  The kernel also leaves, per physical row, the weighted
// L1 norm sum_c s^e(c) |digit| of what it wrote, and raises *bound to the largest of them.
constexpr int kScatterRows = 8;
constexpr int kScatterThreads = 256;
static_assert(kScatterWin == 4 * kScatterThreads, "one int4 per thread and staged row");

struct ScatterArgs {
    const int32_t *M;            // the int32 operand, row-major
    int64_t ld;
    const int32_t *prow_slot, *prow_src, *prow_exp;  // per physical row
    const int32_t *col_k;        // per physical column: source column, -1 = padding
    const int32_t *col_e;        // per physical column: digit level along this operand's column axis
    const int4 *unit_desc;
    int lev_shift;               // where this operand's level sits in unit_desc.w
    const int32_t *win_unit;
    int Mp, Kp, d, ngroups, s, sh;
    int8_t *out;
    unsigned long long *rowsum, *bound;
};

template <bool DENSE>
__global__ __launch_bounds__(kScatterThreads) void scatter_kernel(ScatterArgs a) {
    // rows padded by 16 bytes: lanes that read the same columns of different rows hit different banks
    __shared__ __attribute__((aligned(16))) int32_t tile[kScatterRows][kScatterWin + 4];
    __shared__ int s_slot[kScatterRows], s_src[kScatterRows], s_er[kScatterRows], s_trow[kScatterRows];
    __shared__ unsigned long long s_wsum[kScatterRows];
    __shared__ int s_u0[kMaxGroups + 1], s_ucount[kMaxGroups + 1], s_total;
    const int p0 = blockIdx.x * kScatterRows;
    const int nwin = (a.d + kScatterWin - 1) / kScatterWin;
    const int s = a.s, sh = a.sh, Kp = a.Kp, d = a.d;
    if (threadIdx.x < kScatterRows) {
        const int p = p0 + threadIdx.x;
        s_slot[threadIdx.x] = p < a.Mp ? a.prow_slot[p] : -2;
        s_src[threadIdx.x] = p < a.Mp ? a.prow_src[p] : -1;
        s_er[threadIdx.x] = p < a.Mp ? a.prow_exp[p] : 0;
        s_wsum[threadIdx.x] = 0;
    }
    __syncthreads();
    // s_trow[r]: which staged row holds the source row of physical row r
    if (threadIdx.x < kScatterRows) {
        int r = threadIdx.x;
        while (r > 0 && s_src[r] >= 0 && s_src[r - 1] == s_src[r]) --r;
        s_trow[threadIdx.x] = r;
    }
    __syncthreads();
    const bool ld_vec = (a.ld % 4) == 0 && ((uintptr_t)a.M % 16) == 0;
    auto fetch = [&](int w, int4 (&pre)[kScatterRows]) {
        const int k = w * kScatterWin + (int)threadIdx.x * 4;
#pragma unroll
        for (int r = 0; r < kScatterRows; ++r) {
            pre[r] = make_int4(0, 0, 0, 0);
            const int si = s_src[r];
            if (s_trow[r] != r || si < 0 || w >= nwin) continue;
            const int32_t *src = a.M + (int64_t)si * a.ld;
            if (ld_vec && k + 3 < d) {
                pre[r] = *reinterpret_cast<const int4 *>(src + k);
            } else {
                if (k < d) pre[r].x = src[k];
                if (k + 1 < d) pre[r].y = src[k + 1];
                if (k + 2 < d) pre[r].z = src[k + 2];
                if (k + 3 < d) pre[r].w = src[k + 3];
            }
        }
    };
    int4 pre[kScatterRows];
    fetch(0, pre);
    const int mask = s - 1;
    for (int w = 0; w < nwin; ++w) {
        if (w > 0) __syncthreads();  // the previous window has been consumed
#pragma unroll
        for (int r = 0; r < kScatterRows; ++r)
            *reinterpret_cast<int4 *>(&tile[r][threadIdx.x * 4]) = pre[r];
        if ((int)threadIdx.x < a.ngroups) {
            const int g = threadIdx.x;
            const int u0 = a.win_unit[g * (nwin + 1) + w], u1 = a.win_unit[g * (nwin + 1) + w + 1];
            s_u0[g] = u0;
            s_ucount[g] = u1 - u0;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            int total = 0;
            for (int g = 0; g < a.ngroups; ++g) total += s_ucount[g];
            s_total = total;
        }
        fetch(w + 1, pre);  // in flight while this window is processed
        __syncthreads();
        const int kbase = w * kScatterWin;
        const int total = s_total;
        // work items: (unit, half of the block's rows), flattened over the groups; the last, partial
        // round of such items is dealt out row by row instead, so that it costs one row per thread
        // rather than four
        const int n4 = 2 * total, full = n4 / kScatterThreads * kScatterThreads;
        const int nitems = full + (n4 - full) * (kScatterRows / 2);
        for (int item = threadIdx.x; item < nitems; item += kScatterThreads) {
            int it4 = item, rbeg, rcount;
            if (item < full) {
                rbeg = (item & 1) * (kScatterRows / 2);
                rcount = kScatterRows / 2;
            } else {
                const int t = item - full;
                it4 = full + t / (kScatterRows / 2);
                rbeg = (it4 & 1) * (kScatterRows / 2) + t % (kScatterRows / 2);
                rcount = 1;
            }
            int ui = it4 >> 1, g = 0;
            while (ui >= s_ucount[g]) ui -= s_ucount[g++];
            const int unit = s_u0[g] + ui, q0 = unit * 16;
            const int4 ud = a.unit_desc[unit];
            const int kmin = ud.x, kmax = ud.y;
            const bool run = (ud.z & 1) != 0, uniform = (ud.z & 2) != 0;
            const int ecu = (ud.w >> a.lev_shift) & 0xFF;
            const unsigned nsft = (unsigned)(sh * ((ud.w >> 16) & 0xFF));  // weight of the unit's columns in the row norm
            const bool staged = kmin >= kbase && kmax < kbase + kScatterWin;
            int k[16], ec[16];
            if (kmax >= 0 && !run) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int4 kk = *reinterpret_cast<const int4 *>(a.col_k + q0 + 4 * u);
                    k[4 * u] = kk.x; k[4 * u + 1] = kk.y; k[4 * u + 2] = kk.z; k[4 * u + 3] = kk.w;
                }
            } else {
#pragma unroll
                for (int j = 0; j < 16; ++j) k[j] = kmin + j;
            }
            if (kmax >= 0 && !uniform) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int4 ee = *reinterpret_cast<const int4 *>(a.col_e + q0 + 4 * u);
                    ec[4 * u] = ee.x; ec[4 * u + 1] = ee.y; ec[4 * u + 2] = ee.z; ec[4 * u + 3] = ee.w;
                }
            } else {
#pragma unroll
                for (int j = 0; j < 16; ++j) ec[j] = ecu;
            }
#pragma unroll 1
            for (int rr = 0; rr < rcount; ++rr) {
                const int r = rbeg + rr;
                const int slot = s_slot[r];
                if (slot == -2) break;  // past the last physical row
                int4 *dst = reinterpret_cast<int4 *>(a.out + (int64_t)(p0 + r) * Kp + q0);
                const int er = s_er[r];
                if (slot < 0 || kmax < 0 || (!DENSE && uniform && er + ecu != 0)) {
                    // padding row, padding columns, or a unit that holds no level-0 position
                    *dst = make_int4(0, 0, 0, 0);
                    continue;
                }
                // ---- the source values
                const int32_t *trow = tile[s_trow[r]];
                int32_t v[16];
                if (run && staged) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int4 x = *reinterpret_cast<const int4 *>(trow + (kmin - kbase) + 4 * u);
                        v[4 * u] = x.x; v[4 * u + 1] = x.y; v[4 * u + 2] = x.z; v[4 * u + 3] = x.w;
                    }
                } else {
                    bool miss = false;
#pragma unroll
                    for (int j = 0; j < 16; ++j) {
                        const unsigned off = (unsigned)(k[j] - kbase);
                        const bool in = off < (unsigned)kScatterWin;
                        v[j] = trow[in ? off : 0u];
                        if (!in) v[j] = 0;
                        miss = miss || (!in && k[j] >= 0);
                    }
                    if (miss) {  // rare: a source column outside the staged window
                        const int32_t *src = a.M + (int64_t)s_src[r] * a.ld;
#pragma unroll
                        for (int j = 0; j < 16; ++j) {
                            const unsigned off = (unsigned)(k[j] - kbase);
                            if (k[j] >= 0 && off >= (unsigned)kScatterWin) v[j] = src[k[j]];
                        }
                    }
                }
                // ---- digits (sign-magnitude)
                int pk[4];
                unsigned mag = 0;  // sum of |digit| over the unit
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    int dg[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int x = v[4 * u + i];
                        const int t = er + ec[4 * u + i];
                        if (DENSE) {
                            const unsigned sft = (unsigned)(sh * t);
                            const unsigned av = x < 0 ? 0u - (unsigned)x : (unsigned)x;
                            const int m = sft >= 32u ? 0 : (int)((av >> sft) & (unsigned)mask);
                            dg[i] = x < 0 ? -m : m;
                        } else {
                            // digit 0: x - s * trunc(x / s)
                            const int d0 = x - ((x + ((x >> 31) & mask)) & ~mask);
                            dg[i] = t == 0 ? d0 : 0;
                        }
                    }
                    pk[u] = (int)(__builtin_amdgcn_perm((unsigned)dg[1], (unsigned)dg[0], 0x0c0c0400u) |
                                  __builtin_amdgcn_perm((unsigned)dg[3], (unsigned)dg[2], 0x04000c0cu));
                    mag = __builtin_amdgcn_sad_u8((unsigned)pk[u] ^ 0x80808080u, 0x80808080u, mag);
                }
                *dst = make_int4(pk[0], pk[1], pk[2], pk[3]);
                if (mag)  // one exponent of S per unit; saturating
                    atomicAdd(&s_wsum[r], nsft >= 40u ? (1ull << 50) : ((unsigned long long)mag << nsft));
            }
        }
    }
    __syncthreads();
    if (threadIdx.x < kScatterRows && p0 + (int)threadIdx.x < a.Mp) {
        unsigned long long t = s_wsum[threadIdx.x];
        if (t > (1ull << 60)) t = 1ull << 60;
        a.rowsum[p0 + threadIdx.x] = t;
        if (t) atomicMax(a.bound, t);
    }
}

// Places the digits above digit 0 of the listed OB entries of an operand unpacked by UnpackBoth.
// The remainder floor(|v| / s) of an entry at (R, C) moves to the child of whichever of R and C was
// split first (Alg. 4 lines 7-9 / 11-14) and leaves its own digit 0 there.
//   second == 0 (A): the entry's column chain lives in the column slots of A's unpacking; A_ue then
//     repeats column r of A_u in every column slot of the second unpacking that descends from r
//     (Alg. 2 line 6 / Alg. 4 line 13), so every digit is written once per such slot.
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
    const int32_t *row_phys, *col_phys, *col_sexp;
    int Kp, s, sh;
    int8_t *out;
    unsigned long long *rowsum, *bound;
};

// Both operands in one launch: blocks [0, blocks_a) serve fa, the rest fb.
__global__ void fixup_kernel(FixupArgs fa, FixupArgs fb, int blocks_a) {
    const bool first = (int)blockIdx.x < blocks_a;
    const FixupArgs &f = first ? fa : fb;
    const int block = first ? blockIdx.x : blockIdx.x - blocks_a;
    const int nblocks = first ? blocks_a : gridDim.x - blocks_a;
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
                    const int q = f.col_phys[c];
                    f.out[(int64_t)p * f.Kp + q] = dg;
                    const unsigned nsft = (unsigned)(f.sh * f.col_sexp[q]);
                    const unsigned long long term = nsft >= 40u ? (1ull << 50) : ((unsigned long long)m << nsft);
                    unsigned long long now = atomicAdd(&f.rowsum[p], term) + term;
                    if (now > (1ull << 60)) now = 1ull << 60;
                    // the bound only grows: a plain (possibly stale) read filters most of the updates
                    if (now > __hip_atomic_load(f.bound, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
                        atomicMax(f.bound, now);
                }
            }
        }
    }
}

__global__ void reset_bound_kernel(PlanHeader *hdr) {
    if (threadIdx.x == 0 && blockIdx.x == 0) hdr->bound[0] = hdr->bound[1] = 0;
}

// canon[R][c] = phys[row_phys[R]][col_phys[c]]
__global__ void canonical_kernel(const int8_t *__restrict__ phys, int Kp, const int32_t *row_phys,
                                 const int32_t *col_phys, int nrows, int ncols, int8_t *__restrict__ canon) {
    const int R = blockIdx.x;
    if (R >= nrows) return;
    const int8_t *src = phys + (int64_t)row_phys[R] * Kp;
    for (int c = threadIdx.x; c < ncols; c += blockDim.x) canon[(int64_t)R * ncols + c] = src[col_phys[c]];
}

}  // namespace imu

using namespace imu;

extern "C" int imunpack_unpacked_bytes(const imunpack_plan_t *p, size_t *bytes_A, size_t *bytes_B,
                                       size_t *bytes_workspace) {
    if (!p || !p->valid) return IMUNPACK_EINVAL;
    if (bytes_A) *bytes_A = (size_t)p->hdr.Mp * p->hdr.Kp;
    if (bytes_B) *bytes_B = (size_t)p->hdr.Np * p->hdr.Kp;
    if (bytes_workspace) *bytes_workspace = (size_t)p->hdr.Mp * p->hdr.Np * sizeof(int64_t);
    return IMUNPACK_OK;
}

extern "C" int imunpack_unpack(imunpack_plan_t *p, const int32_t *A, int64_t lda, const int32_t *B,
                               int64_t ldb, int8_t *A_ue, int8_t *B_eu, imunpack_stream_t stream) {
    if (!p || !p->valid || !A || !B || !A_ue || !B_eu || lda < p->d || ldb < p->d) return IMUNPACK_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const PlanHeader &h = p->hdr;
    if (p->bound_pending) IMU_TRY(resolve_bound(p));  // of an earlier unpack of this plan
    // the planner leaves the bounds cleared; a repeated unpack of the same plan clears them again
    if (p->unpacked) hipLaunchKernelGGL(reset_bound_kernel, dim3(1), dim3(64), 0, st, p->d_hdr);
    FixupArgs fx[2] = {};
    int fblocks[2] = {0, 0};
    for (int op = 0; op < 2; ++op) {
        const int rowsP = op ? h.Np : h.Mp;
        if (rowsP <= 0 || h.Kp <= 0) continue;
        const RowLayout &lay = op ? p->layB : p->layA;
        const bool both = (op ? p->sB : p->sA) == IMUNPACK_BOTH;
        ScatterArgs a;
        a.M = op ? B : A; a.ld = op ? ldb : lda;
        a.prow_slot = lay.prow_slot; a.prow_src = lay.prow_src; a.prow_exp = lay.prow_exp;
        a.col_k = p->cols.colA_k;
        a.col_e = op ? p->cols.colB_e : p->cols.colA_e;
        a.unit_desc = p->cols.unit_desc;
        a.lev_shift = op ? 8 : 0;
        a.win_unit = p->cols.win_unit;
        a.Mp = rowsP; a.Kp = h.Kp; a.d = (int)p->d; a.ngroups = h.ngroups; a.s = p->s; a.sh = p->sh;
        a.out = op ? B_eu : A_ue;
        a.rowsum = op ? p->rowsumB : p->rowsumA;
        a.bound = &p->d_hdr->bound[op];
        const dim3 grid((rowsP + kScatterRows - 1) / kScatterRows);
        if (both) hipLaunchKernelGGL(scatter_kernel<false>, grid, dim3(kScatterThreads), 0, st, a);
        else hipLaunchKernelGGL(scatter_kernel<true>, grid, dim3(kScatterThreads), 0, st, a);
        const int nob = op ? h.nobB : h.nobA;
        if (both && nob > 0) {
            FixupArgs &f = fx[op];
            f.ob = op ? p->obcopyB : p->obcopyA;
            f.ob_cap = p->cap[op ? CAP_EDGEB : CAP_EDGEA];
            f.ob_count = op ? &p->d_hdr->nobB : &p->d_hdr->nobA;
            f.second = op;
            f.rows = op ? p->rowB : p->rowA;
            f.cset = op ? p->c2 : p->c1;
            f.c1_child = p->c1.child;
            f.c2_child = p->c2.child;
            f.row_phys = lay.row_phys; f.col_phys = p->cols.col_phys; f.col_sexp = p->cols.col_sexp;
            f.Kp = h.Kp; f.s = p->s; f.sh = p->sh;
            f.out = a.out; f.rowsum = a.rowsum; f.bound = a.bound;
            fblocks[op] = (nob + 255) / 256;
        }
    }
    if (fblocks[0] + fblocks[1] > 0) {  // after both scatters: the fix-up overwrites zeros they wrote
        if (!fblocks[0]) fx[0] = fx[1];  // never dereferenced, but keep the argument well-formed
        if (!fblocks[1]) fx[1] = fx[0];
        hipLaunchKernelGGL(fixup_kernel, dim3(fblocks[0] + fblocks[1]), dim3(256), 0, st, fx[0], fx[1], fblocks[0]);
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
    p->fusable = (m < (1ull << 40)) && (m * (unsigned long long)(p->s - 1) < (1ull << 31));
    p->guess_fusable = p->fusable;
    return IMUNPACK_OK;
}
}  // namespace imu

extern "C" int imunpack_plan_fusable(const imunpack_plan_t *cp) {
    if (!cp || !cp->valid || !cp->unpacked) return 0;
    Plan *p = const_cast<Plan *>(cp);
    if (resolve_bound(p) != IMUNPACK_OK) return 0;
    return p->fusable;
}

namespace imu { int ensure_canonical(Plan *p); }

extern "C" int imunpack_unpack_canonical(const imunpack_plan_t *cp, const int8_t *A_ue, const int8_t *B_eu,
                                         int8_t *A_canon, int8_t *B_canon, imunpack_stream_t stream) {
    if (!cp || !cp->valid) return IMUNPACK_EINVAL;
    Plan *p = const_cast<Plan *>(cp);
    IMU_TRY(ensure_canonical(p));  // host-side renumbering into the paper's order (synchronises)
    hipStream_t st = (hipStream_t)stream;
    const PlanHeader &h = p->hdr;
    if (A_ue && A_canon && h.n_u > 0)
        hipLaunchKernelGGL(canonical_kernel, dim3(h.n_u), dim3(256), 0, st, A_ue, h.Kp, p->canon_rowphysA,
                           p->canon_colphys, h.n_u, h.d_u, A_canon);
    if (B_eu && B_canon && h.h_u > 0)
        hipLaunchKernelGGL(canonical_kernel, dim3(h.h_u), dim3(256), 0, st, B_eu, h.Kp, p->canon_rowphysB,
                           p->canon_colphys, h.h_u, h.d_u, B_canon);
    return launch_status();
}
