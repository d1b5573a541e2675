// Shared declarations of the gfx950 IM-Unpack library (host + device).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/imunpack.h"

namespace imu {

// ---- error plumbing ---------------------------------------------------------------------------
extern thread_local int g_last_hip_error;

#define IMU_HIP(call)                                   \
    do {                                                \
        hipError_t e__ = (call);                        \
        if (e__ != hipSuccess) {                        \
            imu::g_last_hip_error = (int)e__;           \
            return IMUNPACK_EHIP;                       \
        }                                               \
    } while (0)

#define IMU_TRY(expr)                                   \
    do {                                                \
        int rc__ = (expr);                              \
        if (rc__ != IMUNPACK_OK) return rc__;           \
    } while (0)

static inline int launch_status() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return IMUNPACK_EHIP;
    }
    return IMUNPACK_OK;
}

// ---- geometry shared by planner, scatter and GEMM ----------------------------------------------
constexpr int kTile = 256;       // GEMM output tile edge in unpacked rows (both operands)
constexpr int kChunk = 64;       // physical rows the GEMM epilogue holds at a time; no source row straddles a chunk
constexpr int kKPad = 128;       // every exponent group is padded to a multiple of this many columns
constexpr int kMaxGroups = 64;   // distinct diagonal entries of S the planner supports
constexpr int kMaxRuns = 128;    // stretches of consecutive k-tiles that read consecutive blocks of the A store
constexpr uint32_t kNever = 0xFFFFFFFFu;  // split time of a row/column that is never split

// One set of growing row (or column) slots: what Pi (or S) needs per slot, plus the split
// bookkeeping that lets the scatter kernel follow an entry's digits.
struct SlotSet {
    int32_t *root;    // original row / phase-entry column this slot descends from
    int32_t *exp;     // number of splits between root and this slot (digit level along this axis)
    uint32_t *time;   // when this slot was split (order among all splits of the phase), kNever if not
    int32_t *child;   // slot created by that split, -1 if none
    unsigned long long *key;  // appended slots: order among the appended slots (batch, count desc, split slot)
    int32_t cap;
};

// Header kept on the device and mirrored to the host after planning.
struct PlanHeader {
    int32_t n_u, h_u, d1, d_u;       // n', h', columns after unpacking A, d'
    int32_t Mp, Np, Kp;              // physical (padded) sizes
    int32_t KA;                      // stored columns of A (a multiple of 128)
    int32_t ldA, ldB;                // bytes from one physical row to the next in the A store / in B_eu: the width
                                     // rounded up to an odd multiple of 256, so that the rows of a tile that are
                                     // read together spread over the memory channels
    int32_t mtiles, ntiles;
    int32_t lmaxA, lmaxB;            // largest number of digit levels of a row of A / B
    int32_t ngroups;
    int32_t grp_exp[kMaxGroups];     // exponent of s per group, descending
    int32_t grp_k0[kMaxGroups];      // first physical column
    int32_t grp_len[kMaxGroups];     // columns of the group (whole k-tiles)
    int32_t nruns;                   // k-tiles [run_kt0[i], run_kt0[i+1]) read blocks run_blk0[i], run_blk0[i]+1, ... of the A store
    int32_t run_kt0[kMaxRuns];
    int32_t run_blk0[kMaxRuns];
    int32_t run_grp[kMaxRuns];       // the group the run belongs to
    int32_t edgesA, edgesB, obcount; // OB entry lists built for UnpackBoth
    int32_t nobA, nobB;              // OB entries of A / B kept for the scatter (UnpackBoth operands)
    int32_t overflow;                // bit set: which capacity was too small
    int32_t need[10];                // size that would have been needed, per capacity
    int32_t err;                     // IMUNPACK_ERANGE conditions found on the device
    uint32_t cols_done;              // column-layout workgroups that have finished (the last one orders the units)
    int32_t extras;                  // edges that the repeated columns of B_e add to B's OB entries (UnpackBoth on B)
    int32_t reusedB;                 // the second operand's unpacking was taken over from the plan before (keep-weights mode)
    int32_t pad_[2];
    unsigned long long bound[2];     // max over rows of sum_c s^e(c) |digit| for A_ue, B_eu
};

// What a plan in keep-weights mode remembers of the plan before it, on the device: the column unpacking of
// the first operand that the second operand's unpacking was computed for, and the header fields that unpacking left.
struct KeepState {
    int32_t valid, d1, diff, same;
    int32_t h_u, d_u, nobB, edgesB, extras;
    int32_t pad_[7];
    PlanHeader saved;  // the header as that plan left it: the layout of the second operand and of the columns
};

enum CapIndex { CAP_ROWA = 0, CAP_ROWB = 1, CAP_C1 = 2, CAP_C2 = 3, CAP_EDGEA = 4, CAP_EDGEB = 5, CAP_OB = 6,
                CAP_LISTA = 7, CAP_LISTB = 8 };  // the last two: a caller's OB list was too short

// Physical-row description used by scatter and by the GEMM epilogue.
struct RowLayout {
    int32_t *prow_slot;   // [Mp]  canonical slot of physical row, -1 = padding
    int32_t *prow_src;    // [Mp]  source row, -1 = padding
    int32_t *prow_exp;    // [Mp]  digit level of the row
    int32_t *row_phys;    // [n']  physical row of canonical slot
    int32_t *src_pstart;  // [n]   first physical row of source row i
    int32_t *src_nlev;    // [n]   number of levels of source row i
    int32_t *tile_src0;   // [tiles+1] first source row of each tile
    int32_t *chunk_src0;  // [4 tiles+1] first source row of each chunk of kChunk physical rows
    int32_t *tile_flat;   // [tiles]   1 if every source row of the tile has a single level
    // weighted L1 norm  sum_c s^e(c) |digit|  per physical row, in pieces: what the fix-up pass placed
    // (cleared by the planner) and one partial sum per wave of the scatter kernel
    unsigned long long *rowsum;   // [Mp]
    unsigned long long *wavesum;  // [Mp][windows per row]
};

// Columns.  B_eu is stored in full: Kp physical columns, one GEMM k-tile per 128 of them, grouped by
// the exponent of the diagonal entry of S.  A_ue repeats column r of A_u in every column slot of the
// second unpacking that descends from r (Alg. 2 line 6 / Alg. 4 line 13); those copies are not
// stored.  The A store holds every column of A_u once, level by level (level 0 = the d original
// columns in order, level a = the columns appended by a-fold splits, ordered by original column), each
// level padded to whole blocks of 128, plus a few blocks of gathered copies for exponent groups that
// use only a small part of a level; the GEMM reads A's k-tile t from block ktile_ablk[t] of the store.
struct ColLayout {
    int32_t *pcol_slot;   // [Kp] column slot of the second unpacking in this column of B_eu, -1 = zero column
    int32_t *col_phys;    // [d'] column of B_eu of every column slot of the second unpacking
    int32_t *colB_k;      // [Kp] original column (-1 = zero column)
    int32_t *colB_e;      // [Kp] digit level along the columns of B_e
    int32_t *col_sexp;    // [Kp] exponent of the diagonal entry of S
    int4 *unitB;          // [Kp/16] per 16-column unit: x, y = lowest and highest original column (-1: nothing to
                          // read), z bit 0: 16 consecutive original columns, bit 1: one digit level for all of
                          // them, bit 2: one weight for all of them; w = that level | exponent of S << 16
    int32_t *acol_phys;   // [d'] stored column of A that every column slot of the second unpacking reads
    int32_t *apos;        // [columns of A_u] stored column of every column slot of A's unpacking
    int32_t *colA_k;      // [KA] original column (-1 = padding)
    int32_t *colA_e;      // [KA] digit level along the columns of A
    unsigned long long *colA_w;   // [KA] sum of s^e over the column slots that read this stored column (what an
                                  // entry of it weighs in the row norm behind the accumulator bound)
    int4 *unitA;          // [KA/16] as unitB (w = level only)
    unsigned long long *unitA_w;  // [KA/16] the weight of the unit's columns if they share one
    int32_t *ktile_ablk;  // [Kp/128] block of the A store that GEMM k-tile t reads
};

// ---- wave-wide reductions and scans on the vector ALU's data-parallel-primitive moves (shifts within a
// row of 16 lanes, then the last lane of a row broadcast to the following rows) instead of permutes
// through LDS.  Lanes without a source read 0, so these serve sums and maxima of non-negative values.
#if defined(__HIPCC__)
#define IMU_DPP(v, ctrl, rows, zero_fill) __builtin_amdgcn_update_dpp(0, (int)(v), (ctrl), (rows), 0xf, (zero_fill))
// Inclusive prefix sum over the 64 lanes (lane 63 holds the wave's total).
__device__ __forceinline__ int wave_inclusive_sum(int v) {
    v += IMU_DPP(v, 0x111, 0xf, true);   // row_shr:1
    v += IMU_DPP(v, 0x112, 0xf, true);   // row_shr:2
    v += IMU_DPP(v, 0x114, 0xf, true);   // row_shr:4
    v += IMU_DPP(v, 0x118, 0xf, true);   // row_shr:8
    v += IMU_DPP(v, 0x142, 0xa, false);  // row_bcast:15 into rows 1 and 3
    v += IMU_DPP(v, 0x143, 0xc, false);  // row_bcast:31 into rows 2 and 3
    return v;
}
// Sum over the wave, valid in lane 63 only.
__device__ __forceinline__ unsigned wave_sum_lane63(unsigned v) { return (unsigned)wave_inclusive_sum((int)v); }
// Largest of a non-negative value over the wave, valid in lane 63 only.
__device__ __forceinline__ int wave_max_nonneg_lane63(int v) {
    v = max(v, IMU_DPP(v, 0x111, 0xf, true));
    v = max(v, IMU_DPP(v, 0x112, 0xf, true));
    v = max(v, IMU_DPP(v, 0x114, 0xf, true));
    v = max(v, IMU_DPP(v, 0x118, 0xf, true));
    v = max(v, IMU_DPP(v, 0x142, 0xa, false));
    v = max(v, IMU_DPP(v, 0x143, 0xc, false));
    return v;
}
// The same over each half of the wave, valid in lanes 31 and 63.
__device__ __forceinline__ int half_wave_max_nonneg_last(int v) {
    v = max(v, IMU_DPP(v, 0x111, 0xf, true));
    v = max(v, IMU_DPP(v, 0x112, 0xf, true));
    v = max(v, IMU_DPP(v, 0x114, 0xf, true));
    v = max(v, IMU_DPP(v, 0x118, 0xf, true));
    v = max(v, IMU_DPP(v, 0x142, 0xa, false));
    return v;
}
// 6-bit floating-point digits in memory.  The matrix instruction takes, per lane, 32 consecutive columns of a
// row as one 192-bit string (column j of the fragment at bits 6j .. 6j+5).  A row stores its columns in
// groups of 64 (48 bytes): the first 128 bits of the group's two fragments (16 bytes each), then their
// last 64 bits (8 bytes each), so that a lane reads its fragment as one aligned 16-byte and one aligned
// 8-byte piece.  The two 8-byte pieces change places in the rows whose index has bit 4 set: the thirty-two
// rows that an 8-byte LDS read serves together then fall on different banks (rows 112 bytes apart).
// Returns the position, in 32-bit words from the start of the row, of word i (0..5) of fragment `frag`
// (0, 1) of group `grp` in physical row `row`.
__host__ __device__ __forceinline__ int fp6_dword(int row, int grp, int frag, int i) {
    return 12 * grp + (i < 4 ? 4 * frag + i : 8 + 2 * (frag ^ ((row >> 4) & 1)) + (i - 4));
}
// Lane 63's value in every lane (a scalar register).
__device__ __forceinline__ int from_lane63(int v) { return __builtin_amdgcn_readlane(v, 63); }
#endif

}  // namespace imu

// Opaque plan object.
struct imunpack_plan {
    // problem
    int64_t n, d, h;
    int b, sA, sB;
    int s, sh;
    hipStream_t stream;
    // device arena
    char *arena;
    size_t arena_bytes;
    // capacities (grow on overflow)
    int32_t cap[10];
    // views into the arena (valid after a successful imunpack_plan)
    imu::PlanHeader *d_hdr;
    imu::PlanHeader hdr;          // host mirror
    imu::PlanHeader *pin_hdr;     // pinned staging copy of the header (device-to-host copies land here)
    hipEvent_t ready;             // recorded after such a copy; the host polls it
    hipStream_t side;             // carries the copy of the accumulator bounds, so that the caller's stream
                                  // can already hold the GEMM while the host waits for them
    hipEvent_t scattered;         // recorded on the caller's stream after the scatter; `side` waits for it
    int bound_pending;            // the bounds of the last imunpack_unpack have not been read back yet
    int guess_fusable;            // whether the fused GEMM was exact for this plan object the last time
    imu::SlotSet rowA, rowB, c1, c2;
    imu::RowLayout layA, layB;
    imu::ColLayout cols;
    int32_t *statsA[4], *statsB[4];   // rowcnt, colcnt, rowmax, colmax actually used
    // greedy scratch
    unsigned long long *edges;        // two lists of edge_cap packed edges each
    int edge_cap;
    int32_t *rcnt, *ccnt;
    int32_t *extraRows;               // per row of B: how many of those extra edges it has
    int32_t *obcopyA, *obcopyB;       // OB entries of an UnpackBoth operand, kept for the scatter: [3][cap[CAP_EDGEx]]
    int32_t *ob;                      // own OB entry list [3][cap[CAP_OB]] when the caller gave none
    int32_t *tmpL, *tmpCur, *tmpPA, *tmpPB, *tmpE, *tmpK, *tmpR, *tmpOff;
    int ignore_listA, ignore_listB;   // a caller's OB list overflowed: scan the operand ourselves
    int bothA, bothB;                 // slot numbering of the set needs the export-time sort
    // canonical (paper-order) numbering, built lazily by the export / test paths
    int canon_valid;
    int32_t *canon_rowphysA, *canon_rowphysB, *canon_colphys, *canon_acolphys;   // device, indexed by canonical slot
    int32_t *tmpApos;
    int fusable;      // set by imunpack_unpack
    int unpacked;
    int valid;
    int keep_B;       // keep-weights mode: the second operand is the same from plan to plan
    int keep_valid;   // the arena holds a complete unpacking of the second operand and the snapshot it belongs to
    unsigned long long keep_sig;  // ... for the arena layout with this signature
    int32_t *snapRoot, *snapExp, *snapChild;  // the first operand's column slots at that time
    const int8_t *kept_Beu;  // the buffer the last imunpack_unpack wrote B_eu to, while it still matches the plan
    int kept_Beu_fp6;
    imu::KeepState *d_keep;
    int digits_req;   // IMUNPACK_DIGITS_*: what imunpack_plan_set_digits asked for (kept across re-planning)
    int fp6;          // in effect for the current plan: 6-bit floating-point digits (requested and b <= 4)
};

namespace imu {
using Plan = struct ::imunpack_plan;  // the C function imunpack_plan() hides the bare struct name

// Copies bytes [offset, offset + bytes) of the device header into the host mirror and waits for it.
// The wait polls an event instead of blocking in the driver: the wake-up of a blocking wait costs
// tens of microseconds during which the GPU idles between two stages of the path.
int fetch_header(Plan *p, size_t offset, size_t bytes, hipStream_t st);
// Waits for the bounds that imunpack_unpack left in flight and sets p->fusable.
int resolve_bound(Plan *p);
// Bytes from one physical row to the next of the A store (op 0) / of B_eu (op 1) in the digit format in
// effect.  6-bit digits: 96 bytes per k-tile of 128 columns, the same rule against power-of-two pitches.
inline int64_t store_pitch(const Plan *p, int op) {
    if (!p->fp6) return op ? p->hdr.ldB : p->hdr.ldA;
    const int bytes = (op ? p->hdr.Kp : p->hdr.KA) / 4 * 3;
    return bytes >= 2048 ? (((bytes + 255) / 256) | 1) * 256 : bytes;
}
}
