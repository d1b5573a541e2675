// Unpack planner: decides every row / column split of Alg. 1, 2 and 4 (dispatched as in Alg. 5,
// A first, then B on the widened B_e with S_u carried over -- Sec. 4 "Combining everything")
// without touching the operands.  What it produces per unpacked row is the single non-zero of the
// matching column of Pi (source row, exponent of s); per unpacked column the exponent of the
// diagonal entry of S and the original column it copies.
//
// UnpackRow / UnpackColumn are FIFO loops whose result has a closed form: a row (column) whose
// largest magnitude has L base-s digits yields L slots, and the appended slots come level by
// level, within a level in ascending source index.  Slots are therefore assigned by one
// exclusive prefix sum per level.
//
// UnpackBoth is a greedy over OB counts.  A row split changes no other row's count and can only
// lower column counts (and vice versa), so all rows that share the current top count can be split
// as one batch, in index order, without changing the outcome of the sequential algorithm.  The
// greedy runs on the compacted list of OB entries (a tiny fraction of the operand) in a single
// persistent workgroup.
#include "common.h"

#include <type_traits>

#include <algorithm>
#include <atomic>
#include <cstring>
#include <new>
#include <vector>

namespace imu {

constexpr int kPlanThreads = 1024;
constexpr int kPlanWaves = kPlanThreads / 64;

// ---------------------------------------------------------------------------------------------
// workgroup-wide helpers (kPlanThreads threads)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int block_max(int v /* >= 0 */, int *lds /* >= 40 ints */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    v = wave_max_nonneg_lane63(v);
    if (lane == 63) lds[wave] = v;
    __syncthreads();
    int r = lds[0];
#pragma unroll
    for (int w = 1; w < kPlanWaves; ++w) r = max(r, lds[w]);
    __syncthreads();
    return r;
}

__device__ __forceinline__ int load_agent(const int32_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// number of base-s digits of a magnitude (>= 1)
__device__ __forceinline__ int digit_levels(int m, int sh) {
    int L = 1;
    unsigned u = (unsigned)m >> sh;
    while (u) {
        ++L;
        u >>= sh;
    }
    return L;
}

__device__ __forceinline__ void flag_overflow(PlanHeader *hdr, int which, int need) {
    atomicOr(&hdr->overflow, 1 << which);
    atomicMax(&hdr->need[which], need);
}

// Calls emit(x, rank) for every x in [0, N) with flag(x), rank = base + the number of flagged x' < x;
// returns the number of flagged items.  Every wave owns one contiguous segment and ranks its items
// by ballot, so the whole selection costs two workgroup barriers.
template <class F, class E>
__device__ __forceinline__ int ordered_select(int N, int base, F flag, E emit, int *lds /* >= 40 ints */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int seg = ((N + kPlanWaves - 1) / kPlanWaves + 63) & ~63;
    const int lo = wave * seg, hi = min(N, lo + seg);
    int cnt = 0;
    for (int x0 = lo; x0 < hi; x0 += 64) {
        const int x = x0 + lane;
        const bool f = x < hi && flag(x);
        cnt += __popcll(__ballot(f));
    }
    if (lane == 0) lds[wave] = cnt;
    __syncthreads();
    int run = base, total = 0;
#pragma unroll
    for (int w = 0; w < kPlanWaves; ++w) {
        const int c = lds[w];
        if (w < wave) run += c;
        total += c;
    }
    const unsigned long long below = (1ull << lane) - 1ull;
    for (int x0 = lo; x0 < hi; x0 += 64) {
        const int x = x0 + lane;
        const bool f = x < hi && flag(x);
        const unsigned long long mask = __ballot(f);
        if (f) emit(x, run + __popcll(mask & below));
        run += __popcll(mask);
    }
    __syncthreads();
    return total;
}

// Calls emit(x, prefix) for every x in [0, N), prefix = base + sum of value(x') over x' < x; returns
// the sum of all values.
template <class V, class E>
__device__ __forceinline__ int ordered_scan(int N, int base, V value, E emit, int *lds /* >= 40 ints */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int seg = ((N + kPlanWaves - 1) / kPlanWaves + 63) & ~63;
    const int lo = wave * seg, hi = min(N, lo + seg);
    int sum = 0;
    for (int x0 = lo; x0 < hi; x0 += 64) {
        const int x = x0 + lane;
        if (x < hi) sum += value(x);
    }
    sum = wave_inclusive_sum(sum);
    if (lane == 63) lds[wave] = sum;
    __syncthreads();
    int run = base, total = 0;
#pragma unroll
    for (int w = 0; w < kPlanWaves; ++w) {
        const int c = lds[w];
        if (w < wave) run += c;
        total += c;
    }
    for (int x0 = lo; x0 < hi; x0 += 64) {
        const int x = x0 + lane;
        const int v = x < hi ? value(x) : 0;
        const int incl = wave_inclusive_sum(v);
        if (x < hi) emit(x, run + incl - v);
        run += from_lane63(incl);
    }
    __syncthreads();
    return total;
}

// ---------------------------------------------------------------------------------------------
// header / identity
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void identity_slot(const SlotSet &set, int x) {
    set.root[x] = x;
    set.exp[x] = 0;
    set.time[x] = kNever;
    set.child[x] = -1;
}

// Clears the header and makes the first na / nb / nc slots of three sets unsplit originals (a count
// of 0 skips a set).  The counts are known to the host, which has sized the sets for them.
__global__ void setup_kernel(PlanHeader *hdr, SlotSet a, int na, int32_t *count_a, SlotSet b, int nb,
                             int32_t *count_b, SlotSet c, int nc, int32_t *count_c, int32_t *zeroed, int nzeroed,
                             int32_t *zeroed2, int nzeroed2, KeepState *ks) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (ks) ks->diff = ks->same = 0;
        static_assert(sizeof(PlanHeader) % sizeof(int32_t) == 0, "header is cleared word by word");
        for (size_t i = 0; i < sizeof(PlanHeader) / sizeof(int32_t); ++i) reinterpret_cast<int32_t *>(hdr)[i] = 0;
        if (na) *count_a = na;
        if (nb) *count_b = nb;
        if (nc) *count_c = nc;
    }
    const int stride = gridDim.x * blockDim.x;
    for (int x = blockIdx.x * blockDim.x + threadIdx.x; x < na; x += stride) identity_slot(a, x);
    for (int x = blockIdx.x * blockDim.x + threadIdx.x; x < nb; x += stride) identity_slot(b, x);
    for (int x = blockIdx.x * blockDim.x + threadIdx.x; x < nc; x += stride) identity_slot(c, x);
    for (int x = blockIdx.x * blockDim.x + threadIdx.x; x < nzeroed; x += stride) zeroed[x] = 0;
    for (int x = blockIdx.x * blockDim.x + threadIdx.x; x < nzeroed2; x += stride) zeroed2[x] = 0;
}

// slots 0..N-1 become unsplit originals, N read from the device
__global__ void identity_slots_kernel(SlotSet set, const int32_t *n_dev, int32_t *count_out, PlanHeader *hdr,
                                      int which, const int32_t *skip) {
    if (hdr->overflow) return;
    if (skip && *skip) return;  // keep-weights mode: this set is taken over as it stands
    const int N = *n_dev;
    if (N > set.cap) {
        if (blockIdx.x == 0 && threadIdx.x == 0) flag_overflow(hdr, which, N);
        return;
    }
    for (int x = blockIdx.x * blockDim.x + threadIdx.x; x < N; x += gridDim.x * blockDim.x) identity_slot(set, x);
    if (count_out && blockIdx.x == 0 && threadIdx.x == 0) *count_out = N;
}

// ---------------------------------------------------------------------------------------------
// UnpackRow / UnpackColumn in closed form (Alg. 1 / Alg. 2)
// ---------------------------------------------------------------------------------------------
// Base items x = 0..N-1 with largest magnitude maxabs[via ? via[x] : x]; every level l >= 1 appends
// the items that still have a digit there, in ascending x.
__global__ __launch_bounds__(kPlanThreads) void level_major_kernel(
    SlotSet set, const int32_t *maxabs, const int32_t *via, int n_host, const int32_t *n_dev, int sh,
    int32_t *tmpL, int32_t *tmpCur, int32_t *count_out, PlanHeader *hdr, int which, const int32_t *skip) {
    __shared__ int lds[40];
    if (hdr->overflow) return;
    if (skip && *skip) return;  // keep-weights mode: this set is taken over as it stands
    const int N = n_dev ? *n_dev : n_host;
    if (N > set.cap) {
        if (threadIdx.x == 0) flag_overflow(hdr, which, N);
        return;
    }
    int lm = 1;
    for (int x = threadIdx.x; x < N; x += kPlanThreads) {
        const int L = digit_levels(maxabs[via ? via[x] : x], sh);
        tmpL[x] = L;
        tmpCur[x] = x;
        identity_slot(set, x);
        lm = max(lm, L);
    }
    const int lmax = block_max(lm, lds);
    int base = N;
    for (int l = 1; l < lmax; ++l) {
        base += ordered_select(
            N, base, [&](int x) { return tmpL[x] > l; },
            [&](int x, int slot) {
                if (slot >= set.cap) return;
                set.root[slot] = x;
                set.exp[slot] = l;
                set.time[slot] = kNever;
                set.child[slot] = -1;
                const int prev = tmpCur[x];
                set.key[slot] = ((unsigned long long)l << 48) | (unsigned)prev;
                set.child[prev] = slot;
                set.time[prev] = 0;  // split (only this axis splits in this phase, any finite time will do)
                tmpCur[x] = slot;
            },
            lds);
    }
    if (threadIdx.x == 0) {
        *count_out = base;
        if (base > set.cap) flag_overflow(hdr, which, base);
    }
}

// ---------------------------------------------------------------------------------------------
// UnpackBoth (Alg. 4): the greedy
// ---------------------------------------------------------------------------------------------
struct GreedyArgs {
    SlotSet rows, cols;
    const int32_t *cols_init;      // second operand: number of column slots to start from (columns after
                                   // unpacking A), made unsplit originals here; nullptr for the first
    const int32_t *chain_child;    // second operand: child links of the column slots of A's unpacking
    const int32_t *chain_root;     // second operand: original column of each of those slots
    const int32_t *rowcnt, *colcnt, *rowmax;  // the operand's heavy-hitter statistics
    const int32_t *ob;             // OB entries of the operand: [3][ob_cap] rows | columns | values
    int ob_cap;
    const int32_t *ob_count;
    int which_list;
    unsigned long long *edges;     // two lists of ecap packed edges
    int ecap;
    int32_t *ob_keep_count;        // header field: the number of OB entries kept for the scatter
    const int32_t *extra_rows;     // second operand: extra edges per row (repeated columns), else null
    int32_t *rcnt, *ccnt;          // live OB count per row / column slot when LDS cannot hold them
    int32_t *nr_io, *nc_io;        // slot counts (header fields)
    int32_t *ecount_out;
    PlanHeader *hdr;
    int whichR, whichC, whichE;
    int s, sh;
    const int32_t *skip;           // keep-weights mode: non-zero there = nothing to do
};

// An edge of the greedy: an OB entry's current row slot, column slot and the number of base-s digits
// it still has there (>= 2 while it is OB).  Only that number matters: a split moves floor(v / s) on.
constexpr int kEdgeSlotBits = 29;
constexpr unsigned kEdgeSlotMask = (1u << kEdgeSlotBits) - 1u;
// A packed edge is two 32-bit words, so that a pass never needs 64-bit arithmetic: the low word holds
// the row slot, the high word the column slot, and the three bits above each slot number hold the low
// and the high half of the number of digits left (2 .. 63, so a packed edge is never 0).
__device__ __forceinline__ unsigned long long pack_edge(int row, int col, int levels) {
    const unsigned lo = (unsigned)row | (((unsigned)levels & 7u) << kEdgeSlotBits);
    const unsigned hi = (unsigned)col | (((unsigned)levels >> 3) << kEdgeSlotBits);
    return (unsigned long long)lo | ((unsigned long long)hi << 32);
}

// The sequential algorithm splits, at every step, the row or column with the top OB count (rows win
// ties, then the lowest index).  Splitting a row changes no other row's count and only lowers column
// counts, so while rows are being chosen the rows come in (count descending, index ascending) order
// and every row whose count is at least the top column count at the start of the run is chosen
// before any column -- unless a split leaves OB entries in the new row (entries with three or more
// digits), whose count then competes.  Hence:
//   - if no entry has three or more digits, one batch takes all rows with count >= top column count
//     (or all columns with count > top row count);
//   - otherwise a batch takes only the slots that share the top count.
// The starting counts are the operand's scan statistics.  After UnpackA the matrix B_e repeats column
// k of B once per column slot that descends from k (Alg. 2 line 6 / Alg. 4 line 13): such a slot
// starts with the count of column k, and every OB entry (j, k) adds one to row j per extra slot
// (ob_copy_kernel finds those extra edges before this kernel starts).
// A batch is one pass over the live entries: an entry in a split slot keeps digit 0 there and moves
// floor(v / s) to the new slot (Alg. 4 lines 7-9 / 11-14); if that is In-Bound the entry is finished:
// it leaves the count of the crossing slot and the list.  The entries are packed edges (row slot,
// column slot, digits left); the first list comes from ob_copy_kernel, the survivors of every pass are
// written, compacted, to the other of two lists.  The order inside a batch only decides the numbers of the appended slots; it is recorded as
// a sort key (batch, count descending, split slot) and the appended slots are renumbered on the host
// when the plan is exported.
template <bool LDS>
__global__ __launch_bounds__(kPlanThreads) void greedy_both_kernel(GreedyArgs g) {
    extern __shared__ __attribute__((aligned(16))) int32_t lds_counts[];
    __shared__ int s_top[2], s_T[2][4];
    __shared__ int s_pick[kPlanWaves][256];  // per wave: the slots picked in one 256-slot step
    __shared__ int s_found[kPlanWaves], s_positive[kPlanWaves];
    __shared__ int lds[40];
    __shared__ int s_count;
    PlanHeader *hdr = g.hdr;
    if (hdr->overflow) return;
    if (g.skip && *g.skip) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long below = (1ull << lane) - 1ull;
    int nr = *g.nr_io, nc;
    if (g.cols_init) {
        nc = *g.cols_init;
        if (nc > g.cols.cap) {
            if (threadIdx.x == 0) flag_overflow(hdr, g.whichC, nc);
            return;
        }
        for (int x = threadIdx.x; x < nc; x += kPlanThreads) identity_slot(g.cols, x);
    } else {
        nc = *g.nc_io;
    }
    const int nob = *g.ob_count;
    if (nob > g.ob_cap) {
        if (threadIdx.x == 0) flag_overflow(hdr, g.which_list, nob);
        return;
    }
    const int rpad = (g.rows.cap + 7) & ~3, cpad = (g.cols.cap + 7) & ~3;  // int4 reads may run past the last slot
    int32_t *rc = LDS ? lds_counts : g.rcnt;
    int32_t *cc = LDS ? lds_counts + rpad : g.ccnt;
    // ---- starting counts
    int deep = 0;
    const int s2 = g.s * g.s;
    for (int x = threadIdx.x; x < rpad; x += kPlanThreads) {
        rc[x] = x < nr ? g.rowcnt[x] + (g.extra_rows ? g.extra_rows[x] : 0) : 0;
        if (x < nr && g.rowmax[x] >= s2) deep = 1;
    }
    for (int x = threadIdx.x; x < cpad; x += kPlanThreads)
        cc[x] = x < nc ? g.colcnt[g.chain_root ? g.chain_root[x] : x] : 0;
    if (threadIdx.x == 0) {
        s_count = 0;
        s_top[0] = s_top[1] = 0;
    }
    __syncthreads();
    // ---- the first edge list was written by ob_copy_kernel: one packed edge per OB entry, then the extra
    // edges of repeated columns (second operand only; the rows they touch start with that many more OB
    // entries)
    unsigned long long *list0 = g.edges, *list1 = g.edges + ((g.ecap + 1) & ~1);  // both 16-byte aligned
    if (g.chain_child && threadIdx.x == 0) s_count = hdr->extras;
    __syncthreads();
    deep = block_max(deep, lds);
    const int extras = s_count;
    const long long Etotal = (long long)nob + extras;
    if (threadIdx.x == 0) {
        *g.ecount_out = (int)min(Etotal, 2147483647ll);
        *g.ob_keep_count = nob;
    }
    if (Etotal > g.ecap) {
        if (threadIdx.x == 0) flag_overflow(hdr, g.whichE, (int)min(Etotal, 1ll << 30));
        return;
    }
    int E = (int)Etotal, cur = 0;  // live edges; they are in list `cur`
    int prev_kind = -1;            // 1: the batch before split rows, 0: columns
    const long long max_batches = 32ll * Etotal + 64;  // every batch retires >= one digit of one entry
    for (long long bid = 0;; ++bid) {
        if (bid > max_batches || bid >= 65535) {
            if (threadIdx.x == 0) atomicMin(&hdr->err, bid >= 65535 ? IMUNPACK_ERANGE : IMUNPACK_EHIP);
            return;
        }
        // Every wave owns one contiguous segment of the row slots and one of the column slots, four
        // slots per lane.  (1) top counts; the marks the previous batch left in split slots (negative
        // values) are cleared on the way -- a split slot never holds an OB entry again.
        const int segR = ((nr + kPlanWaves - 1) / kPlanWaves + 255) & ~255;
        const int segC = ((nc + kPlanWaves - 1) / kPlanWaves + 255) & ~255;
        int m0 = 0, m1 = 0;
        for (int x0 = wave * segR; x0 < min(nr, (wave + 1) * segR); x0 += 256) {
            const int x = x0 + lane * 4;
            if (x >= nr) continue;
            int4 c = *reinterpret_cast<const int4 *>(&rc[x]);
            if ((c.x | c.y | c.z | c.w) < 0) {
                c = make_int4(max(c.x, 0), max(c.y, 0), max(c.z, 0), max(c.w, 0));
                *reinterpret_cast<int4 *>(&rc[x]) = c;
            }
            m0 = max(max(m0, max(c.x, c.y)), max(c.z, c.w));
        }
        for (int x0 = wave * segC; x0 < min(nc, (wave + 1) * segC); x0 += 256) {
            const int x = x0 + lane * 4;
            if (x >= nc) continue;
            int4 c = *reinterpret_cast<const int4 *>(&cc[x]);
            if ((c.x | c.y | c.z | c.w) < 0) {
                c = make_int4(max(c.x, 0), max(c.y, 0), max(c.z, 0), max(c.w, 0));
                *reinterpret_cast<int4 *>(&cc[x]) = c;
            }
            m1 = max(max(m1, max(c.x, c.y)), max(c.z, c.w));
        }
        m0 = wave_max_nonneg_lane63(m0);
        m1 = wave_max_nonneg_lane63(m1);
        if (lane == 63) {
            atomicMax(&s_top[0], m0);
            atomicMax(&s_top[1], m1);
        }
        __syncthreads();
        const int c0 = s_top[0], c1 = s_top[1];  // cleared again in step 3, past the next barrier
        if (c0 <= 0 && c1 <= 0) break;
        const bool isrow = c0 >= c1;  // rows win ties (Alg. 4: "else if c0 >= c1")
        int32_t *cnt = isrow ? rc : cc, *other = isrow ? cc : rc;
        const SlotSet &mine = isrow ? g.rows : g.cols;
        const int N = isrow ? nr : nc;
        // (2) slots with lo <= count <= hi are split in this batch, numbered in index order
        const int hi = isrow ? c0 : c1;
        int lo = deep ? hi : (isrow ? max(c1, 1) : c0 + 1);
        // (1b) While the sequential algorithm stays on one side, the counts of that side do not change (no
        // entry has three digits) and only the top count of the other side falls, so the next batch would
        // be of the same kind with a lower bound: rows with count >= G(lo), G(lo) = top column count once
        // the rows with count >= lo are gone (columns: count >= F(lo) + 1).  Every slot down to the fixed
        // point of that recursion is split before the other side gets a turn, in (count descending, index)
        // order: one batch.  A read-only pass over the live entries evaluates G at lo, lo-1, lo-2, lo-3 at
        // once (four 8-bit counters per slot of the other side, kept in the unused upper half of that
        // side's count vector), which usually covers several steps of the recursion.
        // Tried only when the batch before was of the same kind: a side's first batch often is its only one.
        const bool again = prev_kind == (isrow ? 1 : 0);
        prev_kind = isrow ? 1 : 0;
        if (LDS && !deep && E > 0 && lo > 1 && again) {
            const int No = isrow ? nc : nr, No4 = (No + 3) & ~3;
            const int top_o = isrow ? c1 : c0;
            if (2 * No4 <= (isrow ? cpad : rpad) - 4 && top_o <= 255) {
                int32_t *tmp = other + No4;  // zero on entry (slots that do not exist yet) and on exit
                const unsigned long long *__restrict__ src = cur ? list1 : list0;
                if (threadIdx.x < 8) (&s_T[0][0])[threadIdx.x] = 0;
                __syncthreads();
                for (int round = 0; round < 256; ++round) {
                    int *T = s_T[round & 1];  // cleared above or during the round before
                    auto count_pass = [&](auto isrow_c) {
                        constexpr bool IR = decltype(isrow_c)::value;
                        constexpr int UW = 8;  // 16-byte loads (two entries each) per thread in flight
                        for (int e0 = 0; e0 < E; e0 += kPlanThreads * 2 * UW) {
                            unsigned long long ed[2 * UW];
#pragma unroll
                            for (int u = 0; u < UW; ++u) {
                                const int idx = e0 + (u * kPlanThreads + (int)threadIdx.x) * 2;
                                if (idx + 1 < E) {
                                    const ulonglong2 t = *reinterpret_cast<const ulonglong2 *>(src + idx);
                                    ed[2 * u] = t.x;
                                    ed[2 * u + 1] = t.y;
                                } else {
                                    ed[2 * u] = idx < E ? src[idx] : 0ull;
                                    ed[2 * u + 1] = 0ull;
                                }
                            }
#pragma unroll
                            for (int u = 0; u < 2 * UW; ++u) {
                                const unsigned elo = (unsigned)ed[u], ehi = (unsigned)(ed[u] >> 32);
                                const unsigned xw = IR ? elo : ehi, ow = IR ? ehi : elo;
                                const int c = cnt[xw & kEdgeSlotMask];  // slot 0's count is harmless for an absent entry ...
                                const int k = (elo | ehi) ? min(4, max(0, lo - c)) : 0;  // the entry outlives the bounds lo, .., lo - k + 1
                                if (k) atomicAdd(reinterpret_cast<unsigned *>(&tmp[ow & kEdgeSlotMask]), 0x01010101u >> (8 * (4 - k)));
                            }
                        }
                    };
                    if (isrow) count_pass(std::true_type{});
                    else count_pass(std::false_type{});
                    __syncthreads();
                    int m0 = 0, m1 = 0, m2 = 0, m3 = 0;
                    if (threadIdx.x < 4) s_T[(round & 1) ^ 1][threadIdx.x] = 0;
                    for (int x = threadIdx.x * 4; x < No4; x += kPlanThreads * 4) {  // read and clear
                        const int4 v = *reinterpret_cast<const int4 *>(&tmp[x]);
                        *reinterpret_cast<int4 *>(&tmp[x]) = make_int4(0, 0, 0, 0);
                        const unsigned w4[4] = {(unsigned)v.x, (unsigned)v.y, (unsigned)v.z, (unsigned)v.w};
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            m0 = max(m0, (int)(w4[u] & 255u));
                            m1 = max(m1, (int)((w4[u] >> 8) & 255u));
                            m2 = max(m2, (int)((w4[u] >> 16) & 255u));
                            m3 = max(m3, (int)(w4[u] >> 24));
                        }
                    }
                    m0 = wave_max_nonneg_lane63(m0);
                    m1 = wave_max_nonneg_lane63(m1);
                    m2 = wave_max_nonneg_lane63(m2);
                    m3 = wave_max_nonneg_lane63(m3);
                    if (lane == 63) {
                        atomicMax(&T[0], m0);
                        atomicMax(&T[1], m1);
                        atomicMax(&T[2], m2);
                        atomicMax(&T[3], m3);
                    }
                    __syncthreads();
                    int now = lo;
                    bool stable = false;
                    for (int j = 0; j < 4; j = lo - now) {  // T[j]: the other side's top count with the bound lo - j
                        const int t = T[j];
                        const int next = isrow ? max(t, 1) : t + 1;
                        if (next >= now) {
                            stable = true;
                            break;
                        }
                        now = next;
                        if (now <= 1) {  // nothing below: every slot that holds an entry is taken
                            stable = true;
                            break;
                        }
                    }
                    lo = now;
                    if (stable) break;
                }
                __syncthreads();  // the cleared counters and the last reads of T, before anything else touches them
            }
        }
        const int seg = isrow ? segR : segC;
        const int wlo = wave * seg, whi = min(N, wlo + seg);
        int found = 0, positive = 0;
        for (int x0 = wlo; x0 < whi; x0 += 256) {
            const int x = x0 + lane * 4;  // counts past slot N-1 (within the padding) are 0 < lo
            const int4 c = x < N ? *reinterpret_cast<const int4 *>(&cnt[x]) : make_int4(0, 0, 0, 0);
            found += __popcll(__ballot(c.x >= lo && c.x <= hi)) + __popcll(__ballot(c.y >= lo && c.y <= hi)) +
                     __popcll(__ballot(c.z >= lo && c.z <= hi)) + __popcll(__ballot(c.w >= lo && c.w <= hi));
            positive += __popcll(__ballot(c.x > 0)) + __popcll(__ballot(c.y > 0)) + __popcll(__ballot(c.z > 0)) +
                        __popcll(__ballot(c.w > 0));
        }
        if (lane == 0) {
            s_found[wave] = found;
            s_positive[wave] = positive;
        }
        __syncthreads();
        int run = 0, nb = 0, npos = 0;
#pragma unroll
        for (int w = 0; w < kPlanWaves; ++w) {
            const int c = s_found[w];
            if (w < wave) run += c;
            nb += c;
            npos += s_positive[w];
        }
        // If no entry has three or more digits and the batch takes every slot of its side that still
        // holds an OB entry, every live entry is finished by it: nothing is left to count.
        const bool finishes = !deep && nb == npos;
        if (N + nb > mine.cap || N + nb >= (1 << kEdgeSlotBits)) {
            if (threadIdx.x == 0) {
                if (N + nb >= (1 << kEdgeSlotBits)) atomicMin(&hdr->err, IMUNPACK_ERANGE);
                else flag_overflow(hdr, isrow ? g.whichR : g.whichC, 2 * (N + nb));
            }
            return;
        }
        // (3) the new slots; a split slot's count is replaced by a mark that names its new slot (only
        // the lane that owns a slot reads its count in steps 1-3).  The picked slots of a step are
        // first compacted into the wave's LDS list, so that the stores run over them densely.
        for (int x0 = wlo; x0 < whi; x0 += 256) {
            const int x = x0 + lane * 4;
            const int4 c = x < N ? *reinterpret_cast<const int4 *>(&cnt[x]) : make_int4(0, 0, 0, 0);
            const int cv[4] = {c.x, c.y, c.z, c.w};
            bool f[4];
            int before = 0, all = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                f[i] = cv[i] >= lo && cv[i] <= hi;
                const unsigned long long m = __ballot(f[i]);
                before += __popcll(m & below);
                all += __popcll(m);
            }
            if (all == 0) continue;  // uniform per wave
            int pos = before;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (f[i]) {
                    s_pick[wave][pos] = (min(cv[i], 0xFFFFFF) << 8) | (lane * 4 + i);
                    cnt[x + i] = -(run + pos + 1);
                    ++pos;
                }
            }
            for (int j = lane; j < all; j += 64) {
                const int pk = s_pick[wave][j];
                const int X = x0 + (pk & 0xFF), newX = N + run + j;
                const int root = mine.root[X], ex = mine.exp[X];
                mine.time[X] = (uint32_t)bid;
                mine.child[X] = newX;
                mine.root[newX] = root;
                mine.exp[newX] = ex + 1;
                mine.time[newX] = kNever;
                mine.child[newX] = -1;
                mine.key[newX] = ((unsigned long long)bid << 48) |
                                 ((unsigned long long)(0xFFFFFF - (pk >> 8)) << 24) | (unsigned)X;
            }
            run += all;
        }
        if (threadIdx.x == 0) {
            s_count = 0;
            s_top[0] = s_top[1] = 0;
        }
        __syncthreads();
        if (finishes) {
            for (int x = threadIdx.x; x < rpad; x += kPlanThreads) rc[x] = 0;
            for (int x = threadIdx.x; x < cpad; x += kPlanThreads) cc[x] = 0;
            if (isrow) nr += nb; else nc += nb;
            break;
        }
        // (4) the pass.  The survivors of U entries per lane are appended with one counter update per wave.
        unsigned long long *dst = cur ? list0 : list1;
        // One CU's vector ALU bounds this pass, so it is written for few instructions: the side of the batch
        // and whether entries can move on (three or more digits) are compile-time cases, the common case
        // (two digits: an entry of a split slot is simply finished) has one predicated LDS update per entry.
        auto process = [&](auto &e, auto isrow_c, auto deep_c) {  // e[u]: packed edge, 0 if absent
            constexpr bool IR = decltype(isrow_c)::value, DP = decltype(deep_c)::value;
            constexpr int U = sizeof(e) / sizeof(unsigned long long);
            unsigned xw[U], ow[U];  // the word that names the slot on the batch's side, and the other one
            int c[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {  // marks do not change during a pass; slot 0's count is harmless for absent edges
                const unsigned lo = (unsigned)e[u], hi = (unsigned)(e[u] >> 32);
                xw[u] = IR ? lo : hi;
                ow[u] = IR ? hi : lo;
                c[u] = cnt[xw[u] & kEdgeSlotMask];
            }
            int off[U], all = 0;  // survivors are packed edge by edge: the lanes of a store write side by side
#pragma unroll
            for (int u = 0; u < U; ++u) {
                bool live = (xw[u] | ow[u]) != 0u;
                const bool split = live && c[u] < 0 && ~c[u] < nb;  // the mark -(k + 1) names new slot N + k
                if constexpr (DP) {
                    if (split) {
                        const unsigned lo = IR ? xw[u] : ow[u], hi = IR ? ow[u] : xw[u];
                        const unsigned levels = (lo >> kEdgeSlotBits) | ((hi >> kEdgeSlotBits) << 3);
                        if (levels > 2u) {  // still OB in the new slot: move on, one digit fewer
                            const unsigned newX = (unsigned)(N + ~c[u]), lev = levels - 1u;
                            atomicAdd(&cnt[newX], 1);
                            const unsigned r = IR ? newX : (lo & kEdgeSlotMask), q = IR ? (hi & kEdgeSlotMask) : newX;
                            e[u] = pack_edge((int)r, (int)q, (int)lev);
                        } else {
                            atomicSub(&other[ow[u] & kEdgeSlotMask], 1);
                            live = false;
                        }
                    }
                } else {
                    if (split) atomicSub(&other[ow[u] & kEdgeSlotMask], 1);
                    live = live && !split;
                }
                const unsigned long long m = __ballot(live);
                const int before = (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
                off[u] = live ? all + before : -1;
                all += __popcll(m);
            }
            if (!all) return;
            int base = 0;
            if (lane == 0) base = atomicAdd(&s_count, all);
            base = __builtin_amdgcn_readfirstlane(base);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (off[u] >= 0) dst[base + off[u]] = e[u];
        };
        auto run_pass = [&](auto isrow_c, auto deep_c) {  // the list of packed edges, two per load
            constexpr int U2 = 8;
            const unsigned long long *__restrict__ src = cur ? list1 : list0;
            auto fetch = [&](int e0, unsigned long long (&fe)[U2]) {
#pragma unroll
                for (int u = 0; u < U2; u += 2) {
                    const int idx = e0 + (u * kPlanThreads + (int)threadIdx.x * 2);
                    if (idx + 1 < E) {
                        const ulonglong2 t = *reinterpret_cast<const ulonglong2 *>(src + idx);
                        fe[u] = t.x;
                        fe[u + 1] = t.y;
                    } else {
                        fe[u] = idx < E ? src[idx] : 0ull;
                        fe[u + 1] = 0ull;
                    }
                }
            };
            unsigned long long ed[U2];
            fetch(0, ed);
            for (int e0 = 0; e0 < E; e0 += kPlanThreads * U2) {
                unsigned long long ed2[U2];
                fetch(e0 + kPlanThreads * U2, ed2);
                process(ed, isrow_c, deep_c);
#pragma unroll
                for (int u = 0; u < U2; ++u) ed[u] = ed2[u];
            }
        };
        if (deep) {
            if (isrow) run_pass(std::true_type{}, std::true_type{});
            else run_pass(std::false_type{}, std::true_type{});
        } else {
            if (isrow) run_pass(std::true_type{}, std::false_type{});
            else run_pass(std::false_type{}, std::false_type{});
        }
        __syncthreads();
        E = s_count;
        cur ^= 1;
        if (isrow) nr += nb; else nc += nb;
    }
    if (threadIdx.x == 0) {
        *g.nr_io = nr;
        *g.nc_io = nc;
    }
}

// ---------------------------------------------------------------------------------------------
// physical layouts
// ---------------------------------------------------------------------------------------------
// Rows: source-major (all digit levels of a source row adjacent, level ascending), and no source
// row straddles a chunk of `chunk` physical rows: kChunk for A (four chunks per GEMM tile), so that Pi_A
// can be applied on the 64 rows the tile's epilogue holds in LDS at a time; kTile for B, whose levels
// are folded along the columns of a tile.  Source row i with unpadded start P_i
// goes to chunk floor(P_i / (kChunk - (Lmax-1))): a closed form, and the rows of a chunk never exceed
// kChunk.
__device__ void rows_layout(const SlotSet &rows, int nbase, const int32_t *count_dev, const RowLayout &lay,
                            int cap_phys, int cap_tiles, int32_t *tmpP_global, PlanHeader *hdr, int operand, int chunk,
                            int *lds, int32_t *fast /* 2 * nbase ints of LDS, or nullptr */) {
    // the level counts and their running sums are scanned and searched over and over: in LDS when they fit
    int32_t *nlev = fast ? fast : lay.src_nlev;
    int32_t *tmpP = fast ? fast + nbase : tmpP_global;
    int lm = 1;
    constexpr int V = 4;  // source rows per thread and step: their chains are walked side by side
    for (int i0 = threadIdx.x; i0 < nbase; i0 += kPlanThreads * V) {
        int R[V], L[V];
#pragma unroll
        for (int u = 0; u < V; ++u) {
            const int i = i0 + u * kPlanThreads;
            R[u] = i < nbase ? rows.child[i] : -1;
            L[u] = 1;
        }
        for (int hop = 0; hop < 64; ++hop) {
            bool more = false;
#pragma unroll
            for (int u = 0; u < V; ++u) {
                if (R[u] >= 0) {
                    ++L[u];
                    R[u] = rows.child[R[u]];
                    more = true;
                }
            }
            if (!more) break;
        }
#pragma unroll
        for (int u = 0; u < V; ++u) {
            const int i = i0 + u * kPlanThreads;
            if (i < nbase) {
                nlev[i] = L[u];
                if (fast) lay.src_nlev[i] = L[u];  // the GEMM epilogue reads it from memory
                lm = max(lm, L[u]);
            }
        }
    }
    const int lmax = block_max(lm, lds);
    const int base = ordered_scan(
        nbase, 0, [&](int x) { return nlev[x]; }, [&](int x, int pre) { tmpP[x] = pre; }, lds);
    // chunks of `chunk` physical rows (a divisor of kTile); source row i goes to chunk floor(P_i / Cp)
    const int Cp = chunk - (lmax - 1);
    if (Cp < 1) {
        if (threadIdx.x == 0) atomicMin(&hdr->err, IMUNPACK_ERANGE);
        return;
    }
    const int nchunks = nbase > 0 ? tmpP[nbase - 1] / Cp + 1 : 0;
    const int kPerTile = kTile / chunk;
    const int ntiles = (nchunks + kPerTile - 1) / kPerTile;
    const int Mp = ntiles * kTile;
    if (Mp > cap_phys || ntiles + 1 > cap_tiles || base != *count_dev) {
        if (threadIdx.x == 0) {
            if (base != *count_dev) atomicMin(&hdr->err, IMUNPACK_EHIP);  // inconsistent plan: internal error
            else flag_overflow(hdr, operand ? CAP_ROWB : CAP_ROWA, 2 * base);
        }
        return;
    }
    for (int ch = threadIdx.x; ch <= ntiles * kPerTile; ch += kPlanThreads) {
        // first i with P_i >= ch * Cp
        int lo = 0, hi = nbase;
        const int want = ch * Cp;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (tmpP[mid] >= want) hi = mid; else lo = mid + 1;
        }
        lay.chunk_src0[ch] = lo;
        if (ch % kPerTile == 0) lay.tile_src0[ch / kPerTile] = lo;
    }
    __syncthreads();
    for (int t = threadIdx.x; t < ntiles; t += kPlanThreads) {
        const int a = lay.tile_src0[t], e = lay.tile_src0[t + 1];
        const int slots = (e < nbase ? tmpP[e] : base) - tmpP[a];
        lay.tile_flat[t] = (slots == e - a) ? 1 : 0;
    }
    for (int p = threadIdx.x; p < Mp; p += kPlanThreads) {
        lay.prow_slot[p] = -1;
        lay.prow_src[p] = -1;
        lay.prow_exp[p] = 0;
        lay.rowsum[p] = 0;
    }
    __syncthreads();
    for (int i0 = threadIdx.x; i0 < nbase; i0 += kPlanThreads * V) {
        int R[V], pst[V], L[V];
#pragma unroll
        for (int u = 0; u < V; ++u) {
            const int i = i0 + u * kPlanThreads;
            R[u] = -1;
            pst[u] = 0;
            L[u] = 0;
            if (i < nbase) {
                const int P = tmpP[i], ch = P / Cp;
                pst[u] = ch * chunk + (P - tmpP[lay.chunk_src0[ch]]);
                L[u] = nlev[i];
                R[u] = i;
                lay.src_pstart[i] = pst[u];
            }
        }
        for (int l = 0; l < 64; ++l) {
            bool more = false;
#pragma unroll
            for (int u = 0; u < V; ++u) {
                if (R[u] >= 0 && l < L[u]) {
                    const int Rc = R[u];
                    R[u] = rows.child[Rc];
                    lay.prow_slot[pst[u] + l] = Rc;
                    lay.prow_src[pst[u] + l] = i0 + u * kPlanThreads;
                    lay.prow_exp[pst[u] + l] = l;
                    lay.row_phys[Rc] = pst[u] + l;
                    more = true;
                }
            }
            if (!more) break;
        }
    }
    if (threadIdx.x == 0) {
        if (operand == 0) { hdr->Mp = Mp; hdr->mtiles = ntiles; hdr->lmaxA = lmax; }
        else { hdr->Np = Mp; hdr->ntiles = ntiles; hdr->lmaxB = lmax; }
    }
}

// Columns.  B_eu is laid out group by group (Alg. 3 runs one GEMM per distinct diagonal entry of S),
// highest exponent first, in whole k-tiles of kKPad columns.  A column slot c of the second unpacking
// descends from slot r = c2.root[c] of the first, which descends from original column k = c1.root[r];
// it holds digit level eB = c2.exp[c] of column r of B_e, its exponent is e = eA + eB with
// eA = c1.exp[r], and the column of A_ue beside it is a copy of column r of A_u.
// The A store holds A_u once: level a (the slots with eA = a) in ascending original column, padded to
// whole k-tiles; level 0 is the d original columns in place.  Inside group e the slots with eA = a
// form a subset of level a.  If that subset is (nearly) all of the level, the group walks the level's
// stored k-tiles as they are and B_eu gets a zero column where the level has a column the group has
// not ("shared": nothing of A is copied); otherwise the subset's columns are gathered, ordered by
// (original column, eA), into k-tiles of their own at the end of the group, and the columns of A they
// need are stored once more in extra blocks behind the levels ("gathered").
constexpr int kColBlocks = 8;    // workgroups that share the column layout, one exponent group at a time each
constexpr int kMaxLevelsA = 16;  // digit levels along the columns of A that the layout supports

__device__ __forceinline__ unsigned long long weight_of(int e, int sh) {  // s^e, saturating at 2^44
    const int bits = e * sh;
    return bits >= 44 ? (1ull << 44) : (1ull << bits);
}

__device__ void cols_layout(const SlotSet &c1, const SlotSet &c2, const ColLayout &cols, int d, int cap_phys,
                            int s, int sh, int32_t *tmpE, int32_t *tmpK, int32_t *tmpR, int32_t *tmpOffAll,
                            PlanHeader *hdr, int *lds, int part) {
    __shared__ int hist2[kMaxGroups * kMaxLevelsA];          // column slots per (exponent e, level a of A)
    __shared__ int cntA[kMaxLevelsA], lvlbase[kMaxLevelsA + 1];  // columns per level of A; first stored column
    __shared__ int kbase[kMaxGroups * kMaxLevelsA];          // first column of B_eu of a shared (e, a), -1: gathered
    __shared__ int s_gk0[kMaxGroups], s_gext[kMaxGroups], s_cbase[kMaxGroups], s_xbase[kMaxGroups], s_ccount[kMaxGroups];
    __shared__ int s_kp, s_ka, s_ka_levels, s_bad, s_la;
    const int D = hdr->d_u, D1 = hdr->d1;
    int32_t *tmpOff = tmpOffAll + (size_t)part * (d + 1);
    for (int t = threadIdx.x; t < kMaxGroups * kMaxLevelsA; t += kPlanThreads) hist2[t] = 0;
    if (threadIdx.x < kMaxLevelsA) cntA[threadIdx.x] = 0;
    if (threadIdx.x == 0) s_bad = 0;
    __syncthreads();
    // every part computes the same per-slot values and the same tables (the stores of the parts
    // coincide); a part then lays out the groups part, part + kColBlocks, ...
    constexpr int V = 8;  // slots per thread and step, loaded side by side
    // ---- levels of A
    for (int r0 = threadIdx.x; r0 < D1; r0 += kPlanThreads * V) {
        int a[V];
#pragma unroll
        for (int u = 0; u < V; ++u) a[u] = r0 + u * kPlanThreads < D1 ? c1.exp[r0 + u * kPlanThreads] : -1;
#pragma unroll
        for (int u = 0; u < V; ++u) {
            if (a[u] < 0) continue;
            if (a[u] < kMaxLevelsA) atomicAdd(&cntA[a[u]], 1);
            else s_bad = 1;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0, la = 1;
        for (int a = 0; a < kMaxLevelsA; ++a) {
            lvlbase[a] = run;
            run += (cntA[a] + kKPad - 1) / kKPad * kKPad;
            if (cntA[a]) la = a + 1;
        }
        lvlbase[kMaxLevelsA] = run;
        s_ka_levels = run;
        s_la = la;
    }
    __syncthreads();
    const int la = s_la;
    // ---- stored column of every column slot of A's unpacking: level 0 in place, level a >= 1 by rank
    // among the original columns whose chain reaches that level
    for (int k = threadIdx.x; k < d; k += kPlanThreads) cols.apos[k] = k;
    for (int a = 1; a < la; ++a) {
        auto slot_at = [&](int k) {
            int r = k;
            for (int i = 0; i < a && r >= 0; ++i) r = c1.child[r];
            return r;
        };
        ordered_select(
            d, lvlbase[a], [&](int k) { return slot_at(k) >= 0; },
            [&](int k, int pos) { cols.apos[slot_at(k)] = pos; }, lds);
    }
    // ---- per column slot of the second unpacking: exponent, levels, original column
    for (int c0 = threadIdx.x; c0 < D; c0 += kPlanThreads * V) {
        int r[V], eb[V], ea[V], k[V];
#pragma unroll
        for (int u = 0; u < V; ++u) {
            const int c = c0 + u * kPlanThreads;
            r[u] = c < D ? c2.root[c] : 0;
            eb[u] = c < D ? c2.exp[c] : 0;
        }
#pragma unroll
        for (int u = 0; u < V; ++u) {
            ea[u] = c1.exp[r[u]];
            k[u] = c1.root[r[u]];
        }
#pragma unroll
        for (int u = 0; u < V; ++u) {
            const int c = c0 + u * kPlanThreads;
            if (c >= D) continue;
            const int e = ea[u] + eb[u];
            tmpE[c] = e | (ea[u] << 8) | (eb[u] << 16);
            tmpK[c] = k[u];
            tmpR[c] = r[u];
            if (e < kMaxGroups && ea[u] < kMaxLevelsA && eb[u] < 256) {
                atomicAdd(&hist2[e * kMaxLevelsA + ea[u]], 1);
            } else {
                atomicMin(&hdr->err, IMUNPACK_ERANGE);
                s_bad = 1;
            }
        }
    }
    __syncthreads();
    // ---- the k-tiles of every group: lane e of the first wave takes exponent e
    if (threadIdx.x < 64) {
        const int e = threadIdx.x;
        int tiles_sh = 0, ccount = 0, members = 0;
        for (int a = 0; a < kMaxLevelsA; ++a) {
            const int m = hist2[e * kMaxLevelsA + a];
            members += m;
            const bool shared = m > 0 && (long long)m * 8 >= (long long)cntA[a] * 7;
            kbase[e * kMaxLevelsA + a] = shared ? tiles_sh * kKPad : -1;  // relative to the group's start for now
            if (shared) tiles_sh += (cntA[a] + kKPad - 1) / kKPad;
            else ccount += m;
        }
        const int tiles_c = (ccount + kKPad - 1) / kKPad;
        const int tiles = tiles_sh + tiles_c;
        int nrun = tiles_c > 0 ? 1 : 0;  // stretches of k-tiles that walk consecutive blocks of the A store
        for (int a = 0; a < kMaxLevelsA; ++a)
            if (kbase[e * kMaxLevelsA + a] >= 0) ++nrun;
        // groups come highest exponent first: sums over the lanes above this one
        int above = tiles, above_c = tiles_c, above_n = members > 0 ? 1 : 0, above_r = nrun;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int t0 = __shfl_down(above, off, 64), t1 = __shfl_down(above_c, off, 64), t2 = __shfl_down(above_n, off, 64),
                      t3 = __shfl_down(above_r, off, 64);
            if (e + off < 64) { above += t0; above_c += t1; above_n += t2; above_r += t3; }
        }
        const int k0 = (above - tiles) * kKPad, xb = above_c - tiles_c, g = above_n - (members > 0 ? 1 : 0);
        if (part == 0) {
            int ri = above_r - nrun;
            for (int a = 0; a < kMaxLevelsA; ++a) {
                const int kb = kbase[e * kMaxLevelsA + a];
                if (kb < 0) continue;
                if (ri < kMaxRuns) {
                    hdr->run_kt0[ri] = (k0 + kb) / kKPad;
                    hdr->run_blk0[ri] = lvlbase[a] / kKPad;
                    hdr->run_grp[ri] = g;
                }
                ++ri;
            }
            if (tiles_c > 0 && ri < kMaxRuns) {
                hdr->run_kt0[ri] = k0 / kKPad + tiles_sh;
                hdr->run_blk0[ri] = s_ka_levels / kKPad + xb;
                hdr->run_grp[ri] = g;
            }
            const int total_r = __shfl(above_r, 0, 64);
            if (e == 0) {
                hdr->nruns = total_r;
                if (total_r > kMaxRuns) atomicMin(&hdr->err, IMUNPACK_ERANGE);
            }
        }
        for (int a = 0; a < kMaxLevelsA; ++a)
            if (kbase[e * kMaxLevelsA + a] >= 0) kbase[e * kMaxLevelsA + a] += k0;
        s_cbase[e] = k0 + tiles_sh * kKPad;
        s_xbase[e] = xb;
        s_ccount[e] = ccount;
        s_gk0[e] = k0;
        s_gext[e] = tiles * kKPad;
        const int total_tiles = __shfl(above, 0, 64), total_c = __shfl(above_c, 0, 64), ngroups = __shfl(above_n, 0, 64);
        if (e == 0) {
            s_kp = total_tiles * kKPad;
            s_ka = s_ka_levels + total_c * kKPad;
        }
        if (members > 0) {
            const long long lim = 2147483647ll / ((long long)(s - 1) * (s - 1));
            if (e * sh > 62 || tiles * kKPad > lim) atomicMin(&hdr->err, IMUNPACK_ERANGE);
            if (part == 0) {
                hdr->grp_exp[g] = e;
                hdr->grp_k0[g] = k0;
                hdr->grp_len[g] = tiles * kKPad;
            }
        }
        if (part == 0 && e == 0) {
            hdr->ngroups = ngroups;
            hdr->Kp = total_tiles * kKPad;
            hdr->KA = s_ka_levels + total_c * kKPad;
            // row pitches: wide rows get an odd multiple of 256 bytes (power-of-two strides put the rows
            // of a tile, which are read together, on the same few memory channels)
            const int wa = s_ka_levels + total_c * kKPad, wb = total_tiles * kKPad;
            hdr->ldA = wa >= 2048 ? (((wa + 255) / 256) | 1) * 256 : wa;
            hdr->ldB = wb >= 2048 ? (((wb + 255) / 256) | 1) * 256 : wb;
            if (total_tiles * kKPad > cap_phys) flag_overflow(hdr, CAP_C2, 2 * D);
        }
    }
    __syncthreads();
    const int Kp = s_kp, KA = s_ka, ka_levels = s_ka_levels;
    if (Kp > cap_phys || s_bad) return;
    // ---- the stored levels of A (first part)
    if (part == 0) {
        for (int q = threadIdx.x; q < ka_levels; q += kPlanThreads) {
            cols.colA_k[q] = -1;
            cols.colA_e[q] = 0;
        }
        __syncthreads();
        for (int r = threadIdx.x; r < D1; r += kPlanThreads) {
            const int q = cols.apos[r];
            cols.colA_k[q] = c1.root[r];
            cols.colA_e[q] = c1.exp[r];
        }
    }
    for (int e = kMaxGroups - 1 - part; e >= 0; e -= kColBlocks) {  // any fixed assignment of groups to parts will do
        const int q0 = s_gk0[e], q1 = q0 + s_gext[e];
        if (q1 == q0) continue;  // uniform
        for (int q = q0 + threadIdx.x; q < q1; q += kPlanThreads) {
            cols.pcol_slot[q] = -1;
            cols.colB_k[q] = -1;
            cols.colB_e[q] = 0;
            cols.col_sexp[q] = e;
        }
        // k-tile table: shared levels walk their stored blocks, gathered k-tiles get blocks of their own
        for (int a = 0; a < kMaxLevelsA; ++a) {
            const int kb = kbase[e * kMaxLevelsA + a];
            if (kb < 0) continue;
            const int nt = (cntA[a] + kKPad - 1) / kKPad;
            for (int j = threadIdx.x; j < nt; j += kPlanThreads) cols.ktile_ablk[kb / kKPad + j] = lvlbase[a] / kKPad + j;
        }
        const int cbase = s_cbase[e], ccount = s_ccount[e], xcol0 = ka_levels + s_xbase[e] * kKPad;
        const int ctiles = (ccount + kKPad - 1) / kKPad;
        for (int j = threadIdx.x; j < ctiles; j += kPlanThreads) cols.ktile_ablk[cbase / kKPad + j] = xcol0 / kKPad + j;
        for (int q = threadIdx.x; q < ctiles * kKPad; q += kPlanThreads) {
            cols.colA_k[xcol0 + q] = -1;
            cols.colA_e[xcol0 + q] = 0;
            cols.colA_w[xcol0 + q] = 0;
        }
        if (ccount > 0)
            for (int k = threadIdx.x; k < d; k += kPlanThreads) tmpOff[k] = 0;
        __syncthreads();
        const unsigned long long w = weight_of(e, sh);
        // shared members go where their column of A is stored; gathered ones are counted per original column
        for (int c0 = threadIdx.x; c0 < D; c0 += kPlanThreads * V) {
            int pe[V], k[V], rr[V];
#pragma unroll
            for (int u = 0; u < V; ++u) {
                const int c = c0 + u * kPlanThreads;
                pe[u] = c < D ? tmpE[c] : -1;
                k[u] = c < D ? tmpK[c] : 0;
                rr[u] = c < D ? tmpR[c] : 0;
            }
#pragma unroll
            for (int u = 0; u < V; ++u) {
                if (pe[u] < 0 || (pe[u] & 0xFF) != e) continue;
                const int a = (pe[u] >> 8) & 0xFF, kb = kbase[e * kMaxLevelsA + a];
                if (kb < 0) {
                    atomicAdd(&tmpOff[k[u]], 1);
                    continue;
                }
                const int c = c0 + u * kPlanThreads, qa = cols.apos[rr[u]], q = kb + (qa - lvlbase[a]);
                cols.pcol_slot[q] = c;
                cols.colB_k[q] = k[u];
                cols.colB_e[q] = (pe[u] >> 16) & 0xFF;
                cols.col_phys[c] = q;
                cols.acol_phys[c] = qa;
                atomicAdd(&cols.colA_w[qa], w);
            }
        }
        if (ccount > 0) {  // uniform
            __syncthreads();
            ordered_scan(
                d, cbase, [&](int k) { return tmpOff[k]; }, [&](int k, int pre) { tmpOff[k] = pre; }, lds);
            for (int c0 = threadIdx.x; c0 < D; c0 += kPlanThreads * V) {
                int pe[V], k[V], q[V];
#pragma unroll
                for (int u = 0; u < V; ++u) {
                    const int c = c0 + u * kPlanThreads;
                    pe[u] = c < D ? tmpE[c] : -1;
                    k[u] = c < D ? tmpK[c] : 0;
                }
#pragma unroll
                for (int u = 0; u < V; ++u) {
                    if (pe[u] < 0 || (pe[u] & 0xFF) != e || kbase[e * kMaxLevelsA + ((pe[u] >> 8) & 0xFF)] >= 0) pe[u] = -1;
                    q[u] = pe[u] >= 0 ? atomicAdd(&tmpOff[k[u]], 1) : 0;
                }
#pragma unroll
                for (int u = 0; u < V; ++u) {
                    if (pe[u] < 0) continue;
                    cols.pcol_slot[q[u]] = c0 + u * kPlanThreads;
                    cols.colB_k[q[u]] = k[u];
                    cols.colB_e[q[u]] = (pe[u] >> 16) & 0xFF;
                    cols.colA_e[xcol0 + (q[u] - cbase)] = (pe[u] >> 8) & 0xFF;
                }
            }
            __syncthreads();
            // gathered columns of one group that copy the same original column: order them by their level along A
            for (int k = threadIdx.x; k < d; k += kPlanThreads) {
                const int end = tmpOff[k], beg = k ? tmpOff[k - 1] : cbase;
                for (int i = beg + 1; i < end; ++i) {
                    const int slot = cols.pcol_slot[i], ea = cols.colA_e[xcol0 + (i - cbase)], eb = cols.colB_e[i];
                    int j = i - 1;
                    while (j >= beg && cols.colA_e[xcol0 + (j - cbase)] > ea) {
                        cols.pcol_slot[j + 1] = cols.pcol_slot[j];
                        cols.colA_e[xcol0 + (j + 1 - cbase)] = cols.colA_e[xcol0 + (j - cbase)];
                        cols.colB_e[j + 1] = cols.colB_e[j];
                        --j;
                    }
                    cols.pcol_slot[j + 1] = slot;
                    cols.colA_e[xcol0 + (j + 1 - cbase)] = ea;
                    cols.colB_e[j + 1] = eb;
                }
            }
            __syncthreads();
            for (int q = cbase + threadIdx.x; q < cbase + ccount; q += kPlanThreads) {
                const int c = cols.pcol_slot[q], qa = xcol0 + (q - cbase);
                cols.col_phys[c] = q;
                cols.acol_phys[c] = qa;
                cols.colA_k[qa] = cols.colB_k[q];
                cols.colA_w[qa] = w;
            }
        }
        __syncthreads();
        // per 16-column unit of B_eu: what the scatter kernel needs to pick its path without the per-column arrays
        for (int u = q0 / 16 + threadIdx.x; u < q1 / 16; u += kPlanThreads) {
            const int qq = 16 * u;
            int kk[16], ee[16];  // all sixteen columns' words at once: one round trip instead of sixteen
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int4 a = reinterpret_cast<const int4 *>(cols.colB_k + qq)[v], b = reinterpret_cast<const int4 *>(cols.colB_e + qq)[v];
                kk[4 * v] = a.x; kk[4 * v + 1] = a.y; kk[4 * v + 2] = a.z; kk[4 * v + 3] = a.w;
                ee[4 * v] = b.x; ee[4 * v + 1] = b.y; ee[4 * v + 2] = b.z; ee[4 * v + 3] = b.w;
            }
            const int k0 = kk[0];
            int kmin = 0x7fffffff, kmax = -1, efirst = -1;
            bool run = k0 >= 0, uniform = true;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int k = kk[j];
                run = run && k == k0 + j;
                if (k < 0) continue;
                kmin = min(kmin, k);
                kmax = max(kmax, k);
                const int eb = ee[j];
                if (efirst < 0) efirst = eb;
                else uniform = uniform && eb == efirst;  // one level for all real columns
            }
            int4 ud;
            ud.x = kmax < 0 ? -1 : kmin;
            ud.y = kmax;
            ud.z = (run ? 1 : 0) | (uniform ? 2 : 0) | 4;
            ud.w = (max(efirst, 0) & 0xFF) | ((e & 0xFF) << 16);
            cols.unitB[u] = ud;
        }
        __syncthreads();
    }
    // The workgroup that finishes last describes the units of the A store: every part has added its
    // weights by then.
    __shared__ int s_last;
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) s_last = atomicAdd(&hdr->cols_done, 1u) == (unsigned)(kColBlocks - 1);
    __syncthreads();
    if (!s_last) return;
    __threadfence();  // what the other workgroups wrote before their increment is visible past this fence
    for (int u = threadIdx.x; u < KA / 16; u += kPlanThreads) {
        const int qq = 16 * u;
        int kmin = 0x7fffffff, kmax = -1, efirst = -1, kfirst = -1, jfirst = 0;
        unsigned long long wfirst = 0;
        bool run = true, uniform = true, onew = true;
        int kk[16], ee[16];  // all sixteen columns' words at once (the fence above has dropped stale cached lines)
        unsigned long long ww[16];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int4 a = reinterpret_cast<const int4 *>(cols.colA_k + qq)[v], b = reinterpret_cast<const int4 *>(cols.colA_e + qq)[v];
            kk[4 * v] = a.x; kk[4 * v + 1] = a.y; kk[4 * v + 2] = a.z; kk[4 * v + 3] = a.w;
            ee[4 * v] = b.x; ee[4 * v + 1] = b.y; ee[4 * v + 2] = b.z; ee[4 * v + 3] = b.w;
        }
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            const ulonglong2 t = reinterpret_cast<const ulonglong2 *>(cols.colA_w + qq)[v];
            ww[2 * v] = t.x;
            ww[2 * v + 1] = t.y;
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int k = kk[j];
            if (k < 0) {
                run = false;
                continue;
            }
            const int ea = ee[j];
            const unsigned long long w = ww[j];
            if (efirst < 0) { efirst = ea; kfirst = k; jfirst = j; wfirst = w; }
            run = run && k == kfirst + (j - jfirst) && jfirst == 0;
            uniform = uniform && ea == efirst;
            onew = onew && w == wfirst;
            kmin = min(kmin, k);
            kmax = max(kmax, k);
        }
        int4 ud;
        ud.x = kmax < 0 ? -1 : kmin;
        ud.y = kmax;
        ud.z = (run && kmax >= 0 ? 1 : 0) | (uniform ? 2 : 0) | (onew ? 4 : 0);
        ud.w = max(efirst, 0) & 0xFF;
        cols.unitA[u] = ud;
        cols.unitA_w[u] = wfirst < (1ull << 44) ? wfirst : (1ull << 44);
    }
}

// One workgroup for the rows of A, one for the rows of B, kColBlocks for the columns.
__global__ __launch_bounds__(kPlanThreads) void layouts_kernel(
    SlotSet rowA, int n, RowLayout layA, int cap_physA, int32_t *tmpPA, SlotSet rowB, int h, RowLayout layB,
    int cap_physB, int32_t *tmpPB, SlotSet c1, SlotSet c2, ColLayout cols, int d, int cap_physC, int s, int sh,
    int32_t *tmpE, int32_t *tmpK, int32_t *tmpR, int32_t *tmpOff, PlanHeader *hdr, int fast_lds, const int32_t *skipB) {
    __shared__ int lds[40];
    extern __shared__ __attribute__((aligned(16))) int32_t fast_rows[];  // 2 * max(n, h) ints, if the launch gave them
    if (hdr->overflow) return;
    if (blockIdx.x >= 1 && skipB && *skipB) return;  // keep-weights mode: these layouts stand as they are
    // rows of A: the GEMM epilogue folds them chunk by chunk; rows of B (columns of C): tile by tile
    if (blockIdx.x == 0)
        rows_layout(rowA, n, &hdr->n_u, layA, cap_physA, cap_physA / kTile + 2, tmpPA, hdr, 0, kChunk, lds, fast_lds ? fast_rows : nullptr);
    else if (blockIdx.x == 1)
        rows_layout(rowB, h, &hdr->h_u, layB, cap_physB, cap_physB / kTile + 2, tmpPB, hdr, 1, kTile, lds, fast_lds ? fast_rows : nullptr);
    else {
        cols_layout(c1, c2, cols, d, cap_physC, s, sh, tmpE, tmpK, tmpR, tmpOff, hdr, lds, (int)blockIdx.x - 2);
        if (blockIdx.x == 2 && threadIdx.x == 0) hdr->bound[0] = hdr->bound[1] = 0;
    }
}

// ---------------------------------------------------------------------------------------------
// strategy pricing (Sec. 4.2)
// ---------------------------------------------------------------------------------------------
// out[0] = sum_i L(rowmaxA_i), out[1] = sum_j L(rowmaxB_j), out[2] = sum_k L(colmaxA_k),
// out[3] = sum_k L(colmaxB_k), out[4] = sum_k L(colmaxA_k) * L(colmaxB_k); L = number of base-s digits.
__global__ __launch_bounds__(256) void price_kernel(const int32_t *rowmaxA, int64_t n, const int32_t *rowmaxB,
                                                    int64_t h, const int32_t *colmaxA, const int32_t *colmaxB,
                                                    int64_t d, int sh, unsigned long long *out) {
    unsigned long long acc[5] = {0, 0, 0, 0, 0};
    const int64_t stride = (int64_t)gridDim.x * blockDim.x, t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t i = t0; i < n; i += stride) acc[0] += digit_levels(rowmaxA[i], sh);
    for (int64_t j = t0; j < h; j += stride) acc[1] += digit_levels(rowmaxB[j], sh);
    for (int64_t k = t0; k < d; k += stride) {
        const int la = digit_levels(colmaxA[k], sh), lb = digit_levels(colmaxB[k], sh);
        acc[2] += la;
        acc[3] += lb;
        acc[4] += (unsigned long long)la * lb;
    }
#pragma unroll
    for (int q = 0; q < 5; ++q) {
        unsigned long long v = acc[q];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        if ((threadIdx.x & 63) == 0 && v) atomicAdd(&out[q], v);
    }
}

__global__ void clear_sums_kernel(unsigned long long *p, int count) {
    if ((int)threadIdx.x < count) p[threadIdx.x] = 0;
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
int scan_i32(const int32_t *Q, int64_t rows, int64_t cols, int64_t ldq, int b,
             const imunpack_stats_t *st, hipStream_t stream);

struct Carver {
    char *base;
    size_t off;
    template <typename T>
    T *take(size_t count) {
        off = (off + 255) & ~(size_t)255;
        T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
        off += count * sizeof(T);
        return p;
    }
};

static void carve_slots(Carver &cv, SlotSet &s, int cap) {
    s.root = cv.take<int32_t>(cap);
    s.exp = cv.take<int32_t>(cap);
    s.time = cv.take<uint32_t>(cap);
    s.child = cv.take<int32_t>(cap);
    s.key = cv.take<unsigned long long>(cap);
    s.cap = cap;
}

static inline int phys_cap_rows(int cap) { return (int)((int64_t)cap * kChunk / (kChunk - 8) + 2 * kTile); }
static inline int phys_cap_cols(int cap) { return cap + kMaxGroups * kKPad; }

// Lays every device array out in the arena for the current capacities; returns the bytes needed.
static size_t carve(Plan *p, char *base, bool own_statsA, bool own_statsB) {
    Carver cv{base, 0};
    const int n = (int)p->n, d = (int)p->d, h = (int)p->h;
    p->d_hdr = cv.take<PlanHeader>(1);
    carve_slots(cv, p->rowA, p->cap[CAP_ROWA]);
    carve_slots(cv, p->rowB, p->cap[CAP_ROWB]);
    carve_slots(cv, p->c1, p->cap[CAP_C1]);
    carve_slots(cv, p->c2, p->cap[CAP_C2]);
    for (int op = 0; op < 2; ++op) {
        RowLayout &l = op ? p->layB : p->layA;
        const int cap = p->cap[op ? CAP_ROWB : CAP_ROWA], nb = op ? h : n;
        const int pc = phys_cap_rows(cap);
        l.prow_slot = cv.take<int32_t>(pc);
        l.prow_src = cv.take<int32_t>(pc);
        l.prow_exp = cv.take<int32_t>(pc);
        l.row_phys = cv.take<int32_t>(cap);
        l.src_pstart = cv.take<int32_t>(nb + 1);
        l.src_nlev = cv.take<int32_t>(nb + 1);
        l.tile_src0 = cv.take<int32_t>(pc / kTile + 2);
        l.chunk_src0 = cv.take<int32_t>(pc / kChunk + 8);
        l.tile_flat = cv.take<int32_t>(pc / kTile + 2);
        l.rowsum = cv.take<unsigned long long>(pc);
        l.wavesum = cv.take<unsigned long long>((size_t)pc * ((phys_cap_cols(p->cap[CAP_C2]) + 1023) / 1024));
    }
    {
        const int kc = phys_cap_cols(p->cap[CAP_C2]);
        p->cols.pcol_slot = cv.take<int32_t>(kc);
        p->cols.col_phys = cv.take<int32_t>(p->cap[CAP_C2]);
        p->cols.colB_k = cv.take<int32_t>(kc);
        p->cols.colB_e = cv.take<int32_t>(kc);
        p->cols.col_sexp = cv.take<int32_t>(kc);
        p->cols.unitB = cv.take<int4>(kc / 16 + 1);
        p->cols.acol_phys = cv.take<int32_t>(p->cap[CAP_C2]);
        p->cols.apos = cv.take<int32_t>(p->cap[CAP_C1]);
        p->cols.colA_k = cv.take<int32_t>(kc);
        p->cols.colA_e = cv.take<int32_t>(kc);
        p->cols.colA_w = cv.take<unsigned long long>(kc);
        p->cols.unitA = cv.take<int4>(kc / 16 + 1);
        p->cols.unitA_w = cv.take<unsigned long long>(kc / 16 + 1);
        p->cols.ktile_ablk = cv.take<int32_t>(kc / kKPad + 1);
        p->tmpE = cv.take<int32_t>(p->cap[CAP_C2]);
        p->tmpK = cv.take<int32_t>(p->cap[CAP_C2]);
        p->tmpR = cv.take<int32_t>(p->cap[CAP_C2]);
        p->tmpOff = cv.take<int32_t>((size_t)kColBlocks * (d + 1));
    }
    p->canon_rowphysA = cv.take<int32_t>(p->cap[CAP_ROWA]);
    p->canon_rowphysB = cv.take<int32_t>(p->cap[CAP_ROWB]);
    p->canon_colphys = cv.take<int32_t>(p->cap[CAP_C2]);
    p->canon_acolphys = cv.take<int32_t>(p->cap[CAP_C2]);
    if (own_statsA) {
        p->statsA[0] = cv.take<int32_t>(n); p->statsA[1] = cv.take<int32_t>(d);
        p->statsA[2] = cv.take<int32_t>(n); p->statsA[3] = cv.take<int32_t>(d);
    }
    if (own_statsB) {
        p->statsB[0] = cv.take<int32_t>(h); p->statsB[1] = cv.take<int32_t>(d);
        p->statsB[2] = cv.take<int32_t>(h); p->statsB[3] = cv.take<int32_t>(d);
    }
    const int maxslots = std::max(std::max(p->cap[CAP_ROWA], p->cap[CAP_ROWB]), std::max(p->cap[CAP_C1], p->cap[CAP_C2]));
    p->tmpL = cv.take<int32_t>(maxslots);
    p->tmpCur = cv.take<int32_t>(maxslots);
    p->tmpPA = cv.take<int32_t>(n + 1);
    p->tmpPB = cv.take<int32_t>(h + 1);
    if (p->sA == IMUNPACK_BOTH || p->sB == IMUNPACK_BOTH) {
        const int ecap = std::max(p->sA == IMUNPACK_BOTH ? p->cap[CAP_EDGEA] : 0,
                                  p->sB == IMUNPACK_BOTH ? p->cap[CAP_EDGEB] : 0);
        p->edges = cv.take<unsigned long long>((size_t)2 * ecap + 2);
        p->obcopyA = cv.take<int32_t>(p->sA == IMUNPACK_BOTH ? (size_t)3 * p->cap[CAP_EDGEA] : 0);
        p->obcopyB = cv.take<int32_t>(p->sB == IMUNPACK_BOTH ? (size_t)3 * p->cap[CAP_EDGEB] : 0);
        p->edge_cap = ecap;
        const int rcap = std::max(p->cap[CAP_ROWA], p->cap[CAP_ROWB]), ccap = std::max(p->cap[CAP_C1], p->cap[CAP_C2]);
        p->rcnt = cv.take<int32_t>(rcap + 8);
    p->extraRows = cv.take<int32_t>(p->sB == IMUNPACK_BOTH ? (size_t)h + 1 : 0);
        p->ccnt = cv.take<int32_t>(ccap + 8);
        p->ob = cv.take<int32_t>((size_t)3 * p->cap[CAP_OB]);
    }
    p->snapRoot = cv.take<int32_t>(p->cap[CAP_C1]);
    p->snapExp = cv.take<int32_t>(p->cap[CAP_C1]);
    p->snapChild = cv.take<int32_t>(p->cap[CAP_C1]);
    p->d_keep = cv.take<KeepState>(1);
    return cv.off + 256;
}

static inline int grid_for(int64_t items, int threads, int maxblocks = 2048) {
    int64_t b = (items + threads - 1) / threads;
    if (b < 1) b = 1;
    if (b > maxblocks) b = maxblocks;
    return (int)b;
}

// The OB entries of an UnpackBoth operand, kept for the scatter's fix-up pass: the caller's list need
// not outlive the call.  Many workgroups, ahead of the (single-workgroup) greedy.  For the second
// operand the same pass finds the edges that the repeated columns add: B_e holds a copy of column k
// of B in every column slot of A's unpacking that descends from k, so an OB entry (j, k) of B is
// also an OB entry (j, c) for every such slot c.  The pass also writes the greedy's first edge list:
// entry t of the OB list packed at position t, the edges of repeated columns behind the last entry.
__global__ __launch_bounds__(256) void ob_copy_kernel(const int32_t *__restrict__ ob, int ob_cap,
                                                      const int32_t *ob_count, int32_t *__restrict__ keep, int keep_cap,
                                                      const int32_t *chain_child, unsigned long long *edges, int ecap,
                                                      int32_t *extras, int32_t *extra_rows, int sh, const int32_t *skip) {
    if (skip && *skip) return;  // keep-weights mode: this operand's unpacking is taken over as it stands
    const int n = min(*ob_count, ob_cap);
    for (int t = blockIdx.x * blockDim.x + threadIdx.x; t < n; t += gridDim.x * blockDim.x) {
        const int j = ob[t], k = ob[ob_cap + t], v = ob[2 * (size_t)ob_cap + t];
        if (t < keep_cap) {
            keep[t] = j;
            keep[keep_cap + t] = k;
            keep[2 * (size_t)keep_cap + t] = v;
        }
        const unsigned av = v < 0 ? 0u - (unsigned)v : (unsigned)v;
        const int L = digit_levels((int)av, sh);
        if (t < ecap) edges[t] = L >= 2 ? pack_edge(j, k, L) : 0ull;  // 0: no edge
        if (!chain_child) continue;
        int c = chain_child[k];
        for (int hop = 0; c >= 0 && hop < 64; c = chain_child[c], ++hop) {
            const int pos = n + atomicAdd(extras, 1);
            if (pos < ecap) edges[pos] = pack_edge(j, c, L);
            atomicAdd(&extra_rows[j], 1);
        }
    }
}

// ---- keep-weights mode (Sec. 4.2: weights are unpacked once, when they are loaded).  The unpacking of the
// second operand depends on the first only through the column slots of the first operand's unpacking
// (which columns of B_e are repeats, and their exponents).  If those are what they were for the plan
// before, the second operand's slots, its kept OB entries and its header fields are taken over.
// One workgroup: compares the column slots with the remembered ones and acts on the verdict.  Same slots: the
// header fields that the second operand's unpacking and the layouts of its rows and of the columns left are
// put back.  Different: its rows start afresh and the column weights are cleared for the column layout to come.
__global__ __launch_bounds__(kPlanThreads) void keep_decide_kernel(
    SlotSet c1, const int32_t *sroot, const int32_t *sexp, const int32_t *schild, KeepState *ks, int host_valid,
    PlanHeader *hdr, SlotSet rowB, int h /* rows that start as unsplit originals */, int32_t *extra_rows, int nextra,
    int32_t *col_weights, int nweights) {
    const int d1 = hdr->d1;
    bool differs = !host_valid || !ks->valid || d1 != ks->d1 || d1 > c1.cap || hdr->overflow != 0;
    if (!differs)
        for (int x = threadIdx.x; x < d1; x += kPlanThreads)
            differs = differs || c1.root[x] != sroot[x] || c1.exp[x] != sexp[x] || c1.child[x] != schild[x];
    const bool same = !__syncthreads_or(differs);
    if (threadIdx.x == 0) {
        ks->same = same;
        hdr->reusedB = same;
        if (same) {
            const PlanHeader &o = ks->saved;
            hdr->h_u = o.h_u; hdr->d_u = o.d_u; hdr->nobB = o.nobB; hdr->edgesB = o.edgesB; hdr->extras = o.extras;
            hdr->Np = o.Np; hdr->Kp = o.Kp; hdr->KA = o.KA; hdr->ldA = o.ldA; hdr->ldB = o.ldB;
            hdr->ntiles = o.ntiles; hdr->lmaxB = o.lmaxB; hdr->ngroups = o.ngroups; hdr->nruns = o.nruns;
        } else if (h) {
            hdr->h_u = h;
        }
    }
    if (same) {  // the group and run tables
        constexpr size_t g0 = offsetof(PlanHeader, grp_exp) / sizeof(int32_t), g1 = offsetof(PlanHeader, nruns) / sizeof(int32_t);
        constexpr size_t r0 = offsetof(PlanHeader, run_kt0) / sizeof(int32_t), r1 = offsetof(PlanHeader, edgesA) / sizeof(int32_t);
        const int32_t *src = reinterpret_cast<const int32_t *>(&ks->saved);
        int32_t *dst = reinterpret_cast<int32_t *>(hdr);
        for (size_t i = g0 + threadIdx.x; i < g1; i += kPlanThreads) dst[i] = src[i];
        for (size_t i = r0 + threadIdx.x; i < r1; i += kPlanThreads) dst[i] = src[i];
        return;
    }
    for (int x = threadIdx.x; x < h; x += kPlanThreads) identity_slot(rowB, x);
    for (int x = threadIdx.x; x < nextra; x += kPlanThreads) extra_rows[x] = 0;
    for (int x = threadIdx.x; x < nweights; x += kPlanThreads) col_weights[x] = 0;
}

// After a plan that unpacked the second operand anew: remember the column slots it was unpacked for and the
// header the plan completed.
__global__ void keep_remember_kernel(SlotSet c1, const PlanHeader *hdr, int32_t *sroot, int32_t *sexp, int32_t *schild,
                                     KeepState *ks) {
    if (ks->same) return;
    if (hdr->overflow || hdr->err || hdr->d1 > c1.cap) {
        if (blockIdx.x == 0 && threadIdx.x == 0) ks->valid = 0;
        return;
    }
    const int d1 = hdr->d1;
    for (int x = blockIdx.x * blockDim.x + threadIdx.x; x < d1; x += gridDim.x * blockDim.x) {
        sroot[x] = c1.root[x];
        sexp[x] = c1.exp[x];
        schild[x] = c1.child[x];
    }
    if (blockIdx.x == 0) {
        const int32_t *src = reinterpret_cast<const int32_t *>(hdr);
        int32_t *dst = reinterpret_cast<int32_t *>(&ks->saved);
        for (size_t i = threadIdx.x; i < sizeof(PlanHeader) / sizeof(int32_t); i += blockDim.x) dst[i] = src[i];
        if (threadIdx.x == 0) {
            ks->d1 = d1;
            ks->valid = 1;
        }
    }
}

static constexpr int kGreedyLdsMax = 136 * 1024;  // dynamic LDS the greedy may use for the two count vectors
static constexpr int kLayoutLdsMax = 128 * 1024;  // dynamic LDS the layouts kernel may use (its static tables take about 12 KiB)

// ob: the operand's OB entry list ([3][ob_cap], count on the device)
static int run_greedy(Plan *p, int phase, const int32_t *ob, int ob_cap, const int32_t *ob_count,
                      int which_list, hipStream_t st, const int32_t *skip = nullptr) {
    PlanHeader *hdr = p->d_hdr;
    const bool first = phase == 1;
    SlotSet &rows = first ? p->rowA : p->rowB;
    SlotSet &cols = first ? p->c1 : p->c2;
    GreedyArgs g;
    g.rows = rows; g.cols = cols;
    g.cols_init = first ? nullptr : &hdr->d1;
    g.chain_child = first ? nullptr : p->c1.child;
    g.chain_root = first ? nullptr : p->c1.root;
    int32_t **stats = first ? p->statsA : p->statsB;
    g.rowcnt = stats[0]; g.colcnt = stats[1]; g.rowmax = stats[2];
    g.ob = ob; g.ob_cap = ob_cap; g.ob_count = ob_count; g.which_list = which_list;
    g.edges = p->edges;
    g.ecap = std::min(p->cap[first ? CAP_EDGEA : CAP_EDGEB], p->edge_cap);
    g.rcnt = p->rcnt; g.ccnt = p->ccnt;
    g.ob_keep_count = first ? &hdr->nobA : &hdr->nobB;
    g.extra_rows = first ? nullptr : p->extraRows;
    g.nr_io = first ? &hdr->n_u : &hdr->h_u;
    g.nc_io = first ? &hdr->d1 : &hdr->d_u;
    g.ecount_out = first ? &hdr->edgesA : &hdr->edgesB;
    g.hdr = hdr;
    g.whichR = first ? CAP_ROWA : CAP_ROWB;
    g.whichC = first ? CAP_C1 : CAP_C2;
    g.whichE = first ? CAP_EDGEA : CAP_EDGEB;
    g.s = p->s; g.sh = p->sh;
    g.skip = skip;
    const size_t lds_bytes = ((size_t)((rows.cap + 7) & ~3) + (size_t)((cols.cap + 7) & ~3)) * sizeof(int32_t);
    static std::atomic<int> opted_in{0};  // the attribute is idempotent: a race sets the same value twice
    if (!opted_in.load(std::memory_order_acquire)) {
        IMU_HIP(hipFuncSetAttribute((const void *)greedy_both_kernel<true>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kGreedyLdsMax));
        opted_in.store(1, std::memory_order_release);
    }
    const int keep_cap = p->cap[first ? CAP_EDGEA : CAP_EDGEB];  // the stride the fix-up pass reads with
    hipLaunchKernelGGL(ob_copy_kernel, dim3(grid_for(ob_cap, 256, 128)), dim3(256), 0, st, ob, ob_cap, ob_count,
                       first ? p->obcopyA : p->obcopyB, keep_cap, (const int32_t *)g.chain_child, g.edges, g.ecap,
                       &hdr->extras, p->extraRows, p->sh, skip);
    if (lds_bytes <= (size_t)kGreedyLdsMax)
        hipLaunchKernelGGL(greedy_both_kernel<true>, dim3(1), dim3(kPlanThreads), lds_bytes, st, g);
    else
        hipLaunchKernelGGL(greedy_both_kernel<false>, dim3(1), dim3(kPlanThreads), 0, st, g);
    return launch_status();
}

static int enqueue_plan(Plan *p, const int32_t *A, int64_t lda, const int32_t *B, int64_t ldb,
                        const imunpack_stats_t *stA, const imunpack_stats_t *stB, bool own_statsA,
                        bool own_statsB, hipStream_t st) {
    PlanHeader *hdr = p->d_hdr;
    const int n = (int)p->n, d = (int)p->d, h = (int)p->h;
    // header cleared; the sets that start as unsplit originals with a size the host knows
    const int idA = p->sA != IMUNPACK_ROW ? n : 0, idC1 = p->sA != IMUNPACK_COL ? d : 0,
              idB = p->sB != IMUNPACK_ROW ? h : 0;
    if (idA > p->rowA.cap || idC1 > p->c1.cap || idB > p->rowB.cap) return IMUNPACK_EINVAL;
    // also cleared: the weights of the stored columns of A (the column layout adds to them)
    const int kcA = phys_cap_cols(p->cap[CAP_C2]);
    // keep-weights mode (UnpackBoth on the second operand): its rows are set up only once it is known that its
    // unpacking has to be redone
    const bool keep = p->keep_B != 0;
    hipLaunchKernelGGL(setup_kernel, dim3(grid_for(std::max(std::max(idA, idC1), std::max(idB, kcA)), 256, 64)),
                       dim3(256), 0, st, hdr, p->rowA, idA, &hdr->n_u, p->c1, idC1, &hdr->d1, p->rowB, keep ? 0 : idB,
                       &hdr->h_u, p->extraRows, (p->sB == IMUNPACK_BOTH && !keep) ? h : 0,
                       reinterpret_cast<int32_t *>(p->cols.colA_w), keep ? 0 : 2 * kcA, keep ? p->d_keep : nullptr);
    // OB entry lists for UnpackBoth: the caller's (from the fused quantize pass) if complete, else
    // this call's own scan produces one.  The two operands are planned one after the other, so one
    // own buffer serves both.
    const bool listA = p->sA == IMUNPACK_BOTH, listB = p->sB == IMUNPACK_BOTH;
    const bool callerA = listA && stA && stA->ob && stA->ob_count && stA->ob_cap > 0 && !p->ignore_listA;
    const bool callerB = listB && stB && stB->ob && stB->ob_count && stB->ob_cap > 0 && !p->ignore_listB;
    const bool scanA = own_statsA || (listA && !callerA), scanB = own_statsB || (listB && !callerB);
    auto scan_operand = [&](const int32_t *M, int rows, int64_t ld, int32_t **own, bool own_stats, bool list) {
        imunpack_stats_t sx;
        memset(&sx, 0, sizeof(sx));
        if (own_stats) { sx.rowcnt = own[0]; sx.colcnt = own[1]; sx.rowmax = own[2]; sx.colmax = own[3]; }
        if (list) { sx.ob = p->ob; sx.ob_cap = p->cap[CAP_OB]; sx.ob_count = &hdr->obcount; }
        return scan_i32(M, rows, d, ld, p->b, &sx, st);
    };
    if (scanA) IMU_TRY(scan_operand(A, n, lda, p->statsA, own_statsA, listA && !callerA));
    // ---- phase 1: Unpack(A, B, I, b, strategy_A)
    if (p->sA == IMUNPACK_ROW) {
        hipLaunchKernelGGL(level_major_kernel, dim3(1), dim3(kPlanThreads), 0, st, p->rowA, p->statsA[2],
                           (const int32_t *)nullptr, n, (const int32_t *)nullptr, p->sh, p->tmpL, p->tmpCur,
                           &hdr->n_u, hdr, (int)CAP_ROWA, (const int32_t *)nullptr);
    } else if (p->sA == IMUNPACK_COL) {
        hipLaunchKernelGGL(level_major_kernel, dim3(1), dim3(kPlanThreads), 0, st, p->c1, p->statsA[3],
                           (const int32_t *)nullptr, d, (const int32_t *)nullptr, p->sh, p->tmpL, p->tmpCur,
                           &hdr->d1, hdr, (int)CAP_C1, (const int32_t *)nullptr);
    } else {
        if (callerA) IMU_TRY(run_greedy(p, 1, stA->ob, (int)stA->ob_cap, stA->ob_count, CAP_LISTA, st));
        else IMU_TRY(run_greedy(p, 1, p->ob, p->cap[CAP_OB], &hdr->obcount, CAP_OB, st));
    }
    if (scanB) IMU_TRY(scan_operand(B, h, ldb, p->statsB, own_statsB, listB && !callerB));
    // ---- phase 2: Unpack(B_e, A_u, S_u, b, strategy_B); B_e has d1 columns
    const int32_t *skip = nullptr;
    if (keep) {
        hipLaunchKernelGGL(keep_decide_kernel, dim3(1), dim3(kPlanThreads), 0, st, p->c1, (const int32_t *)p->snapRoot,
                           (const int32_t *)p->snapExp, (const int32_t *)p->snapChild, p->d_keep, p->keep_valid, hdr, p->rowB,
                           idB, p->extraRows, p->sB == IMUNPACK_BOTH ? h : 0, reinterpret_cast<int32_t *>(p->cols.colA_w),
                           2 * kcA);
        skip = &p->d_keep->same;
    }
    if (p->sB == IMUNPACK_ROW) {
        hipLaunchKernelGGL(level_major_kernel, dim3(1), dim3(kPlanThreads), 0, st, p->rowB, p->statsB[2],
                           (const int32_t *)nullptr, h, (const int32_t *)nullptr, p->sh, p->tmpL, p->tmpCur,
                           &hdr->h_u, hdr, (int)CAP_ROWB, skip);
        hipLaunchKernelGGL(identity_slots_kernel, dim3(grid_for(p->cap[CAP_C2], 256, 64)), dim3(256), 0, st,
                           p->c2, (const int32_t *)&hdr->d1, &hdr->d_u, hdr, (int)CAP_C2, skip);
    } else if (p->sB == IMUNPACK_COL) {
        hipLaunchKernelGGL(level_major_kernel, dim3(1), dim3(kPlanThreads), 0, st, p->c2, p->statsB[3],
                           (const int32_t *)p->c1.root, 0, (const int32_t *)&hdr->d1, p->sh, p->tmpL,
                           p->tmpCur, &hdr->d_u, hdr, (int)CAP_C2, skip);
    } else {
        if (callerB) IMU_TRY(run_greedy(p, 2, stB->ob, (int)stB->ob_cap, stB->ob_count, CAP_LISTB, st, skip));
        else IMU_TRY(run_greedy(p, 2, p->ob, p->cap[CAP_OB], &hdr->obcount, CAP_OB, st, skip));
    }
    // ---- physical layouts
    // the row layouts keep two ints per source row in LDS when that fits beside the column layout's tables
    const size_t fast_bytes = (size_t)2 * std::max(n, h) * sizeof(int32_t);
    const int fast_lds = fast_bytes <= (size_t)kLayoutLdsMax ? 1 : 0;
    static std::atomic<int> layouts_opted_in{0};  // the attribute is idempotent: a race sets the same value twice
    if (!layouts_opted_in.load(std::memory_order_acquire)) {
        IMU_HIP(hipFuncSetAttribute((const void *)layouts_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLayoutLdsMax));
        layouts_opted_in.store(1, std::memory_order_release);
    }
    hipLaunchKernelGGL(layouts_kernel, dim3(2 + kColBlocks), dim3(kPlanThreads), fast_lds ? fast_bytes : 0, st, p->rowA, n, p->layA,
                       phys_cap_rows(p->cap[CAP_ROWA]), p->tmpPA, p->rowB, h, p->layB,
                       phys_cap_rows(p->cap[CAP_ROWB]), p->tmpPB, p->c1, p->c2, p->cols, d,
                       phys_cap_cols(p->cap[CAP_C2]), p->s, p->sh, p->tmpE, p->tmpK, p->tmpR, p->tmpOff, hdr, fast_lds,
                       keep ? (const int32_t *)&p->d_keep->same : (const int32_t *)nullptr);
    if (keep)
        hipLaunchKernelGGL(keep_remember_kernel, dim3(grid_for(p->cap[CAP_C1], 256, 16)), dim3(256), 0, st, p->c1,
                           (const PlanHeader *)hdr, p->snapRoot, p->snapExp, p->snapChild, p->d_keep);
    return launch_status();
}

int poll_ready(Plan *p) {
    hipError_t e = hipErrorNotReady;
    for (long spin = 0; spin < 20000000 && e == hipErrorNotReady; ++spin) e = hipEventQuery(p->ready);
    if (e == hipErrorNotReady) {  // a very long plan: stop burning the core
        (void)hipGetLastError();
        e = hipEventSynchronize(p->ready);
    }
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        (void)hipGetLastError();
        return IMUNPACK_EHIP;
    }
    return IMUNPACK_OK;
}

int fetch_header(Plan *p, size_t offset, size_t bytes, hipStream_t st) {
    if (!p->pin_hdr || offset + bytes > sizeof(PlanHeader)) return IMUNPACK_EINVAL;
    char *pin = reinterpret_cast<char *>(p->pin_hdr) + offset;
    IMU_HIP(hipMemcpyAsync(pin, reinterpret_cast<const char *>(p->d_hdr) + offset, bytes, hipMemcpyDeviceToHost, st));
    IMU_HIP(hipEventRecord(p->ready, st));
    IMU_TRY(poll_ready(p));
    memcpy(reinterpret_cast<char *>(&p->hdr) + offset, pin, bytes);
    return IMUNPACK_OK;
}

}  // namespace imu

using namespace imu;

extern "C" int imunpack_plan(const int32_t *A, int64_t n, int64_t d, int64_t lda, const int32_t *B,
                             int64_t h, int64_t ldb, int b, int strategy_A, int strategy_B,
                             const imunpack_stats_t *stats_A, const imunpack_stats_t *stats_B,
                             imunpack_plan_t **plan, imunpack_stream_t stream) {
    if (!A || !B || !plan || n <= 0 || d <= 0 || h <= 0 || lda < d || ldb < d || b < 2 || b > 8)
        return IMUNPACK_EINVAL;
    if (strategy_A < 0 || strategy_A > 2 || strategy_B < 0 || strategy_B > 2) return IMUNPACK_EINVAL;
    if (n > (1 << 24) || d > (1 << 24) || h > (1 << 24)) return IMUNPACK_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    Plan *p = *plan;
    if (!p) {
        p = new (std::nothrow) Plan();
        if (!p) return IMUNPACK_ENOMEM;
        memset(p, 0, sizeof(*p));
        if (hipHostMalloc((void **)&p->pin_hdr, sizeof(PlanHeader), hipHostMallocDefault) != hipSuccess ||
            hipEventCreateWithFlags(&p->ready, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&p->scattered, hipEventDisableTiming) != hipSuccess ||
            hipStreamCreateWithFlags(&p->side, hipStreamNonBlocking) != hipSuccess) {
            (void)hipGetLastError();
            if (p->side) (void)hipStreamDestroy(p->side);
            if (p->scattered) (void)hipEventDestroy(p->scattered);
            if (p->ready) (void)hipEventDestroy(p->ready);
            if (p->pin_hdr) (void)hipHostFree(p->pin_hdr);
            delete p;
            return IMUNPACK_ENOMEM;
        }
        p->guess_fusable = 1;
    }
    if (p->bound_pending) (void)resolve_bound(p);  // a copy into the header mirror is still in flight
    const bool same = p->valid && p->n == n && p->d == d && p->h == h && p->b == b && p->sA == strategy_A &&
                      p->sB == strategy_B;
    p->valid = 0;
    p->unpacked = 0;
    p->n = n; p->d = d; p->h = h; p->b = b; p->sA = strategy_A; p->sB = strategy_B;
    p->s = 1 << (b - 1); p->sh = b - 1;
    p->stream = st;
    if (!same) {
        // first guesses; every one of them is grown after a run that reports it too small
        p->cap[CAP_ROWA] = std::max(p->cap[CAP_ROWA], (int)(strategy_A == IMUNPACK_COL ? n : 2 * n + 256));
        p->cap[CAP_ROWB] = std::max(p->cap[CAP_ROWB], (int)(strategy_B == IMUNPACK_COL ? h : 2 * h + 256));
        p->cap[CAP_C1] = std::max(p->cap[CAP_C1], (int)(strategy_A == IMUNPACK_ROW ? d : 2 * d + 256));
        p->cap[CAP_C2] = std::max(p->cap[CAP_C2], (int)(2 * d + 512));
        p->cap[CAP_EDGEA] = std::max(p->cap[CAP_EDGEA], (int)std::min<int64_t>(n * d, std::max<int64_t>(n * d / 64, 4096)));
        p->cap[CAP_EDGEB] = std::max(p->cap[CAP_EDGEB], (int)std::min<int64_t>(2 * h * d, std::max<int64_t>(h * d / 64, 4096)));
        p->cap[CAP_OB] = std::max(p->cap[CAP_OB], (int)std::min<int64_t>(std::max(n, h) * d, std::max<int64_t>(std::max(n, h) * d / 64, 4096)));
        p->ignore_listA = p->ignore_listB = 0;
    }
    const bool ownA = !(stats_A && stats_A->rowcnt && stats_A->colcnt && stats_A->rowmax && stats_A->colmax);
    const bool ownB = !(stats_B && stats_B->rowcnt && stats_B->colcnt && stats_B->rowmax && stats_B->colmax);
    int rc = IMUNPACK_OK;
    for (int attempt = 0; attempt < 24; ++attempt) {
        const size_t need = carve(p, nullptr, ownA, ownB);
        if (need > p->arena_bytes) {
            if (p->arena) {
                hipError_t e = hipFree(p->arena);
                p->arena = nullptr;
                p->arena_bytes = 0;
                if (e != hipSuccess) { g_last_hip_error = (int)e; rc = IMUNPACK_EHIP; break; }
            }
            const size_t want = need + need / 4;
            hipError_t e = hipMalloc((void **)&p->arena, want);
            if (e != hipSuccess) { (void)hipGetLastError(); p->arena = nullptr; rc = IMUNPACK_ENOMEM; break; }
            p->arena_bytes = want;
        }
        carve(p, p->arena, ownA, ownB);
        {  // what is kept of the plan before is only good for the same arrays at the same addresses
            unsigned long long sig = (unsigned long long)(uintptr_t)p->arena * 1000003ull + (unsigned long long)(uintptr_t)p->d_keep;
            const long long parts[] = {n, d, h, b, strategy_A, strategy_B, ownA, ownB, (long long)(uintptr_t)B, (long long)ldb};
            for (long long v : parts) sig = sig * 1099511628211ull + (unsigned long long)v;
            for (int c = 0; c <= CAP_OB; ++c) sig = sig * 1099511628211ull + (unsigned long long)p->cap[c];
            if (sig != p->keep_sig) p->keep_valid = 0;
            p->keep_sig = sig;
        }
        if (!ownA) { p->statsA[0] = stats_A->rowcnt; p->statsA[1] = stats_A->colcnt; p->statsA[2] = stats_A->rowmax; p->statsA[3] = stats_A->colmax; }
        if (!ownB) { p->statsB[0] = stats_B->rowcnt; p->statsB[1] = stats_B->colcnt; p->statsB[2] = stats_B->rowmax; p->statsB[3] = stats_B->colmax; }
        rc = enqueue_plan(p, A, lda, B, ldb, stats_A, stats_B, ownA, ownB, st);
        if (rc != IMUNPACK_OK) break;
        rc = fetch_header(p, 0, sizeof(PlanHeader), st);
        if (rc != IMUNPACK_OK) break;
        if (p->hdr.err) { rc = p->hdr.err; p->keep_valid = 0; break; }
        if (!p->hdr.overflow) {
            p->valid = 1;
            p->canon_valid = 0;
            p->keep_valid = p->keep_B;
            if (!p->hdr.reusedB) p->kept_Beu = nullptr;  // what an earlier unpack wrote belongs to another plan
            p->fp6 = p->digits_req == IMUNPACK_DIGITS_FP6 && b <= 4;
            p->bothA = strategy_A == IMUNPACK_BOTH;
            p->bothB = strategy_B == IMUNPACK_BOTH;
            break;
        }
        p->keep_valid = 0;
        if (p->hdr.overflow & (1 << CAP_LISTA)) p->ignore_listA = 1;
        if (p->hdr.overflow & (1 << CAP_LISTB)) p->ignore_listB = 1;
        for (int c = 0; c <= CAP_OB; ++c)
            if (p->hdr.overflow & (1 << c)) {
                int64_t nv = std::max<int64_t>((int64_t)p->hdr.need[c] + p->hdr.need[c] / 8 + 256, (int64_t)p->cap[c] * 2);
                if (nv > (1ll << 30)) { rc = IMUNPACK_ENOMEM; break; }
                p->cap[c] = (int)nv;
            }
        if (rc != IMUNPACK_OK) break;
        rc = IMUNPACK_ENOMEM;  // stays if the attempts run out
    }
    if (rc != IMUNPACK_OK && !p->valid) {
        if (!*plan) {
            if (p->arena) (void)hipFree(p->arena);
            (void)hipStreamDestroy(p->side);
            (void)hipEventDestroy(p->scattered);
            (void)hipEventDestroy(p->ready);
            (void)hipHostFree(p->pin_hdr);
            delete p;
        }
        return rc;
    }
    *plan = p;
    return IMUNPACK_OK;
}

extern "C" int imunpack_plan_dims(const imunpack_plan_t *p, int64_t *n_u, int64_t *d_u, int64_t *h_u,
                                  int32_t *n_groups) {
    if (!p || !p->valid) return IMUNPACK_EINVAL;
    if (n_u) *n_u = p->hdr.n_u;
    if (d_u) *d_u = p->hdr.d_u;
    if (h_u) *h_u = p->hdr.h_u;
    if (n_groups) *n_groups = p->hdr.ngroups;
    return IMUNPACK_OK;
}

extern "C" int imunpack_plan_keep_weights(imunpack_plan_t *p, int keep) {
    if (!p) return IMUNPACK_EINVAL;
    p->keep_B = keep != 0;
    if (!keep) {
        p->keep_valid = 0;
        p->kept_Beu = nullptr;
    }
    return IMUNPACK_OK;
}

extern "C" int imunpack_plan_weights_reused(const imunpack_plan_t *p) {
    return (p && p->valid && p->hdr.reusedB) ? 1 : 0;
}

namespace imu {

// Canonical (paper-order) numbering of the slots of one set.  Slots are appended in runs: a level of
// the closed-form UnpackRow / UnpackColumn, or a batch of UnpackBoth.  Inside a run the paper's
// order is (count at the split descending, index of the split slot ascending), the index being the
// canonical one.  key = run << 48 | (0xFFFFFF - count) << 24 | split slot (internal numbering).
static int canonical_order(const SlotSet &set, int nbase, int count, const std::vector<int> *base_canon,
                           hipStream_t st, std::vector<int> &canon_of, std::vector<unsigned long long> &key) {
    canon_of.assign((size_t)count, 0);
    key.clear();
    for (int x = 0; x < nbase && x < count; ++x) canon_of[x] = base_canon ? (*base_canon)[x] : x;
    const int extra = count - nbase;
    if (extra <= 0) return IMUNPACK_OK;
    key.resize((size_t)extra);
    IMU_HIP(hipMemcpyAsync(key.data(), set.key + nbase, (size_t)extra * sizeof(unsigned long long),
                           hipMemcpyDeviceToHost, st));
    IMU_HIP(hipStreamSynchronize(st));
    std::vector<int> order((size_t)extra);
    std::vector<char> assigned((size_t)count, 0);
    for (int x = 0; x < nbase && x < count; ++x) assigned[x] = 1;
    for (int t = 0; t < extra; ++t) order[t] = t;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return (key[a] >> 48) < (key[b] >> 48); });
    int next = nbase;
    for (size_t lo = 0; lo < order.size();) {
        size_t hi = lo;
        const unsigned long long run = key[order[lo]] >> 48;
        while (hi < order.size() && (key[order[hi]] >> 48) == run) ++hi;
        auto minor = [&](int t) { return (unsigned)((key[t] >> 24) & 0xFFFFFF); };
        auto parent = [&](int t) { return (int)(key[t] & 0xFFFFFF); };
        for (size_t q = lo; q < hi; ++q) {  // the split slot must come from an earlier run
            const int par = parent(order[q]);
            if (par < 0 || par >= count || !assigned[par]) return IMUNPACK_EHIP;
        }
        std::sort(order.begin() + lo, order.begin() + hi, [&](int a, int b) {
            if (minor(a) != minor(b)) return minor(a) < minor(b);
            return canon_of[parent(a)] < canon_of[parent(b)];
        });
        for (size_t q = lo; q < hi; ++q) {
            canon_of[nbase + order[q]] = next++;
            assigned[nbase + order[q]] = 1;
        }
        lo = hi;
    }
    return IMUNPACK_OK;
}

struct CanonHost {
    std::vector<int> rowA, rowB, c1, c2;  // internal slot -> canonical slot
    std::vector<unsigned long long> keyA, keyB, key1, key2;  // sort keys of the appended slots of each set
};

static int fetch_i32(std::vector<int32_t> &dst, const int32_t *src, size_t count, hipStream_t st) {
    dst.resize(count);
    if (count) IMU_HIP(hipMemcpyAsync(dst.data(), src, count * 4, hipMemcpyDeviceToHost, st));
    return IMUNPACK_OK;
}

static int build_canonical(Plan *p, CanonHost &c) {
    hipStream_t st = p->stream;
    const PlanHeader &h = p->hdr;
    IMU_TRY(canonical_order(p->rowA, (int)p->n, h.n_u, nullptr, st, c.rowA, c.keyA));
    IMU_TRY(canonical_order(p->rowB, (int)p->h, h.h_u, nullptr, st, c.rowB, c.keyB));
    IMU_TRY(canonical_order(p->c1, (int)p->d, h.d1, nullptr, st, c.c1, c.key1));
    IMU_TRY(canonical_order(p->c2, h.d1, h.d_u, &c.c1, st, c.c2, c.key2));
    if (!p->canon_valid) {
        // physical row / column of every canonical slot, for imunpack_unpack_canonical
        std::vector<int32_t> phys, out;
        auto upload = [&](const int32_t *dev_phys, const std::vector<int> &canon, int32_t *dev_out) -> int {
            IMU_TRY(fetch_i32(phys, dev_phys, canon.size(), st));
            IMU_HIP(hipStreamSynchronize(st));
            out.assign(canon.size(), 0);
            for (size_t x = 0; x < canon.size(); ++x) out[(size_t)canon[x]] = phys[x];
            if (!out.empty()) IMU_HIP(hipMemcpy(dev_out, out.data(), out.size() * 4, hipMemcpyHostToDevice));
            return IMUNPACK_OK;
        };
        IMU_TRY(upload(p->layA.row_phys, c.rowA, p->canon_rowphysA));
        IMU_TRY(upload(p->layB.row_phys, c.rowB, p->canon_rowphysB));
        IMU_TRY(upload(p->cols.col_phys, c.c2, p->canon_colphys));
        IMU_TRY(upload(p->cols.acol_phys, c.c2, p->canon_acolphys));
        p->canon_valid = 1;
    }
    return IMUNPACK_OK;
}

int ensure_canonical(Plan *p) {
    if (p->canon_valid) return IMUNPACK_OK;
    CanonHost c;
    return build_canonical(p, c);
}

}  // namespace imu

extern "C" int imunpack_plan_export(imunpack_plan_t *p, int32_t *rowA_src, int32_t *rowA_exp,
                                    int32_t *rowB_src, int32_t *rowB_exp, int32_t *col_src,
                                    int32_t *col_exp, int32_t *col_parent, int32_t *ops, int64_t *n_ops) {
    if (!p || !p->valid) return IMUNPACK_EINVAL;
    hipStream_t st = p->stream;
    const PlanHeader &h = p->hdr;
    CanonHost c;
    IMU_TRY(build_canonical(p, c));
    std::vector<int32_t> root, ex, root1, ex1;
    auto rows_out = [&](const SlotSet &set, const std::vector<int> &canon, int32_t *o_src, int32_t *o_exp) -> int {
        if (!o_src && !o_exp) return IMUNPACK_OK;
        IMU_TRY(fetch_i32(root, set.root, canon.size(), st));
        IMU_TRY(fetch_i32(ex, set.exp, canon.size(), st));
        IMU_HIP(hipStreamSynchronize(st));
        for (size_t x = 0; x < canon.size(); ++x) {
            if (o_src) o_src[canon[x]] = root[x];
            if (o_exp) o_exp[canon[x]] = ex[x];
        }
        return IMUNPACK_OK;
    };
    IMU_TRY(rows_out(p->rowA, c.rowA, rowA_src, rowA_exp));
    IMU_TRY(rows_out(p->rowB, c.rowB, rowB_src, rowB_exp));
    if (col_src || col_exp) {
        IMU_TRY(fetch_i32(root, p->c2.root, (size_t)h.d_u, st));
        IMU_TRY(fetch_i32(ex, p->c2.exp, (size_t)h.d_u, st));
        IMU_TRY(fetch_i32(root1, p->c1.root, (size_t)h.d1, st));
        IMU_TRY(fetch_i32(ex1, p->c1.exp, (size_t)h.d1, st));
        IMU_HIP(hipStreamSynchronize(st));
        for (int x = 0; x < h.d_u; ++x) {
            const int r1 = root[x];  // column slot after unpacking A that this column descends from
            if (col_src) col_src[c.c2[x]] = root1[r1];
            if (col_exp) col_exp[c.c2[x]] = ex1[r1] + ex[x];
        }
    }
    // The appended slots in the paper's numbering are numbered in the order their splits were made, and
    // the sort key of an appended slot names the slot that was split for it (low 24 bits, internal
    // numbering) and the run it was made in (level of the closed-form UnpackRow / UnpackColumn, batch of
    // UnpackBoth; a batch holds splits of one kind only).
    const int d = (int)p->d, nA = (int)p->n, nB = (int)p->h;
    auto parent_of = [](const std::vector<unsigned long long> &key, int t) { return (int)(key[(size_t)t] & 0xFFFFFF); };
    if (col_parent) {
        for (int x = 0; x < h.d1; ++x)  // the columns the second call started from: originals and A's appended ones
            col_parent[c.c2[x]] = x < d ? -1 : c.c2[(size_t)parent_of(c.key1, x - d)];
        for (int x = h.d1; x < h.d_u; ++x) col_parent[c.c2[x]] = c.c2[(size_t)parent_of(c.key2, x - h.d1)];
    }
    const int64_t total_ops = (int64_t)(h.n_u - nA) + (h.d1 - d) + (h.h_u - nB) + (h.d_u - h.d1);
    if (n_ops) *n_ops = total_ops;
    if (ops) {
        struct Op { unsigned long long run; int kind, canon, parent; };
        int64_t at = 0;
        for (int call = 0; call < 2; ++call) {
            const std::vector<int> &rc = call ? c.rowB : c.rowA, &cc = call ? c.c2 : c.c1;
            const std::vector<unsigned long long> &rk = call ? c.keyB : c.keyA, &ck = call ? c.key2 : c.key1;
            const int rbase = call ? nB : nA, cbase = call ? h.d1 : d;
            std::vector<Op> seq;
            seq.reserve(rk.size() + ck.size());
            for (size_t t = 0; t < rk.size(); ++t)
                seq.push_back({rk[t] >> 48, 0, rc[(size_t)rbase + t], rc[(size_t)parent_of(rk, (int)t)]});
            for (size_t t = 0; t < ck.size(); ++t)
                seq.push_back({ck[t] >> 48, 1, cc[(size_t)cbase + t], cc[(size_t)parent_of(ck, (int)t)]});
            // one-axis strategies append along one axis only: creation order is the numbering; UnpackBoth
            // interleaves the axes batch by batch
            std::sort(seq.begin(), seq.end(), [](const Op &a, const Op &b) {
                if (a.run != b.run) return a.run < b.run;
                return a.canon < b.canon;
            });
            for (const Op &o : seq) {
                ops[3 * at] = call;
                ops[3 * at + 1] = o.kind;
                ops[3 * at + 2] = o.parent;
                ++at;
            }
        }
    }
    return IMUNPACK_OK;
}

extern "C" int imunpack_plan_destroy(imunpack_plan_t *p) {
    if (!p) return IMUNPACK_OK;
    int rc = IMUNPACK_OK;
    if (p->arena) {
        hipError_t e = hipFree(p->arena);
        if (e != hipSuccess) { g_last_hip_error = (int)e; rc = IMUNPACK_EHIP; }
    }
    if (p->bound_pending) (void)resolve_bound(p);
    if (p->side) (void)hipStreamDestroy(p->side);
    if (p->scattered) (void)hipEventDestroy(p->scattered);
    if (p->ready) (void)hipEventDestroy(p->ready);
    if (p->pin_hdr) (void)hipHostFree(p->pin_hdr);
    delete p;
    return rc;
}

extern "C" int imunpack_price(const imunpack_stats_t *stA, int64_t n, const imunpack_stats_t *stB, int64_t h,
                              int64_t d, int b, void *workspace, int64_t *dims_out, double *ratio_out, int *best_A,
                              int *best_B, imunpack_stream_t stream) {
    if (!stA || !stB || !stA->rowmax || !stA->colmax || !stB->rowmax || !stB->colmax || !workspace || n <= 0 ||
        h <= 0 || d <= 0 || b < 2 || b > 8 || (uintptr_t)workspace % 8)
        return IMUNPACK_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    unsigned long long *sums = static_cast<unsigned long long *>(workspace), host[5];
    static_assert(IMUNPACK_PRICE_WORKSPACE_BYTES >= sizeof(host), "workspace");
    hipLaunchKernelGGL(clear_sums_kernel, dim3(1), dim3(64), 0, st, sums, 5);
    const int64_t longest = std::max(std::max(n, h), d);
    hipLaunchKernelGGL(price_kernel, dim3(grid_for(longest, 256, 1024)), dim3(256), 0, st, stA->rowmax, n,
                       stB->rowmax, h, stA->colmax, stB->colmax, d, b - 1, sums);
    IMU_TRY(launch_status());
    IMU_HIP(hipMemcpyAsync(host, sums, sizeof(host), hipMemcpyDeviceToHost, st));
    IMU_HIP(hipStreamSynchronize(st));
    // (strategy_A, strategy_B): (ROW,ROW), (ROW,COL), (COL,ROW), (COL,COL)
    const unsigned long long dims[4][3] = {{host[0], (unsigned long long)d, host[1]},
                                            {host[0], host[3], (unsigned long long)h},
                                            {(unsigned long long)n, host[2], host[1]},
                                            {(unsigned long long)n, host[4], (unsigned long long)h}};
    double best = 0.0;
    int bi = -1;
    for (int q = 0; q < 4; ++q) {
        for (int c = 0; c < 3; ++c) {
            if (dims[q][c] > (1ull << 62)) return IMUNPACK_ERANGE;
            if (dims_out) dims_out[3 * q + c] = (int64_t)dims[q][c];
        }
        const double r = ((double)dims[q][0] / (double)n) * ((double)dims[q][1] / (double)d) *
                         ((double)dims[q][2] / (double)h);
        if (ratio_out) ratio_out[q] = r;
        if (bi < 0 || r < best) { best = r; bi = q; }
    }
    if (best_A) *best_A = (bi & 2) ? IMUNPACK_COL : IMUNPACK_ROW;
    if (best_B) *best_B = (bi & 1) ? IMUNPACK_COL : IMUNPACK_ROW;
    return IMUNPACK_OK;
}
