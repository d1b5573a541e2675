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

#include <algorithm>
#include <cstring>
#include <new>

namespace imu {

constexpr int kPlanThreads = 1024;
constexpr int kPlanWaves = kPlanThreads / 64;

// ---------------------------------------------------------------------------------------------
// workgroup-wide helpers (kPlanThreads threads)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int block_excl_scan(int v, int &total, int *lds /* >= 40 ints */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int t = __shfl_up(incl, off, 64);
        if (lane >= off) incl += t;
    }
    if (lane == 63) lds[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        int w = lane < kPlanWaves ? lds[lane] : 0;
        int wi = w;
#pragma unroll
        for (int off = 1; off < kPlanWaves; off <<= 1) {
            int t = __shfl_up(wi, off, 64);
            if (lane >= off) wi += t;
        }
        if (lane < kPlanWaves) lds[lane] = wi - w;
        if (lane == kPlanWaves - 1) lds[32] = wi;
    }
    __syncthreads();
    const int res = lds[wave] + incl - v;
    total = lds[32];
    __syncthreads();
    return res;
}

__device__ __forceinline__ int block_max(int v, int *lds /* >= 40 ints */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = max(v, __shfl_xor(v, off, 64));
    if (lane == 0) lds[wave] = v;
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

// ---------------------------------------------------------------------------------------------
// header / identity
// ---------------------------------------------------------------------------------------------
__global__ void init_header_kernel(PlanHeader *hdr) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        PlanHeader z;
        memset(&z, 0, sizeof(z));
        *hdr = z;
    }
}

// slots 0..N-1 become unsplit originals; N comes from the host or from a header field
__global__ void identity_slots_kernel(SlotSet set, int n_host, const int32_t *n_dev, int32_t *count_out,
                                      PlanHeader *hdr, int which) {
    if (hdr->overflow) return;
    const int N = n_dev ? *n_dev : n_host;
    if (N > set.cap) {
        if (blockIdx.x == 0 && threadIdx.x == 0) flag_overflow(hdr, which, N);
        return;
    }
    for (int x = blockIdx.x * blockDim.x + threadIdx.x; x < N; x += gridDim.x * blockDim.x) {
        set.root[x] = x;
        set.exp[x] = 0;
        set.time[x] = kNever;
        set.child[x] = -1;
    }
    if (count_out && blockIdx.x == 0 && threadIdx.x == 0) *count_out = N;
}

// ---------------------------------------------------------------------------------------------
// UnpackRow / UnpackColumn in closed form (Alg. 1 / Alg. 2)
// ---------------------------------------------------------------------------------------------
// Base items x = 0..N-1 with largest magnitude maxabs[via ? via[x] : x]; every level l >= 1 appends
// the items that still have a digit there, in ascending x.
__global__ __launch_bounds__(kPlanThreads) void level_major_kernel(
    SlotSet set, const int32_t *maxabs, const int32_t *via, int n_host, const int32_t *n_dev, int sh,
    int32_t *tmpL, int32_t *tmpCur, int32_t *count_out, PlanHeader *hdr, int which) {
    __shared__ int lds[40];
    if (hdr->overflow) return;
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
        set.root[x] = x;
        set.exp[x] = 0;
        set.time[x] = kNever;
        set.child[x] = -1;
        lm = max(lm, L);
    }
    const int lmax = block_max(lm, lds);
    int base = N;
    for (int l = 1; l < lmax; ++l) {
        for (int x0 = 0; x0 < N; x0 += kPlanThreads) {
            const int x = x0 + threadIdx.x;
            const int flag = (x < N && tmpL[x] > l) ? 1 : 0;
            int total;
            const int slot = base + block_excl_scan(flag, total, lds);
            if (flag && slot < set.cap) {
                set.root[slot] = x;
                set.exp[slot] = l;
                set.time[slot] = kNever;
                set.child[slot] = -1;
                const int prev = tmpCur[x];
                set.child[prev] = slot;
                set.time[prev] = 0;  // split (only this axis splits in this phase, any finite time will do)
                tmpCur[x] = slot;
            }
            base += total;
        }
    }
    if (threadIdx.x == 0) {
        *count_out = base;
        if (base > set.cap) flag_overflow(hdr, which, base);
    }
}

// ---------------------------------------------------------------------------------------------
// UnpackBoth (Alg. 4): OB entry lists
// ---------------------------------------------------------------------------------------------
// Appends every OB entry (|v| >= s) of M (rows x cols, row stride ld) as (row, col, value).
__global__ __launch_bounds__(256) void coo_extract_kernel(const int32_t *__restrict__ M, int64_t rows,
                                                          int64_t cols, int64_t ld, int s,
                                                          int32_t *oR, int32_t *oC, int32_t *oV, int cap,
                                                          int32_t *counter, PlanHeader *hdr) {
    if (hdr->overflow) return;
    const int lane = threadIdx.x & 63;
    const int64_t wave_id = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    const int64_t chunks_per_row = (cols + 63) / 64;
    for (int64_t w = wave_id; w < rows * chunks_per_row; w += nwaves) {
        const int64_t r = w / chunks_per_row;
        const int64_t c = (w % chunks_per_row) * 64 + lane;
        int32_t v = 0;
        if (c < cols) v = M[r * ld + c];
        const bool ob = v >= s || v <= -s;
        const unsigned long long mask = __ballot(ob);
        if (mask == 0) continue;
        int base = 0;
        if (lane == 0) base = atomicAdd(counter, __popcll(mask));
        base = __shfl(base, 0, 64);
        if (ob) {
            const int pos = base + __popcll(mask & ((1ull << lane) - 1ull));
            if (pos < cap) {
                oR[pos] = (int32_t)r;
                oC[pos] = (int32_t)c;
                oV[pos] = v;
            }
        }
    }
}

// After UnpackA the matrix B_e repeats column k of B once per column slot that descends from k
// (Alg. 2 line 6 / Alg. 4 line 13), so each OB entry (j, k) of B becomes one edge per such slot.
__global__ void expand_edges_kernel(const int32_t *rawJ, const int32_t *rawK, const int32_t *rawV,
                                    const int32_t *raw_count, int raw_cap, SlotSet c1, int32_t *eR,
                                    int32_t *eC, int32_t *eV, int cap, int32_t *counter, PlanHeader *hdr) {
    if (hdr->overflow) return;
    const int N = min(*raw_count, raw_cap);
    for (int t = blockIdx.x * blockDim.x + threadIdx.x; t < N; t += gridDim.x * blockDim.x) {
        int len = 0;
        for (int c = rawK[t]; c >= 0 && len < 64; c = c1.child[c]) ++len;
        int pos = atomicAdd(counter, len);
        int left = len;
        for (int c = rawK[t]; c >= 0 && left > 0; c = c1.child[c], ++pos, --left) {
            if (pos < cap) {
                eR[pos] = rawJ[t];
                eC[pos] = c;
                eV[pos] = rawV[t];
            }
        }
    }
}

__global__ void check_count_kernel(const int32_t *count, int cap, PlanHeader *hdr, int which) {
    if (threadIdx.x == 0 && blockIdx.x == 0 && *count > cap) flag_overflow(hdr, which, *count);
}

__global__ void edge_count_kernel(const int32_t *eR, const int32_t *eC, const int32_t *ecount, int32_t *rcnt,
                                  int32_t *ccnt, PlanHeader *hdr) {
    if (hdr->overflow) return;
    const int E = *ecount;
    for (int e = blockIdx.x * blockDim.x + threadIdx.x; e < E; e += gridDim.x * blockDim.x) {
        atomicAdd(&rcnt[eR[e]], 1);
        atomicAdd(&ccnt[eC[e]], 1);
    }
}

// exclusive prefix sums of the two count vectors -> list starts; cursors zeroed
__global__ __launch_bounds__(kPlanThreads) void edge_scan_kernel(const int32_t *rcnt, const int32_t *ccnt,
                                                                 const int32_t *nr_dev, const int32_t *nc_dev,
                                                                 int32_t *rstart, int32_t *rlen,
                                                                 int32_t *cstart, int32_t *clen,
                                                                 PlanHeader *hdr) {
    __shared__ int lds[40];
    if (hdr->overflow) return;
    for (int pass = 0; pass < 2; ++pass) {
        const int32_t *cnt = pass ? ccnt : rcnt;
        int32_t *start = pass ? cstart : rstart, *len = pass ? clen : rlen;
        const int N = pass ? *nc_dev : *nr_dev;
        int base = 0;
        for (int x0 = 0; x0 < N; x0 += kPlanThreads) {
            const int x = x0 + threadIdx.x;
            const int v = x < N ? cnt[x] : 0;
            int total;
            const int ex = block_excl_scan(v, total, lds);
            if (x < N) {
                start[x] = base + ex;
                len[x] = 0;
            }
            base += total;
        }
    }
}

__global__ void edge_fill_kernel(const int32_t *eR, const int32_t *eC, const int32_t *ecount,
                                 const int32_t *rstart, int32_t *rlen, const int32_t *cstart, int32_t *clen,
                                 int32_t *redge, int32_t *cedge, PlanHeader *hdr) {
    if (hdr->overflow) return;
    const int E = *ecount;
    for (int e = blockIdx.x * blockDim.x + threadIdx.x; e < E; e += gridDim.x * blockDim.x) {
        const int R = eR[e], C = eC[e];
        redge[rstart[R] + atomicAdd(&rlen[R], 1)] = e;
        cedge[cstart[C] + atomicAdd(&clen[C], 1)] = e;
    }
}

// ---------------------------------------------------------------------------------------------
// UnpackBoth (Alg. 4): the greedy
// ---------------------------------------------------------------------------------------------
struct GreedyArgs {
    SlotSet rows, cols;
    int32_t *rcnt, *ccnt;          // live OB count per row / column slot
    int32_t *rstart, *rlen;        // per row slot: segment of redge
    int32_t *cstart, *clen;        // per column slot: segment of cedge
    int32_t *redge, *cedge;        // edge ids grouped by row / by column
    int32_t *eR, *eC, *eV;         // current row slot, column slot and remaining value of each edge
    int32_t *batch;
    int batch_cap;
    int32_t *nr_io, *nc_io;        // slot counts (header fields), read at entry, written at exit
    const int32_t *ecount;         // number of edges
    PlanHeader *hdr;
    int whichR, whichC;
    int s, sh;
};

// One batch: split every slot of `mine` listed in batch[0..nb) (ascending index), in that order.
// A split keeps digit 0 in place and moves floor(v / s) to the new slot (Alg. 4 lines 7-9 / 11-14);
// an entry that becomes In-Bound leaves the count of the crossing slot, one that stays OB moves on.
__device__ __forceinline__ void split_batch(const GreedyArgs &g, bool isrow, int N, int nb, uint32_t T) {
    const SlotSet &mine = isrow ? g.rows : g.cols;
    int32_t *cnt = isrow ? g.rcnt : g.ccnt, *other = isrow ? g.ccnt : g.rcnt;
    int32_t *start = isrow ? g.rstart : g.cstart, *len = isrow ? g.rlen : g.clen;
    int32_t *list = isrow ? g.redge : g.cedge;
    int32_t *epos = isrow ? g.eR : g.eC, *ecross = isrow ? g.eC : g.eR;
    for (int r = threadIdx.x; r < nb; r += kPlanThreads) {
        const int X = g.batch[r], newX = N + r;
        mine.time[X] = T + (uint32_t)r;
        mine.child[X] = newX;
        mine.root[newX] = mine.root[X];
        mine.exp[newX] = mine.exp[X] + 1;
        mine.time[newX] = kNever;
        mine.child[newX] = -1;
        start[newX] = start[X];
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int r = wave; r < nb; r += kPlanWaves) {
        const int X = g.batch[r], newX = N + r;
        const int st = start[X], ln = len[X];
        int out = 0;
        for (int off = 0; off < ln; off += 64) {
            const int idx = off + lane;
            const bool valid = idx < ln;
            const int e = valid ? list[st + idx] : 0;
            const int v = valid ? g.eV[e] : 0;
            const int av = v < 0 ? -v : v;
            const bool alive = valid && av >= g.s;
            const int av2 = av >> g.sh;
            const bool surv = alive && av2 >= g.s;
            if (alive) {
                g.eV[e] = v < 0 ? -av2 : av2;
                if (surv)
                    epos[e] = newX;
                else
                    atomicSub(&other[ecross[e]], 1);
            }
            const unsigned long long mask = __ballot(surv);
            if (surv) list[st + out + __popcll(mask & ((1ull << lane) - 1ull))] = e;
            out += __popcll(mask);
        }
        if (lane == 0) {
            len[newX] = out;
            __hip_atomic_store(&cnt[newX], out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&cnt[X], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __syncthreads();
}

__global__ __launch_bounds__(kPlanThreads) void greedy_both_kernel(GreedyArgs g) {
    __shared__ int lds[40];
    if (g.hdr->overflow) return;
    int nr = *g.nr_io, nc = *g.nc_io;
    uint32_t T = 0;
    // every batch retires at least one digit of one OB entry, and an entry has at most 32 digits
    const long long max_batches = 32ll * (long long)(*g.ecount) + 64;
    for (long long it = 0;; ++it) {
        if (it > max_batches) {
            if (threadIdx.x == 0) atomicMin(&g.hdr->err, IMUNPACK_EHIP);
            return;
        }
        int m0 = 0, m1 = 0;
        for (int x = threadIdx.x; x < nr; x += kPlanThreads) m0 = max(m0, load_agent(&g.rcnt[x]));
        for (int x = threadIdx.x; x < nc; x += kPlanThreads) m1 = max(m1, load_agent(&g.ccnt[x]));
        const int c0 = block_max(m0, lds), c1 = block_max(m1, lds);
        if (c0 == 0 && c1 == 0) break;
        const bool isrow = c0 >= c1;  // rows win ties (Alg. 4: "else if c0 >= c1")
        const int32_t *cnt = isrow ? g.rcnt : g.ccnt;
        const int N = isrow ? nr : nc, target = isrow ? c0 : c1;
        const int cap = isrow ? g.rows.cap : g.cols.cap;
        int nb = 0;
        for (int x0 = 0; x0 < N; x0 += kPlanThreads) {
            const int x = x0 + threadIdx.x;
            const int flag = (x < N && load_agent(&cnt[x]) == target) ? 1 : 0;
            int total;
            const int rank = nb + block_excl_scan(flag, total, lds);
            if (flag && rank < g.batch_cap) g.batch[rank] = x;
            nb += total;
        }
        if (N + nb > cap || nb > g.batch_cap) {
            if (threadIdx.x == 0) flag_overflow(g.hdr, isrow ? g.whichR : g.whichC, 2 * (N + nb));
            return;
        }
        __syncthreads();
        split_batch(g, isrow, N, nb, T);
        if (isrow) nr += nb; else nc += nb;
        T += (uint32_t)nb;
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
// row straddles a GEMM tile, so that Pi can be applied inside one tile's epilogue.  Source row i
// with unpadded start P_i goes to tile floor(P_i / (kTile - (Lmax-1))): a closed form, and the
// rows of a tile never exceed kTile.
__global__ __launch_bounds__(kPlanThreads) void rows_layout_kernel(SlotSet rows, int nbase,
                                                                   const int32_t *count_dev, RowLayout lay,
                                                                   int cap_phys, int cap_tiles,
                                                                   int32_t *tmpL, int32_t *tmpP,
                                                                   PlanHeader *hdr, int operand) {
    __shared__ int lds[40];
    __shared__ int s_ntiles;
    if (hdr->overflow) return;
    int lm = 1;
    for (int i = threadIdx.x; i < nbase; i += kPlanThreads) {
        int L = 1;
        for (int R = rows.child[i]; R >= 0 && L < 64; R = rows.child[R]) ++L;
        tmpL[i] = L;
        lm = max(lm, L);
    }
    const int lmax = block_max(lm, lds);
    int base = 0;
    for (int x0 = 0; x0 < nbase; x0 += kPlanThreads) {
        const int x = x0 + threadIdx.x;
        const int v = x < nbase ? tmpL[x] : 0;
        int total;
        const int ex = block_excl_scan(v, total, lds);
        if (x < nbase) tmpP[x] = base + ex;
        base += total;
    }
    __syncthreads();
    const int Tp = kTile - (lmax - 1);
    const int ntiles = nbase > 0 ? tmpP[nbase - 1] / Tp + 1 : 0;
    const int Mp = ntiles * kTile;
    if (Mp > cap_phys || ntiles + 1 > cap_tiles || base != *count_dev) {
        if (threadIdx.x == 0) {
            if (base != *count_dev) atomicMin(&hdr->err, IMUNPACK_EHIP);  // inconsistent plan: internal error
            else flag_overflow(hdr, operand ? CAP_ROWB : CAP_ROWA, 2 * base);
        }
        return;
    }
    for (int t = threadIdx.x; t <= ntiles; t += kPlanThreads) {
        // first i with P_i >= t * Tp
        int lo = 0, hi = nbase;
        const int want = t * Tp;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (tmpP[mid] >= want) hi = mid; else lo = mid + 1;
        }
        lay.tile_src0[t] = (t == ntiles) ? nbase : lo;
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
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nbase; i += kPlanThreads) {
        const int t = tmpP[i] / Tp;
        const int i0 = lay.tile_src0[t];
        const int pst = t * kTile + (tmpP[i] - tmpP[i0]);
        lay.src_pstart[i] = pst;
        lay.src_nlev[i] = tmpL[i];
        int l = 0;
        for (int R = i; R >= 0 && l < tmpL[i]; R = rows.child[R], ++l) {
            lay.prow_slot[pst + l] = R;
            lay.prow_src[pst + l] = i;
            lay.prow_exp[pst + l] = l;
            lay.row_phys[R] = pst + l;
        }
    }
    if (threadIdx.x == 0) {
        if (operand == 0) { hdr->Mp = Mp; hdr->mtiles = ntiles; hdr->lmaxA = lmax; }
        else { hdr->Np = Mp; hdr->ntiles = ntiles; hdr->lmaxB = lmax; }
    }
}

// Columns: grouped by the exponent of the diagonal entry of S (Alg. 3 runs one GEMM per distinct
// entry), highest exponent first, canonical order inside a group, each group zero-padded to a
// multiple of kKPad.
__global__ __launch_bounds__(kPlanThreads) void cols_layout_kernel(SlotSet c1, SlotSet c2, ColLayout cols,
                                                                   int cap_phys, int s, int sh,
                                                                   PlanHeader *hdr) {
    __shared__ int lds[40];
    __shared__ int hist[kMaxGroups];
    __shared__ int s_ng, s_kp;
    if (hdr->overflow) return;
    const int D = hdr->d_u;
    for (int e = threadIdx.x; e < kMaxGroups; e += kPlanThreads) hist[e] = 0;
    __syncthreads();
    for (int c = threadIdx.x; c < D; c += kPlanThreads) {
        const int e = c1.exp[c2.root[c]] + c2.exp[c];
        if (e < kMaxGroups) atomicAdd(&hist[e], 1);
        else atomicMin(&hdr->err, IMUNPACK_ERANGE);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int ng = 0, k0 = 0;
        const long long lim = 2147483647ll / ((long long)(s - 1) * (s - 1));
        for (int e = kMaxGroups - 1; e >= 0; --e) {
            if (!hist[e]) continue;
            if (e * sh > 62 || hist[e] > lim) atomicMin(&hdr->err, IMUNPACK_ERANGE);
            hdr->grp_exp[ng] = e;
            hdr->grp_k0[ng] = k0;
            hdr->grp_len[ng] = hist[e];
            k0 += (hist[e] + kKPad - 1) / kKPad * kKPad;
            ++ng;
        }
        hdr->ngroups = ng;
        hdr->Kp = k0;
        s_ng = ng;
        s_kp = k0;
        if (k0 > cap_phys) flag_overflow(hdr, CAP_C2, 2 * D);
    }
    __syncthreads();
    const int ng = s_ng, Kp = s_kp;
    if (Kp > cap_phys) return;
    for (int q = threadIdx.x; q < Kp; q += kPlanThreads) {
        cols.pcol_slot[q] = -1;
        cols.colA_k[q] = -1;
        cols.colA_c1[q] = 0;
        cols.colA_e[q] = 0;
        cols.colB_e[q] = 0;
        cols.col_sexp[q] = 0;
    }
    __syncthreads();
    for (int g = 0; g < ng; ++g) {
        const int ge = hdr->grp_exp[g];
        int base = hdr->grp_k0[g];
        for (int x0 = 0; x0 < D; x0 += kPlanThreads) {
            const int c = x0 + threadIdx.x;
            int flag = 0, root = 0, ea = 0, eb = 0;
            if (c < D) {
                root = c2.root[c];
                ea = c1.exp[root];
                eb = c2.exp[c];
                flag = (ea + eb == ge) ? 1 : 0;
            }
            int total;
            const int q = base + block_excl_scan(flag, total, lds);
            if (flag) {
                cols.pcol_slot[q] = c;
                cols.col_phys[c] = q;
                cols.colA_k[q] = c1.root[root];
                cols.colA_c1[q] = root;
                cols.colA_e[q] = ea;
                cols.colB_e[q] = eb;
                cols.col_sexp[q] = ge;
            }
            base += total;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
int scan_i32(const int32_t *Q, int64_t rows, int64_t cols, int64_t ldq, int b,
             const imunpack_stats_t *st, hipStream_t stream);
__global__ void fill_i32_kernel(int32_t *p, int64_t count, int32_t value);

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
    s.cap = cap;
}

static inline int phys_cap_rows(int cap) { return (int)((int64_t)cap * kTile / (kTile - 32) + 2 * kTile); }
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
        l.tile_flat = cv.take<int32_t>(pc / kTile + 2);
    }
    {
        const int kc = phys_cap_cols(p->cap[CAP_C2]);
        p->cols.pcol_slot = cv.take<int32_t>(kc);
        p->cols.col_phys = cv.take<int32_t>(p->cap[CAP_C2]);
        p->cols.colA_k = cv.take<int32_t>(kc);
        p->cols.colA_c1 = cv.take<int32_t>(kc);
        p->cols.colA_e = cv.take<int32_t>(kc);
        p->cols.colB_e = cv.take<int32_t>(kc);
        p->cols.col_sexp = cv.take<int32_t>(kc);
    }
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
    p->tmpP = cv.take<int32_t>(maxslots);
    if (p->sA == IMUNPACK_BOTH || p->sB == IMUNPACK_BOTH) {
        const int ecap = std::max(p->sA == IMUNPACK_BOTH ? p->cap[CAP_EDGEA] : 0,
                                  p->sB == IMUNPACK_BOTH ? p->cap[CAP_EDGEB] : 0);
        p->eR = cv.take<int32_t>(ecap); p->eC = cv.take<int32_t>(ecap); p->eV = cv.take<int32_t>(ecap);
        p->redge = cv.take<int32_t>(ecap); p->cedge = cv.take<int32_t>(ecap);
        const int rcap = std::max(p->cap[CAP_ROWA], p->cap[CAP_ROWB]), ccap = std::max(p->cap[CAP_C1], p->cap[CAP_C2]);
        p->rcnt = cv.take<int32_t>(rcap); p->rstart = cv.take<int32_t>(rcap); p->rlen = cv.take<int32_t>(rcap);
        p->ccnt = cv.take<int32_t>(ccap); p->cstart = cv.take<int32_t>(ccap); p->clen = cv.take<int32_t>(ccap);
        p->batch = cv.take<int32_t>(std::max(rcap, ccap));
        if (p->sB == IMUNPACK_BOTH) {
            p->rawJ = cv.take<int32_t>(p->cap[CAP_RAWB]);
            p->rawK = cv.take<int32_t>(p->cap[CAP_RAWB]);
            p->rawV = cv.take<int32_t>(p->cap[CAP_RAWB]);
        }
    }
    return cv.off + 256;
}

static inline int grid_for(int64_t items, int threads, int maxblocks = 2048) {
    int64_t b = (items + threads - 1) / threads;
    if (b < 1) b = 1;
    if (b > maxblocks) b = maxblocks;
    return (int)b;
}

static int run_greedy(Plan *p, int phase, hipStream_t st) {
    PlanHeader *hdr = p->d_hdr;
    const bool first = phase == 1;
    SlotSet &rows = first ? p->rowA : p->rowB;
    SlotSet &cols = first ? p->c1 : p->c2;
    int32_t *nr = first ? &hdr->n_u : &hdr->h_u;
    int32_t *nc = first ? &hdr->d1 : &hdr->d_u;
    int32_t *ecount = first ? &hdr->edgesA : &hdr->edgesB;
    const int ecap = p->cap[first ? CAP_EDGEA : CAP_EDGEB];
    // live counts start at zero for every slot that may ever exist
    hipLaunchKernelGGL(fill_i32_kernel, dim3(grid_for(rows.cap, 256)), dim3(256), 0, st, p->rcnt,
                       (int64_t)rows.cap, 0);
    hipLaunchKernelGGL(fill_i32_kernel, dim3(grid_for(cols.cap, 256)), dim3(256), 0, st, p->ccnt,
                       (int64_t)cols.cap, 0);
    hipLaunchKernelGGL(check_count_kernel, dim3(1), dim3(64), 0, st, ecount, ecap, hdr,
                       first ? CAP_EDGEA : CAP_EDGEB);
    hipLaunchKernelGGL(edge_count_kernel, dim3(grid_for(ecap, 256, 1024)), dim3(256), 0, st, p->eR, p->eC,
                       ecount, p->rcnt, p->ccnt, hdr);
    hipLaunchKernelGGL(edge_scan_kernel, dim3(1), dim3(kPlanThreads), 0, st, p->rcnt, p->ccnt, nr, nc,
                       p->rstart, p->rlen, p->cstart, p->clen, hdr);
    hipLaunchKernelGGL(edge_fill_kernel, dim3(grid_for(ecap, 256, 1024)), dim3(256), 0, st, p->eR, p->eC,
                       ecount, p->rstart, p->rlen, p->cstart, p->clen, p->redge, p->cedge, hdr);
    GreedyArgs g;
    g.rows = rows; g.cols = cols;
    g.rcnt = p->rcnt; g.ccnt = p->ccnt;
    g.rstart = p->rstart; g.rlen = p->rlen; g.cstart = p->cstart; g.clen = p->clen;
    g.redge = p->redge; g.cedge = p->cedge;
    g.eR = p->eR; g.eC = p->eC; g.eV = p->eV;
    g.batch = p->batch;
    g.batch_cap = std::max(std::max(p->cap[CAP_ROWA], p->cap[CAP_ROWB]), std::max(p->cap[CAP_C1], p->cap[CAP_C2]));
    g.nr_io = nr; g.nc_io = nc;
    g.ecount = ecount;
    g.hdr = hdr;
    g.whichR = first ? CAP_ROWA : CAP_ROWB;
    g.whichC = first ? CAP_C1 : CAP_C2;
    g.s = p->s; g.sh = p->sh;
    hipLaunchKernelGGL(greedy_both_kernel, dim3(1), dim3(kPlanThreads), 0, st, g);
    return launch_status();
}

static int enqueue_plan(Plan *p, const int32_t *A, int64_t lda, const int32_t *B, int64_t ldb,
                        bool own_statsA, bool own_statsB, hipStream_t st) {
    PlanHeader *hdr = p->d_hdr;
    const int n = (int)p->n, d = (int)p->d, h = (int)p->h;
    hipLaunchKernelGGL(init_header_kernel, dim3(1), dim3(64), 0, st, hdr);
    if (own_statsA) {
        imunpack_stats_t s{p->statsA[0], p->statsA[1], p->statsA[2], p->statsA[3]};
        IMU_TRY(scan_i32(A, n, d, lda, p->b, &s, st));
    }
    if (own_statsB) {
        imunpack_stats_t s{p->statsB[0], p->statsB[1], p->statsB[2], p->statsB[3]};
        IMU_TRY(scan_i32(B, h, d, ldb, p->b, &s, st));
    }
    // ---- phase 1: Unpack(A, B, I, b, strategy_A)
    if (p->sA == IMUNPACK_ROW) {
        hipLaunchKernelGGL(level_major_kernel, dim3(1), dim3(kPlanThreads), 0, st, p->rowA, p->statsA[2],
                           (const int32_t *)nullptr, n, (const int32_t *)nullptr, p->sh, p->tmpL, p->tmpCur,
                           &hdr->n_u, hdr, (int)CAP_ROWA);
        hipLaunchKernelGGL(identity_slots_kernel, dim3(grid_for(d, 256, 64)), dim3(256), 0, st, p->c1, d,
                           (const int32_t *)nullptr, &hdr->d1, hdr, (int)CAP_C1);
    } else if (p->sA == IMUNPACK_COL) {
        hipLaunchKernelGGL(identity_slots_kernel, dim3(grid_for(n, 256, 64)), dim3(256), 0, st, p->rowA, n,
                           (const int32_t *)nullptr, &hdr->n_u, hdr, (int)CAP_ROWA);
        hipLaunchKernelGGL(level_major_kernel, dim3(1), dim3(kPlanThreads), 0, st, p->c1, p->statsA[3],
                           (const int32_t *)nullptr, d, (const int32_t *)nullptr, p->sh, p->tmpL, p->tmpCur,
                           &hdr->d1, hdr, (int)CAP_C1);
    } else {
        hipLaunchKernelGGL(identity_slots_kernel, dim3(grid_for(n, 256, 64)), dim3(256), 0, st, p->rowA, n,
                           (const int32_t *)nullptr, &hdr->n_u, hdr, (int)CAP_ROWA);
        hipLaunchKernelGGL(identity_slots_kernel, dim3(grid_for(d, 256, 64)), dim3(256), 0, st, p->c1, d,
                           (const int32_t *)nullptr, &hdr->d1, hdr, (int)CAP_C1);
        hipLaunchKernelGGL(coo_extract_kernel, dim3(grid_for((int64_t)n * ((d + 63) / 64) * 64, 256, 4096)),
                           dim3(256), 0, st, A, (int64_t)n, (int64_t)d, lda, p->s, p->eR, p->eC, p->eV,
                           p->cap[CAP_EDGEA], &hdr->edgesA, hdr);
        IMU_TRY(run_greedy(p, 1, st));
    }
    // ---- phase 2: Unpack(B_e, A_u, S_u, b, strategy_B); B_e has d1 columns
    if (p->sB == IMUNPACK_ROW) {
        hipLaunchKernelGGL(level_major_kernel, dim3(1), dim3(kPlanThreads), 0, st, p->rowB, p->statsB[2],
                           (const int32_t *)nullptr, h, (const int32_t *)nullptr, p->sh, p->tmpL, p->tmpCur,
                           &hdr->h_u, hdr, (int)CAP_ROWB);
        hipLaunchKernelGGL(identity_slots_kernel, dim3(grid_for(p->cap[CAP_C2], 256, 64)), dim3(256), 0, st,
                           p->c2, 0, (const int32_t *)&hdr->d1, &hdr->d_u, hdr, (int)CAP_C2);
    } else if (p->sB == IMUNPACK_COL) {
        hipLaunchKernelGGL(identity_slots_kernel, dim3(grid_for(h, 256, 64)), dim3(256), 0, st, p->rowB, h,
                           (const int32_t *)nullptr, &hdr->h_u, hdr, (int)CAP_ROWB);
        hipLaunchKernelGGL(level_major_kernel, dim3(1), dim3(kPlanThreads), 0, st, p->c2, p->statsB[3],
                           (const int32_t *)p->c1.root, 0, (const int32_t *)&hdr->d1, p->sh, p->tmpL,
                           p->tmpCur, &hdr->d_u, hdr, (int)CAP_C2);
    } else {
        hipLaunchKernelGGL(identity_slots_kernel, dim3(grid_for(h, 256, 64)), dim3(256), 0, st, p->rowB, h,
                           (const int32_t *)nullptr, &hdr->h_u, hdr, (int)CAP_ROWB);
        hipLaunchKernelGGL(identity_slots_kernel, dim3(grid_for(p->cap[CAP_C2], 256, 64)), dim3(256), 0, st,
                           p->c2, 0, (const int32_t *)&hdr->d1, &hdr->d_u, hdr, (int)CAP_C2);
        hipLaunchKernelGGL(coo_extract_kernel, dim3(grid_for((int64_t)h * ((d + 63) / 64) * 64, 256, 4096)),
                           dim3(256), 0, st, B, (int64_t)h, (int64_t)d, ldb, p->s, p->rawJ, p->rawK, p->rawV,
                           p->cap[CAP_RAWB], &hdr->rawB, hdr);
        hipLaunchKernelGGL(check_count_kernel, dim3(1), dim3(64), 0, st, &hdr->rawB, p->cap[CAP_RAWB], hdr,
                           (int)CAP_RAWB);
        hipLaunchKernelGGL(expand_edges_kernel, dim3(grid_for(p->cap[CAP_RAWB], 256, 1024)), dim3(256), 0, st,
                           p->rawJ, p->rawK, p->rawV, &hdr->rawB, p->cap[CAP_RAWB], p->c1, p->eR, p->eC,
                           p->eV, p->cap[CAP_EDGEB], &hdr->edgesB, hdr);
        IMU_TRY(run_greedy(p, 2, st));
    }
    // ---- physical layouts
    hipLaunchKernelGGL(rows_layout_kernel, dim3(1), dim3(kPlanThreads), 0, st, p->rowA, n, &hdr->n_u, p->layA,
                       phys_cap_rows(p->cap[CAP_ROWA]), phys_cap_rows(p->cap[CAP_ROWA]) / kTile + 2, p->tmpL,
                       p->tmpP, hdr, 0);
    hipLaunchKernelGGL(rows_layout_kernel, dim3(1), dim3(kPlanThreads), 0, st, p->rowB, h, &hdr->h_u, p->layB,
                       phys_cap_rows(p->cap[CAP_ROWB]), phys_cap_rows(p->cap[CAP_ROWB]) / kTile + 2, p->tmpL,
                       p->tmpP, hdr, 1);
    hipLaunchKernelGGL(cols_layout_kernel, dim3(1), dim3(kPlanThreads), 0, st, p->c1, p->c2, p->cols,
                       phys_cap_cols(p->cap[CAP_C2]), p->s, p->sh, hdr);
    return launch_status();
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
    }
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
        p->cap[CAP_RAWB] = std::max(p->cap[CAP_RAWB], (int)std::min<int64_t>(h * d, std::max<int64_t>(h * d / 64, 4096)));
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
        if (!ownA) { p->statsA[0] = stats_A->rowcnt; p->statsA[1] = stats_A->colcnt; p->statsA[2] = stats_A->rowmax; p->statsA[3] = stats_A->colmax; }
        if (!ownB) { p->statsB[0] = stats_B->rowcnt; p->statsB[1] = stats_B->colcnt; p->statsB[2] = stats_B->rowmax; p->statsB[3] = stats_B->colmax; }
        rc = enqueue_plan(p, A, lda, B, ldb, ownA, ownB, st);
        if (rc != IMUNPACK_OK) break;
        hipError_t e = hipMemcpyAsync(&p->hdr, p->d_hdr, sizeof(PlanHeader), hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e != hipSuccess) { g_last_hip_error = (int)e; rc = IMUNPACK_EHIP; break; }
        if (p->hdr.err) { rc = p->hdr.err; break; }
        if (!p->hdr.overflow) { p->valid = 1; break; }
        for (int c = 0; c < 8; ++c)
            if (p->hdr.overflow & (1 << c)) {
                int64_t nv = std::max<int64_t>((int64_t)p->hdr.need[c] + p->hdr.need[c] / 8 + 256, (int64_t)p->cap[c] * 2);
                if (nv > (1ll << 30)) { rc = IMUNPACK_ENOMEM; break; }
                p->cap[c] = (int)nv;
            }
        if (rc != IMUNPACK_OK) break;
        rc = IMUNPACK_ENOMEM;  // stays if the attempts run out
    }
    if (rc != IMUNPACK_OK && !p->valid) {
        if (!*plan) { if (p->arena) (void)hipFree(p->arena); delete p; }
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

namespace imu {
__global__ void export_cols_kernel(SlotSet c1, SlotSet c2, int D, int32_t *col_src, int32_t *col_exp) {
    for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < D; c += gridDim.x * blockDim.x) {
        const int root = c2.root[c];
        col_src[c] = c1.root[root];
        col_exp[c] = c1.exp[root] + c2.exp[c];
    }
}
}  // namespace imu

extern "C" int imunpack_plan_export(const imunpack_plan_t *p, int32_t *rowA_src, int32_t *rowA_exp,
                                    int32_t *rowB_src, int32_t *rowB_exp, int32_t *col_src,
                                    int32_t *col_exp) {
    if (!p || !p->valid) return IMUNPACK_EINVAL;
    hipStream_t st = p->stream;
    const size_t nA = (size_t)p->hdr.n_u * 4, nB = (size_t)p->hdr.h_u * 4, nC = (size_t)p->hdr.d_u * 4;
    if (rowA_src) IMU_HIP(hipMemcpyAsync(rowA_src, p->rowA.root, nA, hipMemcpyDeviceToHost, st));
    if (rowA_exp) IMU_HIP(hipMemcpyAsync(rowA_exp, p->rowA.exp, nA, hipMemcpyDeviceToHost, st));
    if (rowB_src) IMU_HIP(hipMemcpyAsync(rowB_src, p->rowB.root, nB, hipMemcpyDeviceToHost, st));
    if (rowB_exp) IMU_HIP(hipMemcpyAsync(rowB_exp, p->rowB.exp, nB, hipMemcpyDeviceToHost, st));
    if (col_src || col_exp) {
        // scratch: the level temporaries are free once planning has finished
        int32_t *t_src = p->tmpL, *t_exp = p->tmpCur;
        hipLaunchKernelGGL(export_cols_kernel, dim3(grid_for(p->hdr.d_u, 256, 256)), dim3(256), 0, st, p->c1,
                           p->c2, p->hdr.d_u, t_src, t_exp);
        IMU_TRY(launch_status());
        if (col_src) IMU_HIP(hipMemcpyAsync(col_src, t_src, nC, hipMemcpyDeviceToHost, st));
        if (col_exp) IMU_HIP(hipMemcpyAsync(col_exp, t_exp, nC, hipMemcpyDeviceToHost, st));
    }
    IMU_HIP(hipStreamSynchronize(st));
    return IMUNPACK_OK;
}

extern "C" int imunpack_plan_destroy(imunpack_plan_t *p) {
    if (!p) return IMUNPACK_OK;
    int rc = IMUNPACK_OK;
    if (p->arena) {
        hipError_t e = hipFree(p->arena);
        if (e != hipSuccess) { g_last_hip_error = (int)e; rc = IMUNPACK_EHIP; }
    }
    delete p;
    return rc;
}
