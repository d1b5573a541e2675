// Digit scatter (Sec. 4, Eq. (mod); Alg. 1 l.4-5, Alg. 2 l.4-6, Alg. 4 l.7-8 and 11-13): writes the
// unpacked int8 operands A_ue and B_eu in the plan's physical layout, gathering from the int32
// operands.  HBM-bound: 4 B read per source element, 1 B written per unpacked element.
//
// Where an entry's digits go.  A split of a row (column) keeps digit 0 of every entry of that row
// (column) in place and moves floor(v / s) to the appended row (column); a row or column is split
// at most once.  So the digits of the original entry (i, k) lie on a chain of positions: the
// remainder sitting at (R, C) moves to the child of R if R was split before C, to the child of C
// otherwise, and every other descendant position holds 0.  Position (R, C) with row level eR and
// column level eC therefore holds digit eR + eC of the entry if the chain passes through it, else 0.
#include "common.h"

namespace imu {

// sign(v) * ((|v| >> (sh * t)) & (s - 1)); a shift of 32 or more gives 0
__device__ __forceinline__ int digit_of(int32_t v, int t, int sh, int s) {
    const unsigned sft = (unsigned)(sh * t);
    if (sft >= 32u) return 0;
    const unsigned av = v < 0 ? 0u - (unsigned)v : (unsigned)v;
    const int dg = (int)((av >> sft) & (unsigned)(s - 1));
    return v < 0 ? -dg : dg;
}

// Does the chain of the entry at (row root, column root) pass through (level er, level ec)?
__device__ __forceinline__ bool on_chain(const SlotSet &rows, const SlotSet &cols, int rroot, int croot,
                                         int er, int ec) {
    int r = rroot, c = croot, a = 0, b = 0;
    while (a < er || b < ec) {
        const uint32_t tr = rows.time[r], tc = cols.time[c];
        if (tr < tc) {
            if (a == er) return false;
            r = rows.child[r];
            ++a;
        } else {
            if (b == ec || tc == kNever) return false;
            c = cols.child[c];
            ++b;
        }
    }
    return true;
}

// One workgroup handles kScatterRows consecutive physical rows over the whole padded width, 16 output
// bytes per thread and step, so that the column descriptors are fetched once per row block, the
// source rows (all digit levels of a source row are adjacent) are read from HBM once, and stores are
// 16 bytes wide.  OPERAND 0 writes A_ue: rows from Pi_A, column chain inside the unpacking of A, then
// copied along the columns that unpacking B appended.  OPERAND 1 writes B_eu: rows from Pi_B, column
// chain inside the unpacking of B_e, whose column c copies B[:, k(c)].
constexpr int kScatterRows = 8;

template <int OPERAND>
__global__ __launch_bounds__(256) void scatter_kernel(const int32_t *__restrict__ M, int64_t ld,
                                                      RowLayout lay, ColLayout cols, SlotSet rows,
                                                      SlotSet cset, int Mp, int Kp, int s, int sh,
                                                      int8_t *__restrict__ out,
                                                      unsigned long long *bound) {
    __shared__ unsigned long long red[4][kScatterRows];
    const int p0 = blockIdx.x * kScatterRows;
    int slotR[kScatterRows], srcI[kScatterRows], expR[kScatterRows];
#pragma unroll
    for (int r = 0; r < kScatterRows; ++r) {
        const int p = p0 + r;
        slotR[r] = p < Mp ? lay.prow_slot[p] : -2;
        srcI[r] = p < Mp ? lay.prow_src[p] : 0;
        expR[r] = p < Mp ? lay.prow_exp[p] : 0;
    }
    unsigned long long wsum[kScatterRows];
#pragma unroll
    for (int r = 0; r < kScatterRows; ++r) wsum[r] = 0;
    const bool ld_vec = (ld % 4) == 0 && ((uintptr_t)M % 16) == 0;
    for (int q0 = threadIdx.x * 16; q0 < Kp; q0 += 256 * 16) {
        int k[16], ec[16], sx[16];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int4 kk = *reinterpret_cast<const int4 *>(cols.colA_k + q0 + 4 * u);
            const int4 ee = *reinterpret_cast<const int4 *>((OPERAND == 0 ? cols.colA_e : cols.colB_e) + q0 + 4 * u);
            const int4 ss = *reinterpret_cast<const int4 *>(cols.col_sexp + q0 + 4 * u);
            k[4 * u] = kk.x; k[4 * u + 1] = kk.y; k[4 * u + 2] = kk.z; k[4 * u + 3] = kk.w;
            ec[4 * u] = ee.x; ec[4 * u + 1] = ee.y; ec[4 * u + 2] = ee.z; ec[4 * u + 3] = ee.w;
            sx[4 * u] = ss.x; sx[4 * u + 1] = ss.y; sx[4 * u + 2] = ss.z; sx[4 * u + 3] = ss.w;
        }
        bool run = k[0] >= 0 && (k[0] % 4) == 0 && ld_vec;  // 16 consecutive source columns?
        int ecany = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            run = run && k[j] == k[0] + j;
            ecany |= ec[j];
        }
#pragma unroll
        for (int r = 0; r < kScatterRows; ++r) {
            if (slotR[r] == -2) continue;  // past the last physical row (uniform)
            int4 *dst = reinterpret_cast<int4 *>(out + (int64_t)(p0 + r) * Kp + q0);
            if (slotR[r] < 0) {  // padding row
                *dst = make_int4(0, 0, 0, 0);
                continue;
            }
            const int32_t *src = M + (int64_t)srcI[r] * ld;
            int32_t v[16];
            if (run) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int4 x = *reinterpret_cast<const int4 *>(src + k[0] + 4 * u);
                    v[4 * u] = x.x; v[4 * u + 1] = x.y; v[4 * u + 2] = x.z; v[4 * u + 3] = x.w;
                }
            } else {
#pragma unroll
                for (int j = 0; j < 16; ++j) v[j] = k[j] >= 0 ? src[k[j]] : 0;
            }
            int dg[16];
            const int er = expR[r];
            if (er == 0 && ecany == 0) {  // the common case: digit 0 of every entry
#pragma unroll
                for (int j = 0; j < 16; ++j) dg[j] = digit_of(v[j], 0, sh, s);
            } else {
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int t = er + ec[j];
                    int val = digit_of(v[j], t, sh, s);
                    if (t != 0 && val != 0) {
                        const int croot = OPERAND == 0 ? k[j] : cols.colA_c1[q0 + j];
                        if (!on_chain(rows, cset, srcI[r], croot, er, ec[j])) val = 0;
                    }
                    dg[j] = val;
                }
            }
            int pk[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                pk[u] = (dg[4 * u] & 0xFF) | ((dg[4 * u + 1] & 0xFF) << 8) | ((dg[4 * u + 2] & 0xFF) << 16) |
                        ((dg[4 * u + 3] & 0xFF) << 24);
            *dst = make_int4(pk[0], pk[1], pk[2], pk[3]);
            // weighted L1 norm of the row (saturating): sum_c s^e(c) |digit|
            unsigned long long acc = 0;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const unsigned sft = (unsigned)(sh * sx[j]);
                const unsigned long long mag = (unsigned long long)(dg[j] < 0 ? -dg[j] : dg[j]);
                acc += (mag == 0) ? 0ull : (sft >= 40u ? (1ull << 50) : (mag << sft));
            }
            wsum[r] += acc;
            if (wsum[r] > (1ull << 52)) wsum[r] = 1ull << 52;
        }
    }
    // largest row norm of this block -> global maximum
#pragma unroll
    for (int r = 0; r < kScatterRows; ++r) {
        unsigned long long w = wsum[r];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) w += __shfl_xor(w, off, 64);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6][r] = w;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long best = 0;
        for (int r = 0; r < kScatterRows; ++r) {
            unsigned long long t = red[0][r] + red[1][r] + red[2][r] + red[3][r];
            if (t > (1ull << 60)) t = 1ull << 60;
            best = best > t ? best : t;
        }
        if (best) atomicMax(bound, best);
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
    hipLaunchKernelGGL(reset_bound_kernel, dim3(1), dim3(64), 0, st, p->d_hdr);
    if (h.Mp > 0 && h.Kp > 0)
        hipLaunchKernelGGL(scatter_kernel<0>, dim3((h.Mp + kScatterRows - 1) / kScatterRows), dim3(256), 0, st, A,
                           lda, p->layA, p->cols, p->rowA, p->c1, h.Mp, h.Kp, p->s, p->sh, A_ue,
                           &p->d_hdr->bound[0]);
    if (h.Np > 0 && h.Kp > 0)
        hipLaunchKernelGGL(scatter_kernel<1>, dim3((h.Np + kScatterRows - 1) / kScatterRows), dim3(256), 0, st, B,
                           ldb, p->layB, p->cols, p->rowB, p->c2, h.Np, h.Kp, p->s, p->sh, B_eu,
                           &p->d_hdr->bound[1]);
    IMU_TRY(launch_status());
    IMU_HIP(hipMemcpyAsync(p->hdr.bound, p->d_hdr->bound, sizeof(p->hdr.bound), hipMemcpyDeviceToHost, st));
    IMU_HIP(hipStreamSynchronize(st));
    // |sum_c s^e(c) a_c b_c| <= (s - 1) * min(bound_A, bound_B): the shifted sum of all groups
    // fits int32 iff that is below 2^31.
    const unsigned long long m = p->hdr.bound[0] < p->hdr.bound[1] ? p->hdr.bound[0] : p->hdr.bound[1];
    p->fusable = (m < (1ull << 40)) && (m * (unsigned long long)(p->s - 1) < (1ull << 31));
    p->unpacked = 1;
    return IMUNPACK_OK;
}

extern "C" int imunpack_plan_fusable(const imunpack_plan_t *p) {
    if (!p || !p->valid || !p->unpacked) return 0;
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
