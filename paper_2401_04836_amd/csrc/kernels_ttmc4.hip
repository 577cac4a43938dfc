// Fused order-4 TTMc over a CSF tensor (order-4 form of Sec. 5.3):
//     Y[i,r1,r2,r3] = sum_{j,k,l} X[i,j,k,l] U1[j,r1] U2[k,r2] U3[l,r3]
// as the three-statement tree
//     T1[i,j,k,r3] = X U3 ;  T2[i,j,r2,r3] = T1 U2 ;  Y[i,r1,r2,r3] = T2 U1
// fused on (i,j,k) and (i,j): T1 shrinks to a length-R3 vector per (i,j,k) node and T2 to an
// R2 x R3 matrix per (i,j) fiber -- the largest intermediate is order 2 (the l = 2 solution
// of Sec. 3).
//
// General kernel, ranks up to 16: one wavefront per work item (a range of (i,j) fibers of one
// slice).  Lane = (q, r3) with q = lane/16: the four lane rows split the leaves of a node for
// T1 (then an xor-shuffle sum), and row q holds T2[r2, r3] for r2 = q, q+4, q+8, q+12 and the
// matching 16 x 4 part of Y_i in registers.
#include "plan.hpp"

namespace cst {

struct Ttmc4Args {
    int64_t n_items;
    int R1, R2, R3;
    const int64_t *ptr1, *ptr2;
    const int32_t *idx0, *idx1, *idx2, *idx3;
    const double *vals;
    const SliceItem *items;
    const double *U1, *U2, *U3;
    double *out, *partial;
    int compact;
};

__device__ __forceinline__ int64_t uni64(int64_t v) {
    const int lo = __builtin_amdgcn_readfirstlane(int(v & 0xffffffffll));
    const int hi = __builtin_amdgcn_readfirstlane(int(v >> 32));
    return (int64_t(hi) << 32) | int64_t(uint32_t(lo));
}

__global__ void __launch_bounds__(256)
ttmc4_kernel(Ttmc4Args a) {
    const int lane = threadIdx.x % 64;
    const int64_t w = uni64(int64_t(blockIdx.x) * 4 + threadIdx.x / 64);
    if (w >= a.n_items) return;
    const SliceItem it = a.items[w];
    const int32_t s = __builtin_amdgcn_readfirstlane(it.slice);
    const int64_t fa = uni64(it.begin), fb = uni64(it.end), dest = uni64(it.dest);
    const int R1 = a.R1, R2 = a.R2, R3 = a.R3;
    const int q = lane / 16, c3 = lane % 16;
    const bool col_ok = c3 < R3;
    const int col = col_ok ? c3 : 0;

    double y[16][4];
#pragma unroll
    for (int r = 0; r < 16; ++r)
#pragma unroll
        for (int t = 0; t < 4; ++t) y[r][t] = 0.0;

    for (int64_t f = fa; f < fb; ++f) {
        const int32_t j = __builtin_amdgcn_readfirstlane(a.idx1[f]);
        const int64_t ga = uni64(a.ptr1[f]), gb = uni64(a.ptr1[f + 1]);
        double t2[4] = {0.0, 0.0, 0.0, 0.0};
        for (int64_t g = ga; g < gb; ++g) {
            const int32_t k = __builtin_amdgcn_readfirstlane(a.idx2[g]);
            const int64_t la = uni64(a.ptr2[g]), lb = uni64(a.ptr2[g + 1]);
            double t1 = 0.0;
            for (int64_t n = la; n < lb; n += 4) {
                const int64_t m = n + q;
                if (m < lb) {
                    const int32_t l = a.idx3[m];
                    t1 = fma(a.vals[m], a.U3[int64_t(l) * R3 + col], t1);
                }
            }
            t1 += __shfl_xor(t1, 16, 64);
            t1 += __shfl_xor(t1, 32, 64);
            const double *u2 = a.U2 + int64_t(k) * R2;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int r2 = q + 4 * t;
                if (r2 < R2) t2[t] = fma(u2[r2], t1, t2[t]);
            }
        }
        const double *u1 = a.U1 + int64_t(j) * R1;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (r < R1) {
                const double u = u1[r];
#pragma unroll
                for (int t = 0; t < 4; ++t) y[r][t] = fma(u, t2[t], y[r][t]);
            }
        }
    }
    const int64_t RR = int64_t(R1) * R2 * R3;
    double *base = dest < 0 ? a.out + (a.compact ? int64_t(s) : int64_t(a.idx0[s])) * RR
                            : a.partial + dest * RR;
    if (col_ok) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (r < R1) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int r2 = q + 4 * t;
                    if (r2 < R2) base[(int64_t(r) * R2 + r2) * R3 + c3] = y[r][t];
                }
            }
        }
    }
}

// ---- MFMA kernel (all three ranks equal to 16) ----------------------------------------------
//
// Both dense stages run on the fp64 matrix cores (v_mfma_f64_16x16x4, K = 4):
//   mid level   T2 (16x16) = U2[K,:]^T . T1        K = four "pieces" of (i,j,k) nodes
//   slice level Y_i (16x256) = U1[J,:]^T . T2      K = four "rows" of (i,j) fibers
// The plan cuts every node into pieces of at most two leaves and every fiber into rows of at most
// four pieces (partition.hip); a long node or fiber simply contributes several K entries with the
// same factor row, which is legal by distributivity.  Every K-step therefore does the same,
// loop-free amount of work whatever the skew of the tensor.
// One wavefront per item (a range of rows of one slice), lane = (slot, c), slot = lane/16.
// A K-step takes four rows.  For each of them the slots are the row's four pieces: lane (s,c)
// builds T1_piece_s[r3 = c] from at most two leaves and supplies U2[k_s, r2 = c]; one MFMA gives
// the row's T2 in the accumulator layout (register v of lane (s,c) = T2[r2 = s+4v][r3 = c]).  The
// four T2 tiles pass through a wave-private LDS buffer so that in the slice-level MFMAs slot s
// supplies the tile of row s: B_t = T2_s[r2 = t][r3 = c] for the 16 column tiles, A = U1[j_s, c].
// The plan copies each piece's level-2 index, leaf indices and leaf values into one 32-byte record;
// row ranges are fetched two K-steps ahead and piece records one ahead, so a K-step waits for one
// memory round trip (the factor rows) and issues 21 vector loads.
typedef double v4d __attribute__((ext_vector_type(4)));
constexpr int kT2Stride = 16 * 16 + 16;        // doubles per tile in LDS (+16: bank skew)

struct Ttmc4RowArgs {
    int64_t n_items;
    const int64_t *row_piece;
    const PieceDesc *pieces;
    const int32_t *row_j;
    const int32_t *idx0, *idx3;
    const double *vals;
    const SliceItem *items;
    const double *U1, *U2, *U3;
    double *out, *partial;
    int compact;
};

// PARTS waves share an item, each owning 16/PARTS of the column tiles (fewer accumulator
// registers, more resident waves; the cheap mid level is repeated by every part).
template <int PARTS>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(PARTS == 1 ? 2 : (PARTS == 2 ? 3 : 5), 8)))
ttmc4_mfma_kernel(Ttmc4RowArgs a) {
    constexpr int TN = 16 / PARTS;
    __shared__ double t2buf[4][4 * kT2Stride];
    const int lane = threadIdx.x % 64, wv = threadIdx.x / 64;
    const int part = int(blockIdx.x % unsigned(PARTS));
    const int64_t w = uni64(int64_t(blockIdx.x / unsigned(PARTS)) * 4 + wv);
    if (w >= a.n_items) return;
    const SliceItem it = a.items[w];
    const int32_t s = __builtin_amdgcn_readfirstlane(it.slice);
    const int64_t ra = uni64(it.begin), rb = uni64(it.end), dest = uni64(it.dest);
    const int slot = lane >> 4, c = lane & 15;
    double *lds = t2buf[wv];

    v4d acc[TN];
#pragma unroll
    for (int t = 0; t < TN; ++t) acc[t] = v4d{0.0, 0.0, 0.0, 0.0};

    // row descriptors of a K-step: piece ranges of its four rows (every lane), j of row g+slot
    struct Rows { int64_t pa[4]; int pn[4]; int32_t j; };
    auto load_rows = [&](int64_t g) -> Rows {
        Rows r;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            r.pa[u] = 0;
            r.pn[u] = 0;
            if (g + u < rb) { r.pa[u] = a.row_piece[g + u]; r.pn[u] = int(a.row_piece[g + u + 1] - r.pa[u]); }
        }
        r.j = g + slot < rb ? a.row_j[g + slot] : -1;
        return r;
    };
    // pieces: piece pa[u]+slot of each row -- level-2 index, leaf indices and leaf values in one read
    struct Pieces { int32_t k[4], l0[4], l1[4]; double v0[4], v1[4]; int32_t j; };
    auto load_pieces = [&](const Rows &r) -> Pieces {
        Pieces p;
        p.j = r.j;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            p.k[u] = p.l0[u] = p.l1[u] = -1;
            p.v0[u] = p.v1[u] = 0.0;
            if (slot < r.pn[u]) {
                const PieceDesc d = a.pieces[r.pa[u] + slot];
                p.k[u] = d.k;
                p.l0[u] = d.l0;
                p.l1[u] = d.l1;
                p.v0[u] = d.v0;
                p.v1[u] = d.v1;
            }
        }
        return p;
    };
    Rows r2 = load_rows(ra);
    Pieces cur = load_pieces(r2);
    r2 = load_rows(ra + 4);
    for (int64_t g = ra; g < rb; g += 4) {
        const Pieces nxt = load_pieces(r2);              // K-step g+4
        r2 = load_rows(g + 8);
        const double av = cur.j >= 0 ? a.U1[int64_t(cur.j) * 16 + c] : 0.0;
        // factor rows: U2 entry of each piece, U3 rows of its (at most two) leaves
        double u2[4], x0[4], x1[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            u2[u] = cur.k[u] >= 0 ? a.U2[int64_t(cur.k[u]) * 16 + c] : 0.0;
            x0[u] = cur.l0[u] >= 0 ? a.U3[int64_t(cur.l0[u]) * 16 + c] : 0.0;
            x1[u] = cur.l1[u] >= 0 ? a.U3[int64_t(cur.l1[u]) * 16 + c] : 0.0;
        }
        // mid level
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const double t1 = fma(cur.v1[u], x1[u], cur.v0[u] * x0[u]);
            const v4d t2 = __builtin_amdgcn_mfma_f64_16x16x4f64(u2[u], t1, v4d{0.0, 0.0, 0.0, 0.0}, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 4; ++v) lds[u * kT2Stride + (slot + 4 * v) * 16 + c] = t2[v];
        }
        // slice level: slot s supplies row s; 16 column tiles t = r2
#pragma unroll
        for (int t = 0; t < TN; ++t) {
            const double bv = lds[slot * kT2Stride + (part * TN + t) * 16 + c];
            acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc[t], 0, 0, 0);
        }
        cur = nxt;
    }
    const int64_t RR = 4096;
    double *base = dest < 0 ? a.out + (a.compact ? int64_t(s) : int64_t(a.idx0[s])) * RR
                            : a.partial + dest * RR;
    // acc[t][v] = Y[r1 = slot + 4v][r2 = part*TN + t][r3 = c]
#pragma unroll
    for (int t = 0; t < TN; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) base[((slot + 4 * v) * 16 + part * TN + t) * 16 + c] = acc[t][v];
}

conststn_status launch_ttmc4(const conststn_plan_s *plan, const double *const *dense, double *out,
                             hipStream_t stream) {
    const conststn_csf_s *X = plan->X;
    Ttmc4Args a{};
    a.n_items = plan->n_items;
    a.R1 = plan->rank_of_level[1];
    a.R2 = plan->rank_of_level[2];
    a.R3 = plan->rank_of_level[3];
    a.ptr1 = X->ptr[1].p;
    a.ptr2 = X->ptr[2].p;
    a.idx0 = X->idx[0].p;
    a.idx1 = X->idx[1].p;
    a.idx2 = X->idx[2].p;
    a.idx3 = X->idx[3].p;
    a.vals = X->vals.p;
    a.items = plan->items.p;
    a.U1 = dense[plan->factor_of_level[1]];
    a.U2 = dense[plan->factor_of_level[2]];
    a.U3 = dense[plan->factor_of_level[3]];
    a.out = out;
    a.partial = plan->partial.p;
    a.compact = plan->compact ? 1 : 0;
    if (a.R1 > 16 || a.R2 > 16 || a.R3 > 16) {
        set_error("order-4 TTMc ranks above 16 are not implemented");
        return CONSTSTN_EUNSUPPORTED;
    }
    if (!plan->compact && X->nodes[0] < plan->out_rows)
        CST_TRY(zero_fill(out, plan->out_rows * plan->row_elems, stream));
    if (a.n_items == 0) return CONSTSTN_OK;
    {
        ProfScope prof(plan, stream);
        if (plan->use_rows) {
            Ttmc4RowArgs ra{};
            ra.n_items = plan->n_items;
            ra.row_piece = plan->row_piece.p;
            ra.pieces = plan->pieces.p;
            ra.row_j = plan->row_j.p;
            ra.idx0 = a.idx0;
            ra.idx3 = a.idx3;
            ra.vals = a.vals;
            ra.items = a.items;
            ra.U1 = a.U1;
            ra.U2 = a.U2;
            ra.U3 = a.U3;
            ra.out = out;
            ra.partial = a.partial;
            ra.compact = a.compact;
            const int64_t groups = div_up(a.n_items, 4);
            const int64_t parts = env_int("CONSTSTN_TTMC4_PARTS", 1);
            if (parts == 4)
                ttmc4_mfma_kernel<4><<<dim3(unsigned(groups * 4)), dim3(256), 0, stream>>>(ra);
            else if (parts == 2)
                ttmc4_mfma_kernel<2><<<dim3(unsigned(groups * 2)), dim3(256), 0, stream>>>(ra);
            else
                ttmc4_mfma_kernel<1><<<dim3(unsigned(groups)), dim3(256), 0, stream>>>(ra);
        } else
            ttmc4_kernel<<<dim3(unsigned(div_up(a.n_items, 4))), dim3(256), 0, stream>>>(a);
    }
    CST_HIP(hipGetLastError());
    return launch_ttmc_fixup(plan, out, stream);
}

}  // namespace cst
