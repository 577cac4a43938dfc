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
//   mid level   T2_f (16x16) = U2[K_f,:]^T . T1_f       K = the (i,j,k) nodes of fiber f
//   slice level Y_i (16x256) = U1[J_i,:]^T . T2_i       K = the (i,j) fibers of the item
// One wavefront per item, lane = (slot, c), slot = lane/16.  A K-step takes four fibers.  For
// each of them the slots are four nodes of the fiber: lane (s,c) builds T1_node_s[r3 = c] from
// the node's leaves (VALU) and supplies U2[k_s, r2 = c]; one MFMA per four nodes gives T2_f in
// the accumulator layout (register v of lane (s,c) holds T2[r2 = s+4v][r3 = c]).  The four T2
// tiles go through a wave-private LDS buffer so that in the slice-level MFMAs slot s can supply
// the tile of fiber s: B_t = T2_s[r2 = t][r3 = c] for the 16 column tiles t, A = U1[j_s, r1 = c].
// The loads of the four fibers of a K-step are issued stage by stage for all four together
// (node descriptors, then leaf entries + U2, then U3 rows), so a K-step costs about four memory
// round trips instead of four per fiber; the fibers' own descriptors are fetched a step ahead.
typedef double v4d __attribute__((ext_vector_type(4)));
constexpr int kT2Stride = 16 * 16 + 16;        // doubles per fiber tile in LDS (+16: bank skew)

__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 4)))
ttmc4_mfma_kernel(Ttmc4Args a) {
    __shared__ double t2buf[4][4 * kT2Stride];
    const int lane = threadIdx.x % 64, wv = threadIdx.x / 64;
    const int64_t w = uni64(int64_t(blockIdx.x) * 4 + wv);
    if (w >= a.n_items) return;
    const SliceItem it = a.items[w];
    const int32_t s = __builtin_amdgcn_readfirstlane(it.slice);
    const int64_t fa = uni64(it.begin), fb = uni64(it.end), dest = uni64(it.dest);
    const int slot = lane >> 4, c = lane & 15;
    double *lds = t2buf[wv];

    v4d acc[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) acc[t] = v4d{0.0, 0.0, 0.0, 0.0};

    // per-lane view of the K-step's fibers: lane (slot, c) needs fiber g+slot for the A operand,
    // and every lane needs the node range of all four fibers (kept per lane, loaded once)
    auto fiber_desc = [&](int64_t g, int64_t na[4], int64_t nb[4], int32_t &j) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            na[u] = nb[u] = 0;
            if (g + u < fb) { na[u] = a.ptr1[g + u]; nb[u] = a.ptr1[g + u + 1]; }
        }
        j = g + slot < fb ? a.idx1[g + slot] : -1;
    };
    int64_t na[4], nb[4], nna[4], nnb[4];
    int32_t j, nj;
    fiber_desc(fa, nna, nnb, nj);
    for (int64_t g = fa; g < fb; g += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) { na[u] = nna[u]; nb[u] = nnb[u]; }
        j = nj;
        fiber_desc(g + 4, nna, nnb, nj);
        const double av = j >= 0 ? a.U1[int64_t(j) * 16 + c] : 0.0;

        // stage 1: node descriptors of the first four nodes of each fiber
        int32_t k[4];
        int64_t la[4], lb[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t n = na[u] + slot;
            k[u] = -1;
            la[u] = lb[u] = 0;
            if (n < nb[u]) { k[u] = a.idx2[n]; la[u] = a.ptr2[n]; lb[u] = a.ptr2[n + 1]; }
        }
        // stage 2: U2 row entry, first two leaves of each node
        double u2[4], v0[4], v1[4];
        int32_t l0[4], l1[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            u2[u] = k[u] >= 0 ? a.U2[int64_t(k[u]) * 16 + c] : 0.0;
            l0[u] = l1[u] = -1;
            v0[u] = v1[u] = 0.0;
            if (la[u] < lb[u]) { l0[u] = a.idx3[la[u]]; v0[u] = a.vals[la[u]]; }
            if (la[u] + 1 < lb[u]) { l1[u] = a.idx3[la[u] + 1]; v1[u] = a.vals[la[u] + 1]; }
        }
        // stage 3: U3 rows
        double x0[4], x1[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            x0[u] = l0[u] >= 0 ? a.U3[int64_t(l0[u]) * 16 + c] : 0.0;
            x1[u] = l1[u] >= 0 ? a.U3[int64_t(l1[u]) * 16 + c] : 0.0;
        }
        // stage 4: T1, mid-level MFMA, remainders (nodes with > 2 leaves, fibers with > 4 nodes)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            double t1 = fma(v1[u], x1[u], v0[u] * x0[u]);
            for (int64_t e = la[u] + 2; e < lb[u]; ++e)
                t1 = fma(a.vals[e], a.U3[int64_t(a.idx3[e]) * 16 + c], t1);
            v4d t2 = __builtin_amdgcn_mfma_f64_16x16x4f64(u2[u], t1, v4d{0.0, 0.0, 0.0, 0.0}, 0, 0, 0);
            for (int64_t n0 = na[u] + 4; n0 < nb[u]; n0 += 4) {          // wave-uniform bounds
                const int64_t n = n0 + slot;
                double uu = 0.0, tt = 0.0;
                if (n < nb[u]) {
                    uu = a.U2[int64_t(a.idx2[n]) * 16 + c];
                    for (int64_t e = a.ptr2[n]; e < a.ptr2[n + 1]; ++e)
                        tt = fma(a.vals[e], a.U3[int64_t(a.idx3[e]) * 16 + c], tt);
                }
                t2 = __builtin_amdgcn_mfma_f64_16x16x4f64(uu, tt, t2, 0, 0, 0);
            }
            // accumulator layout -> LDS tile of fiber u: element (r2 = slot + 4v, r3 = c)
#pragma unroll
            for (int v = 0; v < 4; ++v) lds[u * kT2Stride + (slot + 4 * v) * 16 + c] = t2[v];
        }
        // slice level: slot s supplies fiber s; 16 column tiles t = r2
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const double bv = lds[slot * kT2Stride + t * 16 + c];
            acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc[t], 0, 0, 0);
        }
    }
    const int64_t RR = 4096;
    double *base = dest < 0 ? a.out + (a.compact ? int64_t(s) : int64_t(a.idx0[s])) * RR
                            : a.partial + dest * RR;
    // acc[t][v] = Y[r1 = slot + 4v][r2 = t][r3 = c]
#pragma unroll
    for (int t = 0; t < 16; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) base[((slot + 4 * v) * 16 + t) * 16 + c] = acc[t][v];
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
        if (a.R1 == 16 && a.R2 == 16 && a.R3 == 16 && env_int("CONSTSTN_TTMC4_NO_MFMA", 0) == 0)
            ttmc4_mfma_kernel<<<dim3(unsigned(div_up(a.n_items, 4))), dim3(256), 0, stream>>>(a);
        else
            ttmc4_kernel<<<dim3(unsigned(div_up(a.n_items, 4))), dim3(256), 0, stream>>>(a);
    }
    CST_HIP(hipGetLastError());
    return launch_ttmc_fixup(plan, out, stream);
}

}  // namespace cst
