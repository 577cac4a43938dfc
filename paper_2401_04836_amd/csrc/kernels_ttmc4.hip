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
        ttmc4_kernel<<<dim3(unsigned(div_up(a.n_items, 4))), dim3(256), 0, stream>>>(a);
    }
    CST_HIP(hipGetLastError());
    return launch_ttmc_fixup(plan, out, stream);
}

}  // namespace cst
