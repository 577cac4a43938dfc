// Fused three-tensor network of Sec. 1:  Z[i,m] = sum_{j,k,l} U[i,j,k] V[j,l] W[k,l,m]
// evaluated as the tree (U.V).W:
//     T[i,k,l] = U[i,k,j] V[j,l]   loops i,k,j,l      (U stored i>k>j)
//     Z[i,m]   = T[i,k,l] W[k,l,m] loops i,k,l,m      (W stored k>l>m)
// fused on the loops i and k, so T shrinks to one length-L vector per (i,k) fiber of U and no
// full intermediate is formed.
//
// Baseline kernel: one workgroup per root slice i of U.  For each (i,k) fiber the threads
// build T[0..L) in LDS (thread = l, coalesced rows of V), then the wavefronts walk the (k,l)
// fibers of W below root k: lanes take the m leaves and add T[l]*W into a per-wavefront copy
// of Z_i in LDS (no atomics: leaves of one fiber have distinct m).  The copies are added in
// fixed order at the end, so results are bit-reproducible.
#include "plan.hpp"

namespace cst {

struct Sptn3Args {
    int64_t slices;
    int64_t L, M;
    const int64_t *uptr0, *uptr1;
    const int32_t *uidx0, *uidx1, *uidx2;
    const double *uvals;
    const int64_t *wptr0, *wptr1;
    const int32_t *widx1, *widx2;
    const double *wvals;
    const int64_t *w_root_of_k;
    const double *V;
    double *out;
    int compact;
};

__global__ void __launch_bounds__(256)
sptn3_kernel(Sptn3Args a) {
    extern __shared__ double lds[];
    double *T = lds;                         // L
    double *Zw = lds + a.L;                  // 4 x M
    const int64_t s = blockIdx.x;
    const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64;
    const int64_t L = a.L, M = a.M;
    for (int64_t e = tid; e < 4 * M; e += 256) Zw[e] = 0.0;
    const int64_t fa = a.uptr0[s], fb = a.uptr0[s + 1];
    for (int64_t f = fa; f < fb; ++f) {
        const int32_t k = a.uidx1[f];
        const int64_t root = a.w_root_of_k[k];
        if (root < 0) continue;                                   // W has nothing at this k
        const int64_t na = a.uptr1[f], nb = a.uptr1[f + 1];
        __syncthreads();                                          // T free for reuse
        for (int64_t l = tid; l < L; l += 256) {
            double t = 0.0;
            for (int64_t n = na; n < nb; ++n)
                t = fma(a.uvals[n], a.V[int64_t(a.uidx2[n]) * L + l], t);
            T[l] = t;
        }
        __syncthreads();
        const int64_t ga = a.wptr0[root], gb = a.wptr0[root + 1];
        double *Z = Zw + int64_t(wave) * M;
        for (int64_t g = ga + wave; g < gb; g += 4) {
            const double tl = T[a.widx1[g]];
            const int64_t ea = a.wptr1[g], eb = a.wptr1[g + 1];
            for (int64_t e = ea + lane; e < eb; e += 64) {
                const int32_t m = a.widx2[e];
                Z[m] = fma(tl, a.wvals[e], Z[m]);
            }
        }
    }
    __syncthreads();
    const int64_t row = a.compact ? s : int64_t(a.uidx0[s]);
    for (int64_t m = tid; m < M; m += 256)
        a.out[row * M + m] = ((Zw[m] + Zw[M + m]) + Zw[2 * M + m]) + Zw[3 * M + m];
}

conststn_status launch_sptn3(const conststn_plan_s *plan, const double *const *dense, double *out,
                             hipStream_t stream) {
    const conststn_csf_s *U = plan->X, *W = plan->W;
    Sptn3Args a{};
    a.slices = U->nodes[0];
    a.L = W->dims[W->mode_order[1]];
    a.M = W->dims[W->mode_order[2]];
    a.uptr0 = U->ptr[0].p;
    a.uptr1 = U->ptr[1].p;
    a.uidx0 = U->idx[0].p;
    a.uidx1 = U->idx[1].p;
    a.uidx2 = U->idx[2].p;
    a.uvals = U->vals.p;
    a.wptr0 = W->ptr[0].p;
    a.wptr1 = W->ptr[1].p;
    a.widx1 = W->idx[1].p;
    a.widx2 = W->idx[2].p;
    a.wvals = W->vals.p;
    a.w_root_of_k = plan->w_root_of_k.p;
    a.V = dense[0];
    a.out = out;
    a.compact = plan->compact ? 1 : 0;
    const size_t lds_bytes = size_t(a.L + 4 * a.M) * sizeof(double);
    if (lds_bytes > 64 * 1024) {
        set_error("three-tensor kernel needs %zu bytes of LDS (L=%lld, M=%lld); at most 65536 implemented",
                  lds_bytes, (long long)a.L, (long long)a.M);
        return CONSTSTN_EUNSUPPORTED;
    }
    if (!plan->compact && a.slices < plan->out_rows)
        CST_TRY(zero_fill(out, plan->out_rows * plan->row_elems, stream));
    if (a.slices == 0) return CONSTSTN_OK;
    {
        ProfScope prof(plan, stream);
        sptn3_kernel<<<dim3(unsigned(a.slices)), dim3(256), lds_bytes, stream>>>(a);
    }
    CST_HIP(hipGetLastError());
    return CONSTSTN_OK;
}

}  // namespace cst
