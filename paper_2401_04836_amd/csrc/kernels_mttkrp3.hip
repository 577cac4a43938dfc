// Fused order-3 MTTKRP over a CSF tensor (Sec. 5.2):  M[i,r] = sum_{j,k} X[i,j,k] B[j,r] C[k,r].
//
// The schedule is the two-statement tree  T[i,j,r] = X[i,j,k] C[k,r] ; M[i,r] = T[i,j,r] B[j,r]
// fused on the loops i and j, so the intermediate shrinks to one length-R vector per (i,j)
// fiber (the reduced-order dense workspace of Fig. 3b); r is a batch index.
//
// Mapping: the leaf array is cut into equal chunks (partition.hip).  A group of LPR lanes
// owns one chunk and walks it leaf by leaf; each lane keeps two rank entries of the fiber
// vector T and of the slice accumulator in registers.  At a fiber end the group folds
// T * B[j,:] into the accumulator; at a slice end it stores the row (slice wholly inside the
// chunk) or a partial row (slice shared with neighbouring chunks).  A second kernel adds the
// partial rows of shared slices in chunk order, so results are bit-reproducible.
#include "plan.hpp"

namespace cst {

struct MttkrpArgs {
    int64_t nnz, q, n_chunks, slices;
    int R;
    const int64_t *ptr0, *ptr1;
    const int32_t *idx0, *idx1, *idx2;
    const double *vals;
    const int64_t *chunk_fiber;
    const int32_t *chunk_slice;
    const int64_t *slice_leaf;
    const double *B, *C;
    double *out, *partial;
    int compact;
};

template <bool VEC>
__device__ __forceinline__ void load2(const double *__restrict__ row, int r0, int R, double &x, double &y) {
    if (VEC) {
        const double2 v = *reinterpret_cast<const double2 *>(row + r0);
        x = v.x;
        y = v.y;
    } else {
        x = r0 < R ? row[r0] : 0.0;
        y = r0 + 1 < R ? row[r0 + 1] : 0.0;
    }
}

template <bool VEC>
__device__ __forceinline__ void store2(double *__restrict__ row, int r0, int R, double x, double y) {
    if (VEC) {
        *reinterpret_cast<double2 *>(row + r0) = make_double2(x, y);
    } else {
        if (r0 < R) row[r0] = x;
        if (r0 + 1 < R) row[r0 + 1] = y;
    }
}

template <int LPR, bool VEC>
__global__ void __launch_bounds__(256)
mttkrp3_kernel(MttkrpArgs a) {
    const int64_t gid = (int64_t(blockIdx.x) * 256 + threadIdx.x) / LPR;
    const int gl = threadIdx.x % LPR;
    if (gid >= a.n_chunks) return;
    const int r0 = 2 * gl;
    const int R = a.R;
    if (VEC && r0 >= R) return;
    const int64_t n0 = gid * a.q;
    const int64_t n1 = n0 + a.q < a.nnz ? n0 + a.q : a.nnz;
    int64_t f = a.chunk_fiber[gid];
    int32_t s = a.chunk_slice[gid];
    const int32_t s_first = s;
    int64_t fiber_end = a.ptr1[f + 1];
    if (fiber_end > n1) fiber_end = n1;
    int64_t slice_fend = a.ptr0[s + 1];
    int32_t j = a.idx1[f];
    double t0 = 0.0, t1 = 0.0, acc0 = 0.0, acc1 = 0.0;

    auto emit = [&](int32_t sl, double x, double y) {
        const int64_t lo = a.slice_leaf[sl], hi = a.slice_leaf[sl + 1];
        if (lo >= n0 && hi <= n1) {
            const int64_t row = a.compact ? int64_t(sl) : int64_t(a.idx0[sl]);
            store2<VEC>(a.out + row * R, r0, R, x, y);
        } else {
            const int64_t slot = 2 * gid + (sl == s_first ? 0 : 1);
            store2<VEC>(a.partial + slot * R, r0, R, x, y);
        }
    };
    auto fiber_done = [&](int64_t n) {          // n = position after the fiber's last leaf in this chunk
        double b0, b1;
        load2<VEC>(a.B + int64_t(j) * R, r0, R, b0, b1);
        acc0 = fma(b0, t0, acc0);
        acc1 = fma(b1, t1, acc1);
        t0 = 0.0;
        t1 = 0.0;
        if (n < n1) {
            ++f;
            if (f == slice_fend) {
                emit(s, acc0, acc1);
                acc0 = 0.0;
                acc1 = 0.0;
                ++s;
                slice_fend = a.ptr0[s + 1];
            }
            j = a.idx1[f];
            fiber_end = a.ptr1[f + 1];
            if (fiber_end > n1) fiber_end = n1;
        }
    };

    constexpr int U = 4;
    int64_t n = n0;
    while (n + U <= n1) {
        int32_t kk[U];
        double vv[U], c0[U], c1[U];
#pragma unroll
        for (int u = 0; u < U; ++u) { kk[u] = a.idx2[n + u]; vv[u] = a.vals[n + u]; }
#pragma unroll
        for (int u = 0; u < U; ++u) load2<VEC>(a.C + int64_t(kk[u]) * R, r0, R, c0[u], c1[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            t0 = fma(vv[u], c0[u], t0);
            t1 = fma(vv[u], c1[u], t1);
            ++n;
            if (n == fiber_end) fiber_done(n);
        }
    }
    for (; n < n1;) {
        const int32_t k = a.idx2[n];
        const double v = a.vals[n];
        double c0, c1;
        load2<VEC>(a.C + int64_t(k) * R, r0, R, c0, c1);
        t0 = fma(v, c0, t0);
        t1 = fma(v, c1, t1);
        ++n;
        if (n == fiber_end) fiber_done(n);
    }
    emit(s, acc0, acc1);
}

// Rows of slices shared by several chunks: add the partial rows in chunk order.
// One block per slice; G lane groups stride over the chunks, then a fixed-order LDS reduction.
template <int LPR>
__global__ void __launch_bounds__(256)
mttkrp3_fixup_kernel(MttkrpArgs a) {
    constexpr int G = 256 / LPR;
    __shared__ double red[256 * 2];
    const int64_t s = blockIdx.x;
    const int64_t lo = a.slice_leaf[s], hi = a.slice_leaf[s + 1];
    const int64_t ca = lo / a.q, cb = (hi - 1) / a.q;
    if (ca == cb) return;                           // stored directly by the main kernel
    const int g = threadIdx.x / LPR, gl = threadIdx.x % LPR;
    const int r0 = 2 * gl, R = a.R;
    double x = 0.0, y = 0.0;
    for (int64_t c = ca + g; c <= cb; c += G) {
        const int64_t slot = 2 * c + ((c == ca && lo != ca * a.q) ? 1 : 0);
        const double *row = a.partial + slot * R;
        if (r0 < R) x += row[r0];
        if (r0 + 1 < R) y += row[r0 + 1];
    }
    red[threadIdx.x * 2] = x;
    red[threadIdx.x * 2 + 1] = y;
    __syncthreads();
    if (g == 0) {
        for (int gg = 1; gg < G; ++gg) {
            x += red[(gg * LPR + gl) * 2];
            y += red[(gg * LPR + gl) * 2 + 1];
        }
        const int64_t row = a.compact ? s : int64_t(a.idx0[s]);
        if (r0 < R) a.out[row * R + r0] = x;
        if (r0 + 1 < R) a.out[row * R + r0 + 1] = y;
    }
}

template <int LPR>
static conststn_status launch_lpr(const conststn_plan_s *plan, const MttkrpArgs &a, bool vec, hipStream_t stream) {
    const int64_t groups_per_block = 256 / LPR;
    const dim3 grid(unsigned(div_up(a.n_chunks, groups_per_block))), block(256);
    {
        ProfScope prof(plan, stream);
        if (vec)
            mttkrp3_kernel<LPR, true><<<grid, block, 0, stream>>>(a);
        else
            mttkrp3_kernel<LPR, false><<<grid, block, 0, stream>>>(a);
    }
    CST_HIP(hipGetLastError());
    mttkrp3_fixup_kernel<LPR><<<dim3(unsigned(a.slices)), block, 0, stream>>>(a);
    CST_HIP(hipGetLastError());
    return CONSTSTN_OK;
}

conststn_status launch_mttkrp3(const conststn_plan_s *plan, const double *const *dense, double *out,
                               hipStream_t stream) {
    const conststn_csf_s *X = plan->X;
    MttkrpArgs a{};
    a.nnz = X->nnz;
    a.q = plan->chunk_q;
    a.n_chunks = plan->n_chunks;
    a.slices = X->nodes[0];
    a.R = plan->rank_of_level[1];
    a.ptr0 = X->ptr[0].p;
    a.ptr1 = X->ptr[1].p;
    a.idx0 = X->idx[0].p;
    a.idx1 = X->idx[1].p;
    a.idx2 = X->idx[2].p;
    a.vals = X->vals.p;
    a.chunk_fiber = plan->chunk_fiber.p;
    a.chunk_slice = plan->chunk_slice.p;
    a.slice_leaf = plan->slice_leaf.p;
    a.B = dense[plan->factor_of_level[1]];
    a.C = dense[plan->factor_of_level[2]];
    a.out = out;
    a.partial = plan->partial.p;
    a.compact = plan->compact ? 1 : 0;
    if (!plan->compact && a.slices < plan->out_rows)        // rows of empty slices are zero
        CST_TRY(zero_fill(out, plan->out_rows * plan->row_elems, stream));
    if (a.nnz == 0) return CONSTSTN_OK;
    const int R = a.R;
    const bool aligned = (reinterpret_cast<uintptr_t>(a.B) % 16 == 0) && (reinterpret_cast<uintptr_t>(a.C) % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(out) % 16 == 0);
    if (R > 128) { set_error("MTTKRP rank %d above 128 is not implemented", R); return CONSTSTN_EUNSUPPORTED; }
    // smallest power-of-two lane group covering ceil(R/2) lanes; 16-byte accesses when every
    // lane of the group holds two valid, aligned entries
    int lpr = 1;
    while (2 * lpr < R) lpr *= 2;
    const bool vec = aligned && (R % 2 == 0);
    switch (lpr) {
        case 1: return launch_lpr<1>(plan, a, vec, stream);
        case 2: return launch_lpr<2>(plan, a, vec, stream);
        case 4: return launch_lpr<4>(plan, a, vec, stream);
        case 8: return launch_lpr<8>(plan, a, vec, stream);
        case 16: return launch_lpr<16>(plan, a, vec, stream);
        case 32: return launch_lpr<32>(plan, a, vec, stream);
        default: return launch_lpr<64>(plan, a, vec, stream);
    }
}

}  // namespace cst
