// Load-balanced partition of a CSF tree into work units, built on the device at plan time.
//
// Power-law tensors have a few root slices with millions of leaves and very many with a
// handful.  Two partitions are used:
//   * MTTKRP (small accumulators): the LEAF array is cut into equal chunks regardless of
//     slice and fiber boundaries; a chunk that ends inside a fiber or slice contributes a
//     partial sum (legal by distributivity), combined by a fix-up pass.
//   * TTMc (a whole R2 x R3 row block per slice): every slice is cut into items of bounded
//     size; a slice made of several items is summed from partial row blocks by a fix-up pass.
#include <cstring>
#include <algorithm>

#include <cstdlib>

#include "plan.hpp"

namespace cst {

__global__ void zero_fill_kernel(double *p, int64_t n) {
    int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (; i < n; i += stride) p[i] = 0.0;
}

conststn_status zero_fill(double *p, int64_t n, hipStream_t stream) {
    if (n <= 0) return CONSTSTN_OK;
    const int64_t blocks = std::min<int64_t>(div_up(n, 256), 16384);
    zero_fill_kernel<<<dim3(unsigned(blocks)), dim3(256), 0, stream>>>(p, n);
    CST_HIP(hipGetLastError());
    return CONSTSTN_OK;
}

// largest p in [0, n) with ptr[p] <= x   (ptr ascending, ptr[0] <= x < ptr[n])
__device__ __forceinline__ int64_t owner_of(const int64_t *__restrict__ ptr, int64_t lo, int64_t hi, int64_t x) {
    // invariant: ptr[lo] <= x < ptr[hi]
    while (hi - lo > 1) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (ptr[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// slice_leaf[s] = first leaf position below root node s (composition of the child pointers)
__global__ void slice_leaf_kernel(int64_t slices, int levels_below, const int64_t *p0,
                                  const int64_t *p1, const int64_t *p2, int64_t *slice_leaf) {
    const int64_t s = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (s > slices) return;
    int64_t x = s;
    if (levels_below >= 1) x = p0[x];
    if (levels_below >= 2) x = p1[x];
    if (levels_below >= 3) x = p2[x];
    slice_leaf[s] = x;
}

static conststn_status make_slice_leaf(conststn_plan_s *plan) {
    const conststn_csf_s *X = plan->X;
    const int64_t slices = X->nodes[0];
    CST_TRY(plan->slice_leaf.alloc(size_t(slices) + 1));
    const int below = X->order - 1;
    if (below > 3) { set_error("CSF order above 4 is not implemented in the partitioner"); return CONSTSTN_EUNSUPPORTED; }
    slice_leaf_kernel<<<dim3(unsigned(div_up(slices + 1, 256))), dim3(256)>>>(
        slices, below, below >= 1 ? X->ptr[0].p : nullptr, below >= 2 ? X->ptr[1].p : nullptr,
        below >= 3 ? X->ptr[2].p : nullptr, plan->slice_leaf.p);
    CST_HIP(hipGetLastError());
    return CONSTSTN_OK;
}

// ---- MTTKRP: equal chunks of the leaf array ---------------------------------------------

__global__ void mttkrp_chunks_kernel(int64_t n_chunks, int64_t q, int64_t slices, int64_t fibers,
                                     const int64_t *__restrict__ ptr0, const int64_t *__restrict__ ptr1,
                                     int64_t *chunk_fiber, int32_t *chunk_slice) {
    const int64_t c = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (c >= n_chunks) return;
    const int64_t n = c * q;
    const int64_t f = owner_of(ptr1, 0, fibers, n);
    const int64_t s = owner_of(ptr0, 0, slices, f);
    chunk_fiber[c] = f;
    chunk_slice[c] = int32_t(s);
}

__global__ void heavy_slices_kernel(int64_t slices, const int64_t *__restrict__ slice_leaf, int64_t q,
                                    int span, int32_t *list, int *count) {
    const int64_t s = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (s >= slices) return;
    const int64_t ca = slice_leaf[s] / q, cb = (slice_leaf[s + 1] - 1) / q;
    if (cb - ca >= span) list[atomicAdd(count, 1)] = int32_t(s);
}

// ---- MTTKRP rank-32 path: hot-row selection and the re-encoded leaf stream ------------------

__global__ void leaf_histogram_kernel(int64_t nnz, const int32_t *__restrict__ leaf, unsigned *counts) {
    int64_t n = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (; n < nnz; n += stride) atomicAdd(&counts[leaf[n]], 1u);
}

// The same histogram with block-private LDS counters for one window of kHistWindow bins; the
// power-law tensors this path is meant for put a large share of the leaves in a few bins, which
// serialises global atomics.
constexpr int kHistWindow = 16384;
__global__ void __launch_bounds__(256)
leaf_histogram_window_kernel(int64_t nnz, const int32_t *__restrict__ leaf, int32_t lo, unsigned *counts, int64_t dim) {
    __shared__ unsigned h[kHistWindow];
    for (int b = threadIdx.x; b < kHistWindow; b += 256) h[b] = 0;
    __syncthreads();
    int64_t n = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (; n < nnz; n += stride) {
        const unsigned k = unsigned(leaf[n] - lo);
        if (k < unsigned(kHistWindow)) atomicAdd(&h[k], 1u);
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kHistWindow; b += 256)
        if (h[b] && lo + b < dim) atomicAdd(&counts[lo + b], h[b]);
}

__global__ void iota_i32_kernel(int32_t *p, int64_t n) {
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = int32_t(i);
}

__global__ void fill_i32_kernel(int32_t *p, int64_t n, int32_t v) {
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

__global__ void rank_keys_kernel(int64_t n, const unsigned *__restrict__ counts, uint64_t *keys, uint32_t *rows) {
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= n) return;
    keys[i] = uint64_t(0xffffffffu - counts[i]);
    rows[i] = uint32_t(i);
}

__global__ void hot_slots_kernel(int n_hot, const uint32_t *__restrict__ rows_by_count, int32_t *slot_of_row,
                                 int32_t *hot_rows) {
    const int h = blockIdx.x * blockDim.x + threadIdx.x;
    if (h >= n_hot) return;
    hot_rows[h] = int32_t(rows_by_count[h]);
    slot_of_row[rows_by_count[h]] = h;
}

__global__ void encode_leaves_kernel(int64_t nnz, const int32_t *__restrict__ leaf,
                                     const int32_t *__restrict__ slot_of_row, uint32_t *code) {
    int64_t n = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (; n < nnz; n += stride) {
        const int32_t k = leaf[n];
        const int32_t sl = slot_of_row[k];
        code[n] = sl >= 0 ? (0x80000000u | uint32_t(sl)) : uint32_t(k);
    }
}

// mark the last leaf of every fiber (bit 30) and of every slice (bit 29)
__global__ void mark_ends_kernel(int64_t nodes, const int64_t *__restrict__ leaf_end, uint32_t bit,
                                 uint32_t *code) {
    const int64_t p = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (p < nodes) atomicOr(&code[leaf_end[p + 1] - 1], bit);
}

// ---- MTTKRP rank-32 path, split form: filter the CSF by a leaf predicate ----------------------

__global__ void hot_flags_kernel(int64_t nnz, const int32_t *__restrict__ leaf,
                                 const int32_t *__restrict__ slot_of_row, int64_t *flag) {
    int64_t n = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (; n < nnz; n += stride) flag[n] = slot_of_row[leaf[n]] >= 0 ? 1 : 0;
}

// position of leaf boundary x inside the part (part 0: hot leaves, part 1: the others)
__device__ __forceinline__ int64_t part_pos(int64_t x, const int64_t *__restrict__ pos_hot, int64_t nnz,
                                            int64_t total_hot, int part) {
    const int64_t h = x < nnz ? pos_hot[x] : total_hot;
    return part == 0 ? h : x - h;
}

__global__ void part_fiber_keep_kernel(int64_t fibers, const int64_t *__restrict__ ptr1,
                                       const int64_t *__restrict__ pos_hot, int64_t nnz, int64_t total_hot,
                                       int part, int64_t *keep) {
    const int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (f >= fibers) return;
    keep[f] = part_pos(ptr1[f + 1], pos_hot, nnz, total_hot, part) > part_pos(ptr1[f], pos_hot, nnz, total_hot, part) ? 1 : 0;
}

__global__ void part_slice_keep_kernel(int64_t slices, const int64_t *__restrict__ ptr0,
                                       const int64_t *__restrict__ fpos, int64_t fibers, int64_t kept_fibers,
                                       int64_t *keep) {
    const int64_t s = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (s >= slices) return;
    const int64_t a = fpos[ptr0[s]];
    const int64_t b = ptr0[s + 1] < fibers ? fpos[ptr0[s + 1]] : kept_fibers;
    keep[s] = b > a ? 1 : 0;
}

__global__ void part_fill_leaves_kernel(int64_t nnz, const int32_t *__restrict__ leaf,
                                        const double *__restrict__ vals, const int32_t *__restrict__ slot_of_row,
                                        const int64_t *__restrict__ pos_hot, int part, uint32_t *code, double *out_vals) {
    int64_t n = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (; n < nnz; n += stride) {
        const int32_t k = leaf[n];
        const int32_t sl = slot_of_row[k];
        if ((sl >= 0) != (part == 0)) continue;
        const int64_t p = part == 0 ? pos_hot[n] : n - pos_hot[n];
        code[p] = part == 0 ? (0x80000000u | uint32_t(sl)) : uint32_t(k);
        out_vals[p] = vals[n];
    }
}

__global__ void part_fill_fibers_kernel(int64_t fibers, const int64_t *__restrict__ ptr1,
                                        const int32_t *__restrict__ idx1, const int64_t *__restrict__ pos_hot,
                                        int64_t nnz, int64_t total_hot, int part, const int64_t *__restrict__ keep,
                                        const int64_t *__restrict__ fpos, int64_t kept, int64_t part_nnz,
                                        int64_t *ptr1_out, int32_t *idx1_out) {
    const int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (f == 0) ptr1_out[kept] = part_nnz;
    if (f >= fibers || !keep[f]) return;
    ptr1_out[fpos[f]] = part_pos(ptr1[f], pos_hot, nnz, total_hot, part);
    idx1_out[fpos[f]] = idx1[f];
}

__global__ void part_fill_slices_kernel(int64_t slices, const int64_t *__restrict__ ptr0,
                                        const int32_t *__restrict__ idx0, int compact,
                                        const int64_t *__restrict__ keep, const int64_t *__restrict__ spos,
                                        const int64_t *__restrict__ fpos, int64_t kept_slices, int64_t kept_fibers,
                                        int64_t *ptr0_out, int32_t *row_out) {
    const int64_t s = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (s == 0) ptr0_out[kept_slices] = kept_fibers;
    if (s >= slices || !keep[s]) return;
    ptr0_out[spos[s]] = fpos[ptr0[s]];
    row_out[spos[s]] = compact ? int32_t(s) : idx0[s];
}

static conststn_status build_part_tables(MttkrpPart &P, int R, int64_t q) {
    const dim3 block(256);
    CST_TRY(P.slice_leaf.alloc(size_t(P.slices) + 1));
    slice_leaf_kernel<<<dim3(unsigned(div_up(P.slices + 1, 256))), block>>>(P.slices, 2, P.ptr0.p, P.ptr1.p, nullptr,
                                                                          P.slice_leaf.p);
    CST_HIP(hipGetLastError());
    mark_ends_kernel<<<dim3(unsigned(div_up(P.fibers, 256))), block>>>(P.fibers, P.ptr1.p, 0x40000000u, P.code.p);
    mark_ends_kernel<<<dim3(unsigned(div_up(P.slices, 256))), block>>>(P.slices, P.slice_leaf.p, 0x20000000u, P.code.p);
    CST_HIP(hipGetLastError());
    P.chunk_q = q;
    P.n_chunks = div_up(P.nnz, q);
    CST_TRY(P.chunk_fiber.alloc(size_t(P.n_chunks)));
    CST_TRY(P.chunk_slice.alloc(size_t(P.n_chunks)));
    CST_TRY(P.partial.alloc(size_t(P.n_chunks) * 2 * size_t(R)));
    mttkrp_chunks_kernel<<<dim3(unsigned(div_up(P.n_chunks, 256))), block>>>(P.n_chunks, q, P.slices, P.fibers,
                                                                           P.ptr0.p, P.ptr1.p, P.chunk_fiber.p,
                                                                           P.chunk_slice.p);
    CST_HIP(hipGetLastError());
    const int64_t max_heavy = P.nnz / (int64_t(kHeavySpan) * q) + 1;
    CST_TRY(P.heavy_slices.alloc(size_t(max_heavy)));
    DevBuf<int> hcount;
    CST_TRY(hcount.alloc(1));
    CST_HIP(hipMemset(hcount.p, 0, sizeof(int)));
    heavy_slices_kernel<<<dim3(unsigned(div_up(P.slices, 256))), block>>>(P.slices, P.slice_leaf.p, q, kHeavySpan,
                                                                         P.heavy_slices.p, hcount.p);
    CST_HIP(hipGetLastError());
    CST_HIP(hipMemcpy(&P.n_heavy, hcount.p, sizeof(int), hipMemcpyDeviceToHost));
    CST_TRY(P.heavy_partial.alloc(size_t(P.n_heavy) * kHeavySegments * size_t(R)));
    return CONSTSTN_OK;
}


static conststn_status build_mttkrp3_split(conststn_plan_s *plan, const int32_t *slot_of_row) {
    const conststn_csf_s *X = plan->X;
    const int64_t nnz = X->nnz, fibers = X->nodes[1], slices = X->nodes[0];
    const int R = plan->rank_of_level[1];
    const dim3 block(256);
    DevBuf<int64_t> flag, pos_hot;
    CST_TRY(flag.alloc(nnz));
    CST_TRY(pos_hot.alloc(nnz));
    hot_flags_kernel<<<dim3(unsigned(std::min<int64_t>(div_up(nnz, 256), 16384))), block>>>(nnz, X->idx[2].p, slot_of_row, flag.p);
    CST_HIP(hipGetLastError());
    int64_t total_hot = 0;
    CST_TRY(exscan(flag.p, pos_hot.p, nnz, &total_hot));
    flag.release();
    for (int part = 0; part < 2; ++part) {
        MttkrpPart &P = plan->part[part];
        P.nnz = part == 0 ? total_hot : nnz - total_hot;
        P.slices = P.fibers = 0;
        P.n_chunks = 0;
        if (P.nnz == 0) continue;
        DevBuf<int64_t> keepf, fpos, keeps, spos;
        CST_TRY(keepf.alloc(fibers));
        CST_TRY(fpos.alloc(fibers));
        CST_TRY(keeps.alloc(slices));
        CST_TRY(spos.alloc(slices));
        part_fiber_keep_kernel<<<dim3(unsigned(div_up(fibers, 256))), block>>>(fibers, X->ptr[1].p, pos_hot.p, nnz,
                                                                              total_hot, part, keepf.p);
        CST_HIP(hipGetLastError());
        CST_TRY(exscan(keepf.p, fpos.p, fibers, &P.fibers));
        part_slice_keep_kernel<<<dim3(unsigned(div_up(slices, 256))), block>>>(slices, X->ptr[0].p, fpos.p, fibers,
                                                                              P.fibers, keeps.p);
        CST_HIP(hipGetLastError());
        CST_TRY(exscan(keeps.p, spos.p, slices, &P.slices));
        CST_TRY(P.code.alloc(size_t(P.nnz)));
        CST_TRY(P.vals.alloc(size_t(P.nnz)));
        CST_TRY(P.ptr1.alloc(size_t(P.fibers) + 1));
        CST_TRY(P.idx1.alloc(size_t(P.fibers)));
        CST_TRY(P.ptr0.alloc(size_t(P.slices) + 1));
        CST_TRY(P.row_of_slice.alloc(size_t(P.slices)));
        part_fill_leaves_kernel<<<dim3(unsigned(std::min<int64_t>(div_up(nnz, 256), 16384))), block>>>(
            nnz, X->idx[2].p, X->vals.p, slot_of_row, pos_hot.p, part, P.code.p, P.vals.p);
        part_fill_fibers_kernel<<<dim3(unsigned(div_up(fibers, 256))), block>>>(
            fibers, X->ptr[1].p, X->idx[1].p, pos_hot.p, nnz, total_hot, part, keepf.p, fpos.p, P.fibers, P.nnz,
            P.ptr1.p, P.idx1.p);
        part_fill_slices_kernel<<<dim3(unsigned(div_up(slices, 256))), block>>>(
            slices, X->ptr[0].p, X->idx[0].p, plan->compact ? 1 : 0, keeps.p, spos.p, fpos.p, P.slices, P.fibers,
            P.ptr0.p, P.row_of_slice.p);
        CST_HIP(hipGetLastError());
        CST_TRY(build_part_tables(P, R, plan->chunk_q));
        CST_HIP(hipDeviceSynchronize());
    }
    plan->split = true;
    {
        // hot and cold wavefronts per workgroup of the one-launch form (44 = four and four); 0 = two launches
        const int64_t dual = plan->opt("mttkrp_dual", 44);
        if (dual == 44 || dual == 35 || dual == 53 || dual == 88) {
            plan->mttkrp_dual = int(dual);
            CST_TRY(plan->mttkrp_out2.alloc(size_t(plan->out_rows * plan->row_elems)));
        }
    }
    return CONSTSTN_OK;
}

static conststn_status build_mttkrp3_r32_encoding(conststn_plan_s *plan) {
    const conststn_csf_s *X = plan->X;
    const int64_t nnz = X->nnz;
    const int64_t dim = X->dims[X->mode_order[2]];
    plan->n_hot = 0;
    if (plan->rank_of_level[1] != 32 || dim >= (int64_t(1) << 28) || nnz == 0 ||
        X->dims[X->mode_order[1]] >= (int64_t(1) << 28))
        return CONSTSTN_OK;                               // the kernel indexes factor rows with 32 bits
    int64_t want = plan->opt("mttkrp_hot", 256);
    if (want > dim) want = dim;
    want = std::min<int64_t>(want, 608);                 // 608 rows x 256 B = 152 KB of LDS at most
    DevBuf<unsigned> counts;
    DevBuf<int32_t> slot_of_row;
    DevBuf<uint64_t> rank_key_a, rank_key_b;
    DevBuf<uint32_t> rank_row_a, rank_row_b;
    CST_TRY(counts.alloc(dim));
    CST_TRY(rank_key_a.alloc(dim));
    CST_TRY(rank_key_b.alloc(dim));
    CST_TRY(rank_row_a.alloc(dim));
    CST_TRY(rank_row_b.alloc(dim));
    CST_TRY(slot_of_row.alloc(dim));
    CST_HIP(hipMemset(counts.p, 0, size_t(dim) * sizeof(unsigned)));
    const dim3 block(256);
    if (dim <= 4 * kHistWindow) {
        for (int64_t lo = 0; lo < dim; lo += kHistWindow)
            leaf_histogram_window_kernel<<<dim3(unsigned(std::min<int64_t>(div_up(nnz, 256 * 64), 2048))), block>>>(
                nnz, X->idx[2].p, int32_t(lo), counts.p, dim);
    } else {
        leaf_histogram_kernel<<<dim3(unsigned(std::min<int64_t>(div_up(nnz, 256), 8192))), block>>>(nnz, X->idx[2].p, counts.p);
    }
    CST_HIP(hipGetLastError());
    // rows by falling count: ascending stable sort on (2^32 - 1 - count), ties keep the lower row first
    rank_keys_kernel<<<dim3(unsigned(div_up(dim, 256))), block>>>(dim, counts.p, rank_key_a.p, rank_row_a.p);
    fill_i32_kernel<<<dim3(unsigned(div_up(dim, 256))), block>>>(slot_of_row.p, dim, -1);
    CST_HIP(hipGetLastError());
    const uint64_t *keys_sorted = nullptr;
    const uint32_t *rows_sorted = nullptr;
    CST_TRY(radix_sort_pairs_u64(rank_key_a.p, rank_key_b.p, rank_row_a.p, rank_row_b.p, dim, 32, hipStream_t(0),
                                 &keys_sorted, &rows_sorted));
    CST_TRY(plan->hot_rows.alloc(size_t(want)));
    hot_slots_kernel<<<dim3(unsigned(div_up(want, 256))), block>>>(int(want), rows_sorted, slot_of_row.p,
                                                                  plan->hot_rows.p);
    CST_HIP(hipGetLastError());
    CST_TRY(plan->leaf_code.alloc(size_t(nnz)));
    encode_leaves_kernel<<<dim3(unsigned(std::min<int64_t>(div_up(nnz, 256), 16384))), block>>>(
        nnz, X->idx[2].p, slot_of_row.p, plan->leaf_code.p);
    CST_HIP(hipGetLastError());
    mark_ends_kernel<<<dim3(unsigned(div_up(X->nodes[1], 256))), block>>>(X->nodes[1], X->ptr[1].p, 0x40000000u,
                                                                        plan->leaf_code.p);
    mark_ends_kernel<<<dim3(unsigned(div_up(X->nodes[0], 256))), block>>>(X->nodes[0], plan->slice_leaf.p,
                                                                        0x20000000u, plan->leaf_code.p);
    CST_HIP(hipGetLastError());
    CST_HIP(hipDeviceSynchronize());
    plan->n_hot = int(want);
    if (plan->opt("mttkrp_split", 1) == 1) CST_TRY(build_mttkrp3_split(plan, slot_of_row.p));
    return CONSTSTN_OK;
}

conststn_status build_mttkrp3_tables(conststn_plan_s *plan) {
    const conststn_csf_s *X = plan->X;
    const int64_t nnz = X->nnz;
    const int R = plan->rank_of_level[1];
    CST_TRY(make_slice_leaf(plan));
    // chunk length: short enough for >= ~64K independent lane groups, long enough that the
    // two partial rows per chunk stay a small fraction of the traffic
    int64_t q = plan->opt("mttkrp_chunk", 0);
    if (q <= 0) {
        q = nnz / 262144;
        q = std::max<int64_t>(64, std::min<int64_t>(q, 512));
    }
    q = div_up(q, 16) * 16;                      // the rank-32 kernel reads leaves 16 at a time
    plan->chunk_q = q;
    plan->n_chunks = div_up(nnz, q);
    CST_TRY(plan->chunk_fiber.alloc(size_t(plan->n_chunks)));
    CST_TRY(plan->chunk_slice.alloc(size_t(plan->n_chunks)));
    CST_TRY(plan->partial.alloc(size_t(plan->n_chunks) * 2 * size_t(R)));
    if (plan->n_chunks > 0) {
        mttkrp_chunks_kernel<<<dim3(unsigned(div_up(plan->n_chunks, 256))), dim3(256)>>>(
            plan->n_chunks, q, X->nodes[0], X->nodes[1], X->ptr[0].p, X->ptr[1].p,
            plan->chunk_fiber.p, plan->chunk_slice.p);
        CST_HIP(hipGetLastError());
    }
    // slices shared by many chunks: listed for the two-stage fix-up (at most nnz / (span * q))
    plan->n_heavy = 0;
    const int64_t max_heavy = nnz / (int64_t(kHeavySpan) * q) + 1;
    CST_TRY(plan->heavy_slices.alloc(size_t(max_heavy)));
    DevBuf<int> hcount;
    CST_TRY(hcount.alloc(1));
    CST_HIP(hipMemset(hcount.p, 0, sizeof(int)));
    if (X->nodes[0] > 0) {
        heavy_slices_kernel<<<dim3(unsigned(div_up(X->nodes[0], 256))), dim3(256)>>>(
            X->nodes[0], plan->slice_leaf.p, q, kHeavySpan, plan->heavy_slices.p, hcount.p);
        CST_HIP(hipGetLastError());
    }
    CST_HIP(hipMemcpy(&plan->n_heavy, hcount.p, sizeof(int), hipMemcpyDeviceToHost));
    CST_TRY(plan->heavy_partial.alloc(size_t(plan->n_heavy) * kHeavySegments * size_t(R)));
    CST_HIP(hipDeviceSynchronize());
    CST_TRY(build_mttkrp3_r32_encoding(plan));
    return prepare_mttkrp3_launch(plan);
}

// ---- TTMc: bounded items inside slices ----------------------------------------------------

__global__ void ttmc_count_kernel(int64_t slices, const int64_t *__restrict__ unit_ptr, int64_t split,
                                  int64_t max_pieces, int64_t *pieces, int64_t *part_cnt, int64_t *is_split) {
    const int64_t s = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (s >= slices) return;
    const int64_t len = unit_ptr[s + 1] - unit_ptr[s];
    int64_t p = len <= split ? 1 : (len + split - 1) / split;
    if (max_pieces > 0 && p > max_pieces) p = max_pieces;     // bounds the partial blocks of one slice
    pieces[s] = p;
    part_cnt[s] = p > 1 ? p : 0;
    is_split[s] = p > 1 ? 1 : 0;
}

__global__ void ttmc_fill_kernel(int64_t slices, const int64_t *__restrict__ unit_ptr,
                                 const int64_t *__restrict__ pieces, const int64_t *__restrict__ item_off,
                                 const int64_t *__restrict__ part_off, const int64_t *__restrict__ split_rank,
                                 int order, const int64_t *__restrict__ ptr0, const int64_t *__restrict__ ptr1,
                                 SliceItem *items, int32_t *split_slices, int64_t *split_first,
                                 int32_t *split_count) {
    const int64_t s = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (s >= slices) return;
    const int64_t a = unit_ptr[s], len = unit_ptr[s + 1] - a, np = pieces[s];
    for (int64_t p = 0; p < np; ++p) {
        SliceItem it;
        it.slice = int32_t(s);
        it.pad = 0;
        // 128-bit safe: len < 2^40 and np < 2^31 in practice; split products to stay in range
        it.begin = a + (len / np) * p + ((len % np) * p) / np;
        it.end = (p + 1 == np) ? a + len : a + (len / np) * (p + 1) + ((len % np) * (p + 1)) / np;
        it.first = 0;
        if (order == 3) it.first = owner_of(ptr1, ptr0[s], ptr0[s + 1], it.begin);
        it.dest = np > 1 ? part_off[s] + p : -1;
        items[item_off[s] + p] = it;
    }
    if (np > 1) {
        const int64_t r = split_rank[s];
        split_slices[r] = int32_t(s);
        split_first[r] = part_off[s];
        split_count[r] = int32_t(np);
    }
}

// Exclusive prefix sum in three steps: every workgroup scans a tile of 2048 entries and reports its sum,
// the tile sums are scanned (recursively, the same way), every tile adds its offset.
constexpr int kScanTile = 2048;      // 256 threads x 8 entries

__global__ void __launch_bounds__(256)
scan_tile_kernel(const int64_t *in, int64_t *out, int64_t n, int64_t *tile_sums) {
    __shared__ int64_t wave_sum[4];
    const int64_t base = int64_t(blockIdx.x) * kScanTile + int64_t(threadIdx.x) * 8;
    int64_t v[8], s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) { v[i] = base + i < n ? in[base + i] : 0; s += v[i]; }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t inc = s;
    for (int off = 1; off < 64; off <<= 1) {
        const int64_t t = __shfl_up(inc, off, 64);
        if (lane >= off) inc += t;
    }
    if (lane == 63) wave_sum[wave] = inc;
    __syncthreads();
    int64_t run = inc - s;
    for (int w = 0; w < wave; ++w) run += wave_sum[w];
#pragma unroll
    for (int i = 0; i < 8; ++i) { if (base + i < n) out[base + i] = run; run += v[i]; }
    if (threadIdx.x == 255) tile_sums[blockIdx.x] = run;
}

__global__ void __launch_bounds__(256)
scan_add_kernel(int64_t *out, int64_t n, const int64_t *__restrict__ tile_offsets) {
    const int64_t base = int64_t(blockIdx.x) * kScanTile + int64_t(threadIdx.x) * 8;
    const int64_t off = tile_offsets[blockIdx.x];
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if (base + i < n) out[base + i] += off;
}

static conststn_status exscan_device(const int64_t *in, int64_t *out, int64_t n) {
    const int64_t tiles = div_up(n, kScanTile);
    DevBuf<int64_t> sums, offs;
    CST_TRY(sums.alloc(size_t(tiles)));
    scan_tile_kernel<<<dim3(unsigned(tiles)), dim3(256)>>>(in, out, n, sums.p);
    CST_HIP(hipGetLastError());
    if (tiles > 1) {
        CST_TRY(offs.alloc(size_t(tiles)));
        CST_TRY(exscan_device(sums.p, offs.p, tiles));
        scan_add_kernel<<<dim3(unsigned(tiles)), dim3(256)>>>(out, n, offs.p);
        CST_HIP(hipGetLastError());
    }
    CST_HIP(hipDeviceSynchronize());      // the tile tables are released on return
    return CONSTSTN_OK;
}

conststn_status exscan(int64_t *in, int64_t *out, int64_t n, int64_t *total_host) {
    if (n <= 0) { *total_host = 0; return CONSTSTN_OK; }
    // the last input is read before the scan, so that in and out may be one array
    int64_t last_in = 0, last_out = 0;
    CST_HIP(hipMemcpy(&last_in, in + (n - 1), sizeof(int64_t), hipMemcpyDeviceToHost));
    CST_TRY(exscan_device(in, out, n));
    CST_HIP(hipMemcpy(&last_out, out + (n - 1), sizeof(int64_t), hipMemcpyDeviceToHost));
    *total_host = last_in + last_out;
    return CONSTSTN_OK;
}

// ---- TTMc order-3 MFMA path: fibers refined into rows of bounded length ----------------------

__global__ void fiber_rows_kernel(int64_t fibers, const int64_t *__restrict__ ptr1, int64_t *rows_of) {
    const int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (f < fibers) rows_of[f] = (ptr1[f + 1] - ptr1[f] + kRowLeaves - 1) / kRowLeaves;
}

// Besides the tables, a sort key per row: (slice, 16 - leaves).  Sorting by it orders the rows of
// a slice from long to short, so the four rows of one K-step have (nearly) the same number of
// leaves and the leaf stage wastes no gather instructions on the shortest of them.
__global__ void fill_rows_kernel(int64_t fibers, int64_t slices, const int64_t *__restrict__ ptr0,
                                 const int64_t *__restrict__ ptr1, const int32_t *__restrict__ idx1,
                                 const int64_t *__restrict__ row_off, int64_t *row_leaf, int32_t *row_j,
                                 int32_t *row_cnt, uint64_t *row_key, uint32_t *row_id) {
    const int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (f >= fibers) return;
    int64_t lo = 0, hi = slices;                // slice of fiber f: last s with ptr0[s] <= f
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (ptr0[mid] <= f) lo = mid; else hi = mid;
    }
    const int64_t a = ptr1[f], b = ptr1[f + 1];
    int64_t r = row_off[f];
    for (int64_t n = a; n < b; n += kRowLeaves, ++r) {
        const int cnt = int(b - n < kRowLeaves ? b - n : kRowLeaves);
        row_leaf[r] = n;
        row_j[r] = idx1[f];
        row_cnt[r] = cnt;
        row_key[r] = (uint64_t(lo) << 8) | uint64_t(kRowLeaves - cnt);
        row_id[r] = uint32_t(r);
    }
}

__global__ void permute_rows_kernel(int64_t rows, const uint32_t *__restrict__ order,
                                    const int64_t *__restrict__ leaf_in, const int32_t *__restrict__ j_in,
                                    const int32_t *__restrict__ cnt_in, RowDesc *out) {
    const int64_t r = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (r >= rows) return;
    const uint32_t src = order[r];
    out[r] = RowDesc{leaf_in[src], cnt_in[src], j_in[src]};
}

__global__ void slice_rows_kernel(int64_t slices, int64_t fibers, const int64_t *__restrict__ ptr0,
                                  const int64_t *__restrict__ row_off, int64_t total_rows,
                                  int64_t *slice_row) {
    const int64_t s = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (s > slices) return;
    const int64_t f = ptr0[s];
    slice_row[s] = f < fibers ? row_off[f] : total_rows;
}


static conststn_status build_rows_core(int64_t slices, int64_t fibers, const int64_t *ptr0, const int64_t *ptr1,
                                       const int32_t *idx1, DevBuf<RowDesc> &rows_out, DevBuf<int64_t> &slice_row,
                                       int64_t &n_rows) {
    DevBuf<int64_t> rows_of, row_off;
    CST_TRY(rows_of.alloc(fibers));
    CST_TRY(row_off.alloc(fibers));
    const dim3 block(256);
    fiber_rows_kernel<<<dim3(unsigned(div_up(fibers, 256))), block>>>(fibers, ptr1, rows_of.p);
    CST_HIP(hipGetLastError());
    CST_TRY(exscan(rows_of.p, row_off.p, fibers, &n_rows));
    const int64_t rows = n_rows;
    if (rows >= (int64_t(1) << 31)) { set_error("more than 2^31 rows"); return CONSTSTN_EUNSUPPORTED; }
    CST_TRY(rows_out.alloc(size_t(rows)));
    CST_TRY(slice_row.alloc(size_t(slices) + 1));
    {
        DevBuf<int64_t> leaf0;
        DevBuf<int32_t> j0, cnt0;
        DevBuf<uint32_t> id0, id1;
        DevBuf<uint64_t> key0, key1;
        CST_TRY(leaf0.alloc(size_t(rows)));
        CST_TRY(j0.alloc(size_t(rows)));
        CST_TRY(cnt0.alloc(size_t(rows)));
        CST_TRY(id0.alloc(size_t(rows)));
        CST_TRY(id1.alloc(size_t(rows)));
        CST_TRY(key0.alloc(size_t(rows)));
        CST_TRY(key1.alloc(size_t(rows)));
        fill_rows_kernel<<<dim3(unsigned(div_up(fibers, 256))), block>>>(
            fibers, slices, ptr0, ptr1, idx1, row_off.p, leaf0.p, j0.p, cnt0.p, key0.p, id0.p);
        CST_HIP(hipGetLastError());
        if (rows > 0) {
            // stable sort by (slice, 16 - leaves): rows stay inside their slice, longest first
            const int end_bit = 8 + ceil_log2_u64(uint64_t(slices) + 1);
            const uint64_t *keys_sorted = nullptr;
            const uint32_t *order = nullptr;
            CST_TRY(radix_sort_pairs_u64(key0.p, key1.p, id0.p, id1.p, rows, end_bit, hipStream_t(0), &keys_sorted, &order));
            permute_rows_kernel<<<dim3(unsigned(div_up(rows, 256))), block>>>(
                rows, order, leaf0.p, j0.p, cnt0.p, rows_out.p);
            CST_HIP(hipGetLastError());
        }
        CST_HIP(hipDeviceSynchronize());
    }
    slice_rows_kernel<<<dim3(unsigned(div_up(slices + 1, 256))), block>>>(
        slices, fibers, ptr0, row_off.p, n_rows, slice_row.p);
    CST_HIP(hipGetLastError());
    CST_HIP(hipDeviceSynchronize());
    return CONSTSTN_OK;
}

static conststn_status build_rows(conststn_plan_s *plan) {
    const conststn_csf_s *X = plan->X;
    return build_rows_core(X->nodes[0], X->nodes[1], X->ptr[0].p, X->ptr[1].p, X->idx[1].p, plan->rows,
                           plan->slice_row, plan->n_rows_tab);
}

// ---- TTMc order-4 MFMA path: nodes -> pieces (<= kPieceLeaves leaves), fibers -> rows (<= 4 pieces)

__global__ void count_units_kernel(int64_t n, const int64_t *__restrict__ ptr, int64_t per, int64_t *cnt) {
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) cnt[i] = (ptr[i + 1] - ptr[i] + per - 1) / per;
}

// Order-4 MFMA path.  The pieces of a fiber are taken four at a time ("groups", the K = 4 of the
// mid-level matrix instruction; the last group of a fiber is padded with empty records) and the
// fibers of a slice four at a time ("K-steps", the K = 4 of the slice-level instruction).  The
// kernel then walks one flat stream of groups; everything it needs to know about the structure
// travels in the records: flag bits in the k field say whether a group ends its fiber, ends its
// K-step or starts one, and in the first group of a K-step the spare field of slot s holds the
// level-1 index of the K-step's fiber s.
__global__ void fiber_groups_kernel(int64_t fibers, int64_t nodes, const int64_t *__restrict__ ptr1,
                                    const int64_t *__restrict__ piece_off, int64_t total_pieces,
                                    int64_t *groups_of) {
    const int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (f >= fibers) return;
    const int64_t a = piece_off[ptr1[f]];
    const int64_t b = ptr1[f + 1] < nodes ? piece_off[ptr1[f + 1]] : total_pieces;
    groups_of[f] = (b - a + 3) / 4;
}

__global__ void slice_ksteps_kernel(int64_t slices, const int64_t *__restrict__ ptr0, int64_t *ksteps_of) {
    const int64_t s = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (s < slices) ksteps_of[s] = (ptr0[s + 1] - ptr0[s] + 3) / 4;
}

__global__ void kstep_groups_kernel(int64_t slices, const int64_t *__restrict__ ptr0,
                                    const int64_t *__restrict__ slice_kstep, const int64_t *__restrict__ grp_off,
                                    int64_t total_ksteps, int64_t total_groups, int64_t *kstep_group) {
    const int64_t s = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (s == 0) kstep_group[total_ksteps] = total_groups;
    if (s >= slices) return;
    int64_t k = slice_kstep[s];
    for (int64_t f = ptr0[s]; f < ptr0[s + 1]; f += 4, ++k) kstep_group[k] = grp_off[f];
}

__global__ void fill_groups_kernel(int64_t fibers, int64_t slices, const int64_t *__restrict__ ptr0,
                                   const int64_t *__restrict__ ptr1, const int64_t *__restrict__ ptr2,
                                   const int32_t *__restrict__ idx1, const int32_t *__restrict__ idx2,
                                   const int32_t *__restrict__ idx3, const double *__restrict__ vals,
                                   const int64_t *__restrict__ grp_off, PieceDesc *rec) {
    const int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (f >= fibers) return;
    int64_t lo = 0, hi = slices;                // slice of fiber f: last s with ptr0[s] <= f
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (ptr0[mid] <= f) lo = mid; else hi = mid;
    }
    const int64_t fa = ptr0[lo], fb = ptr0[lo + 1];
    const int q = int((f - fa) & 3);
    const bool closes_kstep = q == 3 || f + 1 == fb;
    int64_t r = grp_off[f] * 4;                 // next record
    const int64_t r0 = r;
    auto put = [&](int32_t k, int32_t l0, int32_t l1, double v0, double v1) {
        PieceDesc d;
        d.k = k;
        d.l0 = l0;
        d.l1 = l1;
        d.pad = 0;
        d.v0 = v0;
        d.v1 = v1;
        rec[r++] = d;
    };
    for (int64_t n = ptr1[f]; n < ptr1[f + 1]; ++n) {
        const int64_t end = ptr2[n + 1];
        for (int64_t e = ptr2[n]; e < end; e += kPieceLeaves)
            put(idx2[n], idx3[e], e + 1 < end ? idx3[e + 1] : idx3[e], vals[e], e + 1 < end ? vals[e + 1] : 0.0);
    }
    // Empty records, and the absent second leaf above, name rows the fiber uses anyway and carry the
    // value 0: the kernel then needs no test for them, and a factor row that is not finite spoils only
    // results it belongs to.
    {
        const int64_t n0 = ptr1[f], e0 = ptr2[n0];
        while ((r - r0) & 3) put(idx2[n0], idx3[e0], idx3[e0], 0.0, 0.0);
    }
    // structure flags on every record of a group; level-1 indices on the first group of a K-step
    const int64_t groups = (r - r0) >> 2;
    for (int64_t g = 0; g < groups; ++g) {
        uint32_t flags = 0;
        if (g + 1 == groups) flags |= kGrpEndsFiber | (closes_kstep ? kGrpEndsKstep : 0u);
        if (g == 0 && q == 0) flags |= kGrpStartsKstep;
        for (int sl = 0; sl < 4; ++sl) {
            PieceDesc &d = rec[r0 + g * 4 + sl];
            d.k = int32_t(uint32_t(d.k) | flags);
            if (g == 0 && q == 0) d.pad = f + sl < fb ? idx1[f + sl] : -1;
        }
    }
}

static conststn_status build_piece_groups(conststn_plan_s *plan) {
    const conststn_csf_s *X = plan->X;
    const int64_t slices = X->nodes[0], fibers = X->nodes[1], nodes = X->nodes[2];
    const int64_t K = X->dims[X->mode_order[2]];
    if (K >= (int64_t(1) << 28)) { set_error("level-2 extent of 2^28 or more"); return CONSTSTN_EUNSUPPORTED; }
    const dim3 block(256);
    DevBuf<int64_t> cnt, piece_off, groups_of, grp_off, ksteps_of;
    CST_TRY(cnt.alloc(nodes));
    CST_TRY(piece_off.alloc(nodes));
    count_units_kernel<<<dim3(unsigned(div_up(nodes, 256))), block>>>(nodes, X->ptr[2].p, kPieceLeaves, cnt.p);
    CST_HIP(hipGetLastError());
    int64_t total_pieces = 0;
    CST_TRY(exscan(cnt.p, piece_off.p, nodes, &total_pieces));
    CST_TRY(groups_of.alloc(fibers));
    CST_TRY(grp_off.alloc(fibers));
    fiber_groups_kernel<<<dim3(unsigned(div_up(fibers, 256))), block>>>(fibers, nodes, X->ptr[1].p, piece_off.p,
                                                                       total_pieces, groups_of.p);
    CST_HIP(hipGetLastError());
    int64_t total_groups = 0;
    CST_TRY(exscan(groups_of.p, grp_off.p, fibers, &total_groups));
    plan->n_pieces = total_groups * 4;
    CST_TRY(ksteps_of.alloc(slices));
    CST_TRY(plan->slice_row.alloc(size_t(slices) + 1));             // first K-step of each slice
    slice_ksteps_kernel<<<dim3(unsigned(div_up(slices, 256))), block>>>(slices, X->ptr[0].p, ksteps_of.p);
    CST_HIP(hipGetLastError());
    int64_t total_ksteps = 0;
    CST_TRY(exscan(ksteps_of.p, plan->slice_row.p, slices, &total_ksteps));
    CST_HIP(hipMemcpy(plan->slice_row.p + slices, &total_ksteps, sizeof(int64_t), hipMemcpyHostToDevice));
    plan->n_rows_tab = total_ksteps;
    CST_TRY(plan->kstep_group.alloc(size_t(total_ksteps) + 1));
    kstep_groups_kernel<<<dim3(unsigned(div_up(slices, 256))), block>>>(slices, X->ptr[0].p, plan->slice_row.p,
                                                                       grp_off.p, total_ksteps, total_groups,
                                                                       plan->kstep_group.p);
    CST_HIP(hipGetLastError());
    CST_TRY(plan->pieces.alloc(size_t(plan->n_pieces)));
    fill_groups_kernel<<<dim3(unsigned(div_up(fibers, 256))), block>>>(
        fibers, slices, X->ptr[0].p, X->ptr[1].p, X->ptr[2].p, X->idx[1].p, X->idx[2].p, X->idx[3].p, X->vals.p,
        grp_off.p, plan->pieces.p);
    CST_HIP(hipGetLastError());
    CST_HIP(hipDeviceSynchronize());
    return CONSTSTN_OK;
}

// Cuts every slice (a range of units: leaves, fibers or rows) into items of about `split` units
// (at most max_pieces items per slice when max_pieces > 0); slices made of several items get
// partial-result slots.
static conststn_status build_items_core(int64_t slices, const int64_t *unit_ptr, int64_t split, int64_t max_pieces,
                                        int order, const int64_t *ptr0, const int64_t *ptr1, int64_t row_elems,
                                        DevBuf<SliceItem> &items, int64_t &n_items, int64_t &n_partials,
                                        int64_t &n_split, DevBuf<int32_t> &split_slices,
                                        DevBuf<int64_t> &split_first, DevBuf<int32_t> &split_count,
                                        DevBuf<double> &partial) {
    DevBuf<int64_t> pieces, part_cnt, is_split, item_off, part_off, split_rank;
    CST_TRY(pieces.alloc(slices));
    CST_TRY(part_cnt.alloc(slices));
    CST_TRY(is_split.alloc(slices));
    CST_TRY(item_off.alloc(slices));
    CST_TRY(part_off.alloc(slices));
    CST_TRY(split_rank.alloc(slices));
    const dim3 grid(unsigned(div_up(slices, 256))), block(256);
    ttmc_count_kernel<<<grid, block>>>(slices, unit_ptr, split, max_pieces, pieces.p, part_cnt.p, is_split.p);
    CST_HIP(hipGetLastError());
    CST_TRY(exscan(pieces.p, item_off.p, slices, &n_items));
    CST_TRY(exscan(part_cnt.p, part_off.p, slices, &n_partials));
    CST_TRY(exscan(is_split.p, split_rank.p, slices, &n_split));
    CST_TRY(items.alloc(size_t(n_items)));
    CST_TRY(split_slices.alloc(size_t(n_split)));
    CST_TRY(split_first.alloc(size_t(n_split)));
    CST_TRY(split_count.alloc(size_t(n_split)));
    CST_TRY(partial.alloc(size_t(n_partials) * size_t(row_elems)));
    ttmc_fill_kernel<<<grid, block>>>(slices, unit_ptr, pieces.p, item_off.p, part_off.p, split_rank.p, order, ptr0,
                                      ptr1, items.p, split_slices.p, split_first.p, split_count.p);
    CST_HIP(hipGetLastError());
    return CONSTSTN_OK;
}

// ---- TTMc order-3 streaming path: flat K-step table and workgroup batches ----------------------

__global__ void item_ksteps_kernel(int64_t n_items, const SliceItem *__restrict__ items, int64_t item_cost,
                                   int64_t *ksteps_of, int64_t *cost_of) {
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= n_items) return;
    const int64_t k = (items[i].end - items[i].begin + 3) / 4;
    ksteps_of[i] = k;
    cost_of[i] = k + item_cost;
}

// last i in [0, n) with off[i] <= x  (off ascending, off[0] <= x)
__device__ __forceinline__ int64_t last_le(const int64_t *__restrict__ off, int64_t n, int64_t x) {
    int64_t lo = 0, hi = n;
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (off[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ void fill_ksteps_kernel(int64_t n_ksteps, int64_t n_items, const SliceItem *__restrict__ items,
                                   const int64_t *__restrict__ kstep_off, const int32_t *__restrict__ idx0,
                                   int compact, KStepDesc *out) {
    const int64_t g = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (g >= n_ksteps) return;
    const int64_t i = last_le(kstep_off, n_items, g);
    const SliceItem it = items[i];
    const int64_t r0 = it.begin + 4 * (g - kstep_off[i]);
    const int64_t left = it.end - r0;
    const bool last = left <= 4;
    KStepDesc d;
    d.row0 = int32_t(r0);
    d.meta = int32_t(left < 4 ? left : 4) | (last ? 8 : 0);
    d.dest = 0;
    if (last) d.dest = it.dest < 0 ? (compact ? int64_t(it.slice) : int64_t(idx0[it.slice])) : ~it.dest;
    out[g] = d;
}

// Workgroup w starts at the first item whose cost prefix reaches the w-th cut: batches hold whole items.
// The cuts are `target` apart for the first n1 batches, a quarter of it for the next n2 and a sixteenth
// after that, so that the last workgroups to start are short ones and the chip drains evenly.
__global__ void stream_batches_kernel(int64_t n_wg, int64_t n_items, const int64_t *__restrict__ cost_off,
                                      const int64_t *__restrict__ kstep_off, int64_t target, int64_t n1, int64_t n2,
                                      int64_t n_ksteps, int32_t *wg_kstep) {
    const int64_t w = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (w > n_wg) return;
    if (w == n_wg) { wg_kstep[w] = int32_t(n_ksteps); return; }
    const int64_t t4 = target / 4 > 0 ? target / 4 : 1, t16 = target / 16 > 0 ? target / 16 : 1;
    const int64_t x = w < n1 ? w * target : (w < n1 + n2 ? n1 * target + (w - n1) * t4
                                                          : n1 * target + n2 * t4 + (w - n1 - n2) * t16);
    int64_t i = last_le(cost_off, n_items, x);
    if (cost_off[i] < x) ++i;                       // first item with prefix >= x
    wg_kstep[w] = i < n_items ? int32_t(kstep_off[i]) : int32_t(n_ksteps);
}

static conststn_status build_stream_tables(conststn_plan_s *plan) {
    const int64_t n_items = plan->n_items;
    plan->n_ksteps = plan->n_stream_wg = 0;
    if (n_items == 0) return CONSTSTN_OK;
    // an item costs its K-steps plus the store of its row block
    const int64_t item_cost = std::max<int64_t>(plan->opt("ttmc3_itemcost", 2), 0);
    const int64_t target = std::max<int64_t>(plan->opt("ttmc3_batch", 2048), 1);
    DevBuf<int64_t> ksteps_of, cost_of, kstep_off, cost_off;
    CST_TRY(ksteps_of.alloc(n_items));
    CST_TRY(cost_of.alloc(n_items));
    CST_TRY(kstep_off.alloc(n_items));
    CST_TRY(cost_off.alloc(n_items));
    const dim3 block(256);
    item_ksteps_kernel<<<dim3(unsigned(div_up(n_items, 256))), block>>>(n_items, plan->items.p, item_cost,
                                                                       ksteps_of.p, cost_of.p);
    CST_HIP(hipGetLastError());
    int64_t total_cost = 0;
    CST_TRY(exscan(ksteps_of.p, kstep_off.p, n_items, &plan->n_ksteps));
    CST_TRY(exscan(cost_of.p, cost_off.p, n_items, &total_cost));
    if (plan->n_ksteps >= (int64_t(1) << 31)) { set_error("more than 2^31 K-steps"); return CONSTSTN_EUNSUPPORTED; }
    CST_TRY(plan->ksteps.alloc(size_t(plan->n_ksteps)));
    fill_ksteps_kernel<<<dim3(unsigned(div_up(plan->n_ksteps, 256))), block>>>(
        plan->n_ksteps, n_items, plan->items.p, kstep_off.p, plan->X->idx[0].p, plan->compact ? 1 : 0, plan->ksteps.p);
    CST_HIP(hipGetLastError());
    // three quarters of the work in full batches, a fifth in quarter batches, the rest in sixteenths
    const int64_t t4 = std::max<int64_t>(target / 4, 1), t16 = std::max<int64_t>(target / 16, 1);
    const int64_t n1 = total_cost * 3 / 4 / target;
    const int64_t n2 = std::max<int64_t>(total_cost - n1 * target, 0) * 4 / 5 / t4;
    const int64_t n3 = div_up(std::max<int64_t>(total_cost - n1 * target - n2 * t4, 0), t16);
    plan->n_stream_wg = n1 + n2 + n3;
    CST_TRY(plan->wg_kstep.alloc(size_t(plan->n_stream_wg) + 1));
    stream_batches_kernel<<<dim3(unsigned(div_up(plan->n_stream_wg + 1, 256))), block>>>(
        plan->n_stream_wg, n_items, cost_off.p, kstep_off.p, target, n1, n2, plan->n_ksteps, plan->wg_kstep.p);
    CST_HIP(hipGetLastError());
    CST_HIP(hipDeviceSynchronize());
    return CONSTSTN_OK;
}

// Order-4 matrix-core path: one wavefront per item, so the longest items go first (the last round of
// workgroups then holds the short ones).  Cost = matrix instructions: one per group, sixteen per K-step.
__global__ void item_cost_keys_kernel(int64_t n_items, const SliceItem *__restrict__ items,
                                      const int64_t *__restrict__ kstep_group, uint64_t *keys, uint32_t *ids) {
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= n_items) return;
    const int64_t cost = (kstep_group[items[i].end] - kstep_group[items[i].begin]) + 16 * (items[i].end - items[i].begin);
    keys[i] = uint64_t(0xffffffffu) - uint64_t(cost < 0xffffffffll ? cost : 0xffffffffll);
    ids[i] = uint32_t(i);
}

__global__ void permute_items_kernel(int64_t n_items, const uint32_t *__restrict__ order,
                                     const SliceItem *__restrict__ in, SliceItem *out) {
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n_items) out[i] = in[order[i]];
}

static conststn_status order_items_by_cost(conststn_plan_s *plan) {
    const int64_t n = plan->n_items;
    if (n >= (int64_t(1) << 32)) return CONSTSTN_OK;
    DevBuf<uint64_t> ka, kb;
    DevBuf<uint32_t> ia, ib;
    DevBuf<SliceItem> sorted;
    CST_TRY(ka.alloc(n));
    CST_TRY(kb.alloc(n));
    CST_TRY(ia.alloc(n));
    CST_TRY(ib.alloc(n));
    CST_TRY(sorted.alloc(n));
    const dim3 grid(unsigned(div_up(n, 256))), block(256);
    item_cost_keys_kernel<<<grid, block>>>(n, plan->items.p, plan->kstep_group.p, ka.p, ia.p);
    CST_HIP(hipGetLastError());
    const uint64_t *ks = nullptr;
    const uint32_t *order = nullptr;
    CST_TRY(radix_sort_pairs_u64(ka.p, kb.p, ia.p, ib.p, n, 32, hipStream_t(0), &ks, &order));
    permute_items_kernel<<<grid, block>>>(n, order, plan->items.p, sorted.p);
    CST_HIP(hipGetLastError());
    CST_HIP(hipMemcpy(plan->items.p, sorted.p, size_t(n) * sizeof(SliceItem), hipMemcpyDeviceToDevice));
    CST_HIP(hipDeviceSynchronize());
    return CONSTSTN_OK;
}

conststn_status build_ttmc_tables(conststn_plan_s *plan) {
    const conststn_csf_s *X = plan->X;
    const int64_t slices = X->nodes[0];
    CST_TRY(make_slice_leaf(plan));
    plan->n_items = plan->n_partials = plan->n_split = 0;
    if (slices == 0) return CONSTSTN_OK;
    int order = X->order;
    // order 3 splits by leaves, order 4 by level-1 fibers (each carries a whole sub-tree)
    const int64_t *unit_ptr = order == 3 ? plan->slice_leaf.p : X->ptr[0].p;
    int64_t split = order == 3 ? plan->opt("ttmc3_split", 4096) : plan->opt("ttmc4_split", 256);
    // ranks that are multiples of 16 take the MFMA kernel, whose items are ranges of rows
    plan->use_rows = order == 3 && plan->rank_of_level[1] % 16 == 0 && plan->rank_of_level[2] % 16 == 0 &&
                     plan->rank_of_level[1] <= 64 && plan->rank_of_level[2] <= 64 &&
                     plan->opt("ttmc3_mfma", 1) == 1;
    if (plan->use_rows) {
        CST_TRY(build_rows(plan));
        unit_ptr = plan->slice_row.p;
        // larger items mean fewer partial row blocks for the fix-up pass to add; keep at least
        // about 8192 items for the chip
        split = plan->opt("ttmc3_rowsplit", std::min<int64_t>(std::max<int64_t>(plan->n_rows_tab / 8192, 256), 2048));
        order = 0;                                   // items carry no 'first fiber'
    }
    // (extents below 2^25: the matrix-core kernel reaches the factor rows with 32-bit byte offsets)
    const conststn_csf_s *X4 = plan->X;
    const bool small_extents = order != 4 || (X4->dims[X4->mode_order[1]] < (int64_t(1) << 25) &&
                                              X4->dims[X4->mode_order[2]] < (int64_t(1) << 25) &&
                                              X4->dims[X4->mode_order[3]] < (int64_t(1) << 25));
    if (order == 4 && plan->rank_of_level[1] == 16 && plan->rank_of_level[2] == 16 && small_extents &&
        plan->rank_of_level[3] == 16 && plan->opt("ttmc4_mfma", 1) == 1) {
        plan->use_rows = true;
        CST_TRY(build_piece_groups(plan));
        unit_ptr = plan->slice_row.p;                 // items are ranges of K-steps (four fibers each)
        // (with the items ordered by cost their length matters little: 2.95 ms per launch on the 40 M-nonzero
        // tensor for 64 to 128 K-steps per item, and the fewer partial row blocks the shorter the fix-up pass)
        split = plan->opt("ttmc4_ksplit", std::min<int64_t>(std::max<int64_t>(plan->n_rows_tab / 8192, 64), 128));
    }
    CST_TRY(build_items_core(slices, unit_ptr, split, 0, order, X->ptr[0].p, X->ptr[1].p, plan->row_elems,
                             plan->items, plan->n_items, plan->n_partials, plan->n_split, plan->split_slices,
                             plan->split_first, plan->split_count, plan->partial));
    CST_HIP(hipDeviceSynchronize());
    if (X->order == 4 && plan->use_rows && plan->n_items > 1) CST_TRY(order_items_by_cost(plan));
    // streaming form of the order-3 matrix-core path: R3 of 32 or 64 (two column tiles per multiplying
    // wavefront), rows and output blocks reachable with the table's 32-bit fields
    plan->use_stream = X->order == 3 && plan->use_rows && (plan->rank_of_level[2] == 32 || plan->rank_of_level[2] == 64) &&
                       plan->opt("ttmc3_stream", 1) == 1;
    if (plan->use_stream) {
        int np = int(plan->opt("ttmc3_producers", 4));
        plan->stream_producers = np == 2 || np == 3 || np == 6 || np == 8 ? np : 4;
        CST_TRY(build_stream_tables(plan));
    }
    return CONSTSTN_OK;
}

// ---- three-tensor network: where does index k sit among W's root nodes ---------------------

__global__ void fill_i64_kernel(int64_t *p, int64_t n, int64_t v) {
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

__global__ void w_roots_kernel(int64_t roots, const int32_t *__restrict__ idx0, int64_t *root_of_k) {
    const int64_t p = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (p < roots) root_of_k[idx0[p]] = p;
}

// ---- three-tensor network, tiled path: W re-stored as dense 16 x 16 (l, m) tiles -------------
//
// Below one root k of W the (l, m) plane is cut into tiles of 16 x 16; only the tiles that hold
// a nonzero are kept, zero-filled elsewhere.  Per (root, l tile): a bit mask of the m tiles
// present and the index of the first of them (tiles of one l tile are stored in m order).
// Inside a tile the 256 values are laid out for the consumer's matrix instruction: value
// (l', m') with l' = 4v + s sits at  (v/2)*128 + (s*16 + m')*2 + (v&1), so that lane (s, m') of
// a wavefront reads its four values as two 16-byte words, the wavefront 1 KB at a time.

__device__ inline int64_t root_of_fiber(const int64_t *__restrict__ ptr0, int64_t roots, int64_t g) {
    int64_t lo = 0, hi = roots;                 // last root with ptr0[root] <= g
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (ptr0[mid] <= g) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ void w_tile_mask_kernel(int64_t fibers, int64_t roots, int64_t LT,
                                   const int64_t *__restrict__ ptr0, const int64_t *__restrict__ ptr1,
                                   const int32_t *__restrict__ idx1, const int32_t *__restrict__ idx2,
                                   uint32_t *mask) {
    const int64_t g = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (g >= fibers) return;
    const int64_t r = root_of_fiber(ptr0, roots, g);
    uint32_t mine = 0;
    for (int64_t e = ptr1[g]; e < ptr1[g + 1]; ++e) mine |= 1u << (idx2[e] >> 4);
    atomicOr(&mask[r * LT + (idx1[g] >> 4)], mine);
}

__global__ void w_tile_count_kernel(int64_t n, const uint32_t *__restrict__ mask, int64_t *cnt) {
    const int64_t x = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (x < n) cnt[x] = __popc(mask[x]);
}

__global__ void w_tile_fill_kernel(int64_t fibers, int64_t roots, int64_t LT,
                                   const int64_t *__restrict__ ptr0, const int64_t *__restrict__ ptr1,
                                   const int32_t *__restrict__ idx1, const int32_t *__restrict__ idx2,
                                   const double *__restrict__ vals, const uint32_t *__restrict__ mask,
                                   const int64_t *__restrict__ first, double *tiles) {
    const int64_t g = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (g >= fibers) return;
    const int64_t r = root_of_fiber(ptr0, roots, g);
    const int32_t l = idx1[g];
    const int64_t cell = r * LT + (l >> 4);
    const uint32_t present = mask[cell];
    const int64_t base = first[cell];
    const int lp = l & 15, v = lp >> 2, sl = lp & 3;
    for (int64_t e = ptr1[g]; e < ptr1[g + 1]; ++e) {
        const int32_t m = idx2[e];
        const int mt = m >> 4;
        const int64_t tile = base + __popc(present & ((1u << mt) - 1u));
        tiles[tile * 256 + (v >> 1) * 128 + (sl * 16 + (m & 15)) * 2 + (v & 1)] = vals[e];
    }
}

__global__ void w_first_u32_kernel(int64_t n, const int64_t *__restrict__ first, uint32_t *out) {
    const int64_t x = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (x < n) out[x] = uint32_t(first[x]);
}

// Leaves of U per (k chunk, group of 16 slices) pair: the workgroups of the tiled kernels take the pairs
// in falling order of it, so that the last round of workgroups holds the light ones.
__global__ void sp_pair_cost_kernel(int64_t fibers, int64_t slices, const int64_t *__restrict__ ptr0,
                                    const int64_t *__restrict__ ptr1, const int32_t *__restrict__ idx1,
                                    int64_t k_per, int n_groups, unsigned *cost) {
    const int64_t f = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (f >= fibers) return;
    const int64_t s = root_of_fiber(ptr0, slices, f);
    const int64_t pair = (int64_t(idx1[f]) / k_per) * n_groups + s / kSpGroup;
    atomicAdd(&cost[pair], unsigned(ptr1[f + 1] - ptr1[f]));
}

__global__ void sp_pair_keys_kernel(int64_t n, const unsigned *__restrict__ cost, uint64_t *keys, uint32_t *ids) {
    const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i >= n) return;
    keys[i] = uint64_t(0xffffffffu - cost[i]);
    ids[i] = uint32_t(i);
}

static conststn_status build_sp_wg_order(conststn_plan_s *plan) {
    const conststn_csf_s *U = plan->X;
    const int64_t groups = div_up(U->nodes[0], kSpGroup), n = groups * plan->sp_kc;
    if (n <= 1 || n >= (int64_t(1) << 31) || U->nodes[1] == 0) return CONSTSTN_OK;
    DevBuf<unsigned> cost;
    DevBuf<uint64_t> ka, kb;
    DevBuf<uint32_t> ia, ib;
    CST_TRY(cost.alloc(n));
    CST_TRY(ka.alloc(n));
    CST_TRY(kb.alloc(n));
    CST_TRY(ia.alloc(n));
    CST_TRY(ib.alloc(n));
    const dim3 block(256);
    fill_i32_kernel<<<dim3(unsigned(div_up(n, 256))), block>>>(reinterpret_cast<int32_t *>(cost.p), n, 0);
    sp_pair_cost_kernel<<<dim3(unsigned(div_up(U->nodes[1], 256))), block>>>(
        U->nodes[1], U->nodes[0], U->ptr[0].p, U->ptr[1].p, U->idx[1].p, plan->sp_k_per, int(groups), cost.p);
    sp_pair_keys_kernel<<<dim3(unsigned(div_up(n, 256))), block>>>(n, cost.p, ka.p, ia.p);
    CST_HIP(hipGetLastError());
    const uint64_t *ks = nullptr;
    const uint32_t *order = nullptr;
    CST_TRY(radix_sort_pairs_u64(ka.p, kb.p, ia.p, ib.p, n, 32, hipStream_t(0), &ks, &order));
    CST_TRY(plan->sp_wg_order.alloc(size_t(n)));
    CST_HIP(hipMemcpy(plan->sp_wg_order.p, order, size_t(n) * sizeof(uint32_t), hipMemcpyDeviceToDevice));
    CST_HIP(hipDeviceSynchronize());
    return CONSTSTN_OK;
}

static conststn_status build_w_tiles(conststn_plan_s *plan) {
    const conststn_csf_s *U = plan->X, *W = plan->W;
    const int64_t J = U->dims[U->mode_order[2]];
    const int64_t L = W->dims[W->mode_order[1]], M = W->dims[W->mode_order[2]];
    const int64_t K = W->dims[W->mode_order[0]];
    plan->w_tiled = false;
    if (plan->opt("sptn3_tiled", 1) == 0) return CONSTSTN_OK;          // 0 = baseline kernel
    if (M > 16 * kSpMaxMTiles || J > kSpMaxJ || J * L >= (int64_t(1) << 29) || W->nnz == 0 || U->nnz == 0)
        return CONSTSTN_OK;
    const int64_t roots = W->nodes[0], fibers = W->nodes[1];
    const int64_t LT = div_up(L, 16), cells = roots * LT;
    CST_TRY(plan->w_tile_mask.alloc(size_t(cells)));
    const dim3 block(256), fgrid(unsigned(div_up(fibers, 256))), cgrid(unsigned(div_up(cells, 256)));
    fill_i32_kernel<<<cgrid, block>>>(reinterpret_cast<int32_t *>(plan->w_tile_mask.p), cells, 0);
    CST_HIP(hipGetLastError());
    w_tile_mask_kernel<<<fgrid, block>>>(fibers, roots, LT, W->ptr[0].p, W->ptr[1].p, W->idx[1].p,
                                         W->idx[2].p, plan->w_tile_mask.p);
    CST_HIP(hipGetLastError());
    DevBuf<int64_t> cnt, first;
    CST_TRY(cnt.alloc(size_t(cells)));
    CST_TRY(first.alloc(size_t(cells)));
    w_tile_count_kernel<<<cgrid, block>>>(cells, plan->w_tile_mask.p, cnt.p);
    CST_HIP(hipGetLastError());
    int64_t n_tiles = 0;
    CST_TRY(exscan(cnt.p, first.p, cells, &n_tiles));
    if (n_tiles >= (int64_t(1) << 31) - 1) return CONSTSTN_OK;
    // The dense tiles pay off when they are reasonably full.  A scattered W (about one nonzero per
    // tile) would be blown up 256-fold: below one nonzero in sixteen cells, or when the tiles do not fit
    // the free device memory, the baseline kernel (which needs no tiles) takes the plan instead.
    size_t free_b = 0, total_b = 0;
    CST_HIP(hipMemGetInfo(&free_b, &total_b));
    if (plan->opt("sptn3_tiled", 1) != 2 && (n_tiles * 16 > W->nnz || size_t(n_tiles + 1) * 2048 > free_b / 2)) {
        plan->w_tile_mask.release();
        return CONSTSTN_OK;
    }
    plan->n_w_tiles = n_tiles;
    // one more, all-zero tile at the end: the target of loads that have nothing to fetch
    CST_TRY(plan->w_tiles.alloc(size_t(n_tiles + 1) * 256));
    CST_TRY(zero_fill(plan->w_tiles.p, (n_tiles + 1) * 256, hipStream_t(0)));
    w_tile_fill_kernel<<<fgrid, block>>>(fibers, roots, LT, W->ptr[0].p, W->ptr[1].p, W->idx[1].p,
                                         W->idx[2].p, W->vals.p, plan->w_tile_mask.p, first.p,
                                         plan->w_tiles.p);
    CST_HIP(hipGetLastError());
    CST_TRY(plan->w_tile_first.alloc(size_t(cells)));
    w_first_u32_kernel<<<cgrid, block>>>(cells, first.p, plan->w_tile_first.p);
    CST_HIP(hipGetLastError());
    // slices go in groups of 16; the k range is cut into chunks so that the grid fills the chip
    const int64_t groups = div_up(U->nodes[0], kSpGroup);
    int64_t want = plan->opt("sptn3_wgs", 8000);
    int64_t n_kc = std::min<int64_t>(std::max<int64_t>(div_up(want, groups), 1), std::min<int64_t>(K, 64));
    plan->sp_k_per = div_up(K, n_kc);
    plan->sp_kc = int(div_up(K, plan->sp_k_per));
    if (plan->sp_kc > 1)
        CST_TRY(plan->partial.alloc(size_t(plan->sp_kc) * size_t(U->nodes[0]) * size_t(M)));
    plan->w_tiled = true;
    CST_TRY(build_sp_wg_order(plan));
    plan->sp_two_waves = plan->opt("sptn3_waves", 2) == 2 && sptn3_two_waves_fit(int((J + 31) / 32));
    return CONSTSTN_OK;
}

conststn_status build_sptn3_tables(conststn_plan_s *plan) {
    const conststn_csf_s *W = plan->W;
    const int64_t K = W->dims[W->mode_order[0]];
    CST_TRY(plan->w_root_of_k.alloc(size_t(K)));
    fill_i64_kernel<<<dim3(unsigned(div_up(K, 256))), dim3(256)>>>(plan->w_root_of_k.p, K, -1);
    CST_HIP(hipGetLastError());
    if (W->nodes[0] > 0) {
        w_roots_kernel<<<dim3(unsigned(div_up(W->nodes[0], 256))), dim3(256)>>>(W->nodes[0], W->idx[0].p,
                                                                              plan->w_root_of_k.p);
        CST_HIP(hipGetLastError());
    }
    CST_TRY(build_w_tiles(plan));
    CST_HIP(hipDeviceSynchronize());
    return prepare_sptn3_launch(plan);
}

}  // namespace cst
