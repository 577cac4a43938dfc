// Generic executor for contraction trees over ONE CSF tensor and dense operands -- any order,
// any rank extents, any legal loop order and fusion choice, any output mode (Sec. 2.2 / 4.2: a
// schedule is a tree of binary contractions; fusion changes the size of the intermediates, never
// their values).
//
// A tensor on the path from the CSF operand X to the result is stored in one of two ways:
//   by prefix  indexed by a PREFIX of X's CSF levels plus dense indices: one dense block per CSF
//              node of that depth ("sparse like X above, dense below" -- the sparsity structure
//              Sec. 2.1 assigns to a contraction result, restricted to prefixes);
//   dense      when it keeps CSF indices that are not a prefix (an output mode other than the
//              root, Sec. 5.3): a dense array over the extents of all its indices.
// A product of two dense tensors whose leading indices are a CSF prefix, and whose consumer joins it
// with a tensor that is sparse like X to at least that depth, is computed by prefix too ("lifted"):
// inside the fused loop nest of Fig. 3b only the entries at X's nodes are ever read.
//
// Two kernels.  A statement
//        out[x_0..x_{d'-1}, O...] = in[x_0..x_{d-1}, I...] * F[...]        (d' <= d)
// whose result is stored by prefix and whose other input F is a dense tensor not indexed by a kept
// level runs with one thread per result element, which walks the CSF subtree below its node and
// the contracted dense indices in a fixed order: deterministic, no atomics.  Every other statement
// (a result that keeps a non-prefix level, an input indexed by a kept level, a lifted input or
// result) runs with one thread per (node of the deeper input, dense result element): the thread
// finds its ancestors by binary search in the pointer arrays, forms its term and, where several
// nodes meet in one result element, adds it with a hardware fp64 atomic.  Statements whose two
// inputs are both dense and not lifted use the first kernel with an empty prefix.
//
// A sum over more than CONSTSTN_GENERIC_SPAN nodes below one result node (a power-law slice) is
// not left to a single thread: the node's children are cut into segments, the first kernel writes
// one partial sum per (segment, element) and a second pass adds them in segment order --
// still a fixed order.
//
// Intermediates are held whole in device memory.  This is the slow, always-applicable path; the
// tuned kernels of the other files take the schedules they match.
#include <algorithm>
#include <set>

#include "plan.hpp"
#include <type_traits>

namespace cst {

__global__ void __launch_bounds__(256)
generic_stmt_kernel(GenStmt g) {
    const int64_t gid = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const bool segmented = g.n_segs > 0;
    if (gid >= (segmented ? g.n_segs : g.out_nodes) * g.out_block) return;
    const int64_t unit = gid / g.out_block;                 // a result node, or a segment of one
    const int64_t p = segmented ? g.seg[3 * unit] : unit;
    int64_t rem = gid - unit * g.out_block;
    int64_t in_off = 0, f_off0 = 0, out_off = 0;
    for (int q = g.n_out - 1; q >= 0; --q) {
        const int64_t o = rem % g.extent[q];
        rem /= g.extent[q];
        in_off += o * g.in_stride[q];
        f_off0 += o * g.f_stride[q];
        out_off += o * g.out_stride[q];
    }
    // contracted dense indices: mixed-radix counter with running offsets
    const int nr = g.n_red;
    auto inner = [&](int64_t node, int64_t f_off, double &acc) {
        // X itself is the case in_block = 1 with no dense index: one value per leaf
        const int64_t base = node * g.in_block + in_off;
        int64_t cnt[kGenMaxIdx] = {0};
        int64_t io = 0, fo = 0;
        for (;;) {
            acc = fma(g.in[base + io], g.f[f_off + fo], acc);
            int q = g.n_out + nr - 1;
            for (; q >= g.n_out; --q) {
                io += g.in_stride[q];
                fo += g.f_stride[q];
                if (++cnt[q] < g.extent[q]) break;
                io -= g.in_stride[q] * g.extent[q];
                fo -= g.f_stride[q] * g.extent[q];
                cnt[q] = 0;
            }
            if (q < g.n_out) break;
        }
    };
    double acc = 0.0;
    const int D = g.d_in - g.d_out;               // CSF levels summed over
    if (D == 0) {
        inner(p, f_off0, acc);
    } else if (D == 1 && nr == 0) {
        // the common shape (one level summed, no dense index summed) without the bookkeeping arrays,
        // which the compiler can only keep in scratch memory
        int64_t c0, c1;
        if (segmented) { c0 = g.seg[3 * unit + 1]; c1 = g.seg[3 * unit + 2]; }
        else if (g.d_out == 0) { c0 = 0; c1 = g.roots; }
        else { c0 = g.ptr[g.d_out - 1][p]; c1 = g.ptr[g.d_out - 1][p + 1]; }
        const int32_t *ix = g.idx[g.d_out];
        const int64_t fs = g.f_level_stride[g.d_out];
        // eight children at a time: their loads are in flight together, the sum keeps its order
        int64_t c = c0;
        for (; c + 8 <= c1; c += 8) {
            int32_t iv[8];
            double xv[8], yv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) iv[u] = ix[c + u];
#pragma unroll
            for (int u = 0; u < 8; ++u) xv[u] = g.in[(c + u) * g.in_block + in_off];
#pragma unroll
            for (int u = 0; u < 8; ++u) yv[u] = g.f[f_off0 + int64_t(iv[u]) * fs];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc = fma(xv[u], yv[u], acc);
        }
        for (; c < c1; ++c)
            acc = fma(g.in[c * g.in_block + in_off], g.f[f_off0 + int64_t(ix[c]) * fs], acc);
    } else {
        int64_t cur[CONSTSTN_MAX_ORDER], end[CONSTSTN_MAX_ORDER], foff[CONSTSTN_MAX_ORDER];
        int l = 0;
        if (segmented) { cur[0] = g.seg[3 * unit + 1]; end[0] = g.seg[3 * unit + 2]; }
        else if (g.d_out == 0) { cur[0] = 0; end[0] = g.roots; }
        else { cur[0] = g.ptr[g.d_out - 1][p]; end[0] = g.ptr[g.d_out - 1][p + 1]; }
        foff[0] = f_off0;
        for (;;) {
            if (cur[l] < end[l]) {
                const int L = g.d_out + l;
                const int64_t c = cur[l]++;
                const int64_t fo = foff[l] + int64_t(g.idx[L][c]) * g.f_level_stride[L];
                if (l == D - 1) {
                    inner(c, fo, acc);
                } else {
                    foff[l + 1] = fo;
                    cur[l + 1] = g.ptr[L][c];
                    end[l + 1] = g.ptr[L][c + 1];
                    ++l;
                }
            } else {
                if (l == 0) break;
                --l;
            }
        }
    }
    if (segmented) { g.partial[unit * g.out_block + out_off] = acc; return; }
    const int64_t row = g.scatter_rows ? int64_t(g.idx[0][p]) : p;
    g.out[row * g.out_block + out_off] = acc;
}

// A fused producer / consumer pair (Sec. 2.2, Fig. 3b) in the shape the chains of Sec. 5.2 have:
//        T[x_0..x_d, O...]   = X[x_0..x_d, x_{d+1}] * F1[x_{d+1}, O'...]           (X's leaf level summed)
//        out[x_0..x_{d-1}, O...] = T[x_0..x_d, O...] * F[x_d, O''...]              (level d summed)
// with the same dense indices O on both results.  The intermediate is one scalar per thread: a
// group of W lanes owns one result node (or one segment of its leaves) and W of its result elements,
// lane j element j.  What every lane of the group needs alike -- the leaves' indices and values, the
// fibers' ends and indices -- is read once, lane j taking the j-th leaf (fiber) of a window of W, and
// handed round with lane shuffles; only the rows of the two factors are read by every lane.  Fixed
// order of addition, no atomics.
// SMALL: both factors are below 2 GiB with fewer than 2^24 rows of fewer than 2^24 bytes, so that a row's
// byte offset is one 24-bit multiply-add instead of 64-bit arithmetic.
// V: result elements per lane, 1 or 2.  Two when the plan found that the innermost dense index is even,
// runs with stride 1 through every factor and the result, and every row begins on 16 bytes: a lane then
// reads its two entries of a row with one 16-byte load, and a gather instruction costs the address unit
// about as much for 16 bytes per lane as for 8.
template <int V> struct GenVals { double v[V]; };
template <int W, bool SMALL, int U, int V>
__global__ void __launch_bounds__(256)
generic_fused_kernel(GenStmt g) {
    using offs = typename std::conditional<SMALL, uint32_t, int64_t>::type;
    using vals = GenVals<V>;
    const int64_t grp = (int64_t(blockIdx.x) * 256 + threadIdx.x) / W;
    const int j = int(threadIdx.x) % W;
    const bool segmented = g.n_segs > 0;
    const int64_t chunks = (g.out_block + W * V - 1) / (W * V);
    if (grp >= (segmented ? g.n_segs : g.out_nodes) * chunks) return;        // whole groups leave together
    const int64_t unit = grp / chunks;
    const int64_t p = segmented ? g.seg[3 * unit] : unit;
    const int64_t o_lin = ((grp - unit * chunks) * W + j) * V;
    const bool live = o_lin < g.out_block;                   // idle lanes compute element 0 and store nothing
    int64_t rem = live ? o_lin : 0;
    int64_t f_off0 = 0, f1_off0 = 0, out_off = 0, fu_off0[U + 1] = {};
    for (int q = g.n_out - 1; q >= 0; --q) {
        const int64_t o = rem % g.extent[q];
        rem /= g.extent[q];
        f_off0 += o * g.f_stride[q];
        f1_off0 += o * g.f1_stride[q];
        out_off += o * g.out_stride[q];
#pragma unroll
        for (int v = 0; v < U; ++v) fu_off0[v] += o * g.fu_stride[v][q];
    }
    // The levels above the leaves are numbered from the fibers (0) up to the summed level (U).  For
    // each: the factor's base, this lane's byte offset in a row of it, the rows' stride in bytes.
    const int fiber_level = g.d_in - 1;
    const char *lb[U + 1];
    offs l_lane[U + 1], l_fs[U + 1];
#pragma unroll
    for (int v = 0; v < U; ++v) {
        lb[v] = reinterpret_cast<const char *>(g.fu[v]);
        l_lane[v] = offs(fu_off0[v] * 8);
        l_fs[v] = offs(g.fu_level_stride[v] * 8);
    }
    lb[U] = reinterpret_cast<const char *>(g.f);
    l_lane[U] = offs(f_off0 * 8);
    l_fs[U] = offs(g.f_level_stride[g.d_out] * 8);
    const offs f1_lane = offs(f1_off0 * 8), fs1 = offs(g.f1_level_stride * 8);
    const char *f1b = reinterpret_cast<const char *>(g.f1);
    auto row = [](const char *base, int32_t i, offs stride, offs lane) -> vals {
        const char *at;
        if constexpr (SMALL) at = base + (__umul24(uint32_t(i), stride) + lane);
        else at = base + (int64_t(i) * stride + lane);
        vals r;
        if constexpr (V == 2) {
            const double2 x = *reinterpret_cast<const double2 *>(at);
            r.v[0] = x.x;
            r.v[1] = x.y;
        } else {
            r.v[0] = *reinterpret_cast<const double *>(at);
        }
        return r;
    };
    auto zero = []() { vals r; for (int e = 0; e < V; ++e) r.v[e] = 0.0; return r; };
    auto fma_s = [](double x, const vals &y, vals &acc) { for (int e = 0; e < V; ++e) acc.v[e] = fma(x, y.v[e], acc.v[e]); };
    auto fma_v = [](const vals &x, const vals &y, vals &acc) { for (int e = 0; e < V; ++e) acc.v[e] = fma(x.v[e], y.v[e], acc.v[e]); };
    int64_t c0, c1;                                          // the result node's children
    if (g.d_out == 0) { c0 = 0; c1 = g.roots; }
    else { c0 = g.ptr[g.d_out - 1][p]; c1 = g.ptr[g.d_out - 1][p + 1]; }
    const int32_t *ix = g.idx[fiber_level];
    const int64_t *lptr = g.ptr[fiber_level];                // X's leaves below each fiber
    // A segment is a range of leaves and may begin and end inside a fiber, or inside a node of a level
    // above: then the node's factor multiplies each part of its sum, and the second pass adds the parts.
    int64_t e0 = 0, e_end = 0;
    if (c0 < c1) {
        if (segmented) { e0 = g.seg[3 * unit + 1]; e_end = g.seg[3 * unit + 2]; }
        else if (U == 0) { e0 = lptr[c0]; e_end = lptr[c1]; }
        else if (g.out_leaf) { e0 = g.out_leaf[p]; e_end = g.out_leaf[p + 1]; }
        else e_end = g.nodes[g.d_in];
    }
    constexpr int kFar = 1 << 30;                            // positions count from e0 and saturate here
    auto near = [&](int64_t e) { const int64_t d = e - e0; return d < kFar ? int(d) : kFar; };
    const int n_total = near(e_end);                         // the plan keeps a unit's leaves below kFar
    vals s[U + 1];                                           // running sums: s[v] over the finished children of the
#pragma unroll
    for (int v = 0; v <= U; ++v) s[v] = zero();
    if (n_total > 0) {                                       // current node of level v + 1 (s[U]: of the result node)
        // the last node of [lo, hi) whose first leaf is not after e0
        auto holder = [&](const int64_t *first_leaf, int64_t lo, int64_t hi) {
            while (hi - lo > 1) {
                const int64_t mid = lo + ((hi - lo) >> 1);
                if (first_leaf[mid] <= e0) lo = mid; else hi = mid;
            }
            return lo;
        };
        // levels above the fibers: the current node, where it ends, its factor, and the same one node ahead
        int64_t cu[U + 1];
        int endu[U + 1], endu2[U + 1];
        vals fvu[U + 1], fvu2[U + 1];
        auto upper_ahead = [&](int v) {                      // (endu2, fvu2) of node cu + 1 of level v
            const int L = fiber_level - v;
            if (cu[v] + 1 >= g.nodes[L]) { endu2[v] = kFar; return; }
            endu2[v] = near(g.leaf_end[v - 1][cu[v] + 2]);
            fvu2[v] = row(lb[v], g.idx[L][cu[v] + 1], l_fs[v], l_lane[v]);
        };
#pragma unroll
        for (int v = U; v >= 1; --v) {
            const int L = fiber_level - v;
            const int64_t lo = segmented ? holder(g.leaf_end[v - 1], c0, c1) : c0;
            cu[v] = lo;
            endu[v] = near(g.leaf_end[v - 1][lo + 1]);
            fvu[v] = row(lb[v], g.idx[L][lo], l_fs[v], l_lane[v]);
            upper_ahead(v);
            c0 = g.ptr[L][lo];
            c1 = g.ptr[L][lo + 1];
        }
        int64_t c = segmented ? holder(lptr, c0, c1) : c0;   // the fiber that holds leaf e0
        if (U > 0) c1 = g.nodes[fiber_level];                // fibers past the unit's last end at or after its last leaf
        const int32_t *lix = g.idx[g.d_in] + e0;
        const double *lx = g.in + e0;
        // window of W fibers from cw on: lane j holds the end and the index of fiber cw + j
        int64_t cw = c;
        int w_end, w_ix;
        auto load_fibers = [&]() {
            const int64_t cc = cw + j < c1 ? cw + j : c1 - 1;
            w_end = near(lptr[cc + 1]);
            w_ix = ix[cc];
        };
        load_fibers();
        int next = __shfl(w_end, 0, W);                      // end of the current fiber, its factor; then the same one fiber ahead
        vals fv = row(lb[0], __shfl(w_ix, 0, W), l_fs[0], l_lane[0]);
        int next2 = kFar;
        vals fv2 = zero();
        auto look_ahead = [&]() {                            // (next2, fv2) for fiber c + 1
            if (c + 1 >= c1) { next2 = kFar; return; }
            if (c + 1 - cw == W) { cw = c + 1; load_fibers(); }
            const int k = int(c + 1 - cw);
            next2 = __shfl(w_end, k, W);
            fv2 = row(lb[0], __shfl(w_ix, k, W), l_fs[0], l_lane[0]);
        };
        look_ahead();
        // window of W leaves: lane j holds leaf ew + j; the next window is read while this one is summed
        int32_t l_ix, l_ix2;
        double l_x, l_x2;
        auto load_leaves = [&](int ew, int32_t &iv, double &xv) {
            const bool in = ew + j < n_total;
            iv = in ? lix[ew + j] : 0;
            xv = in ? lx[ew + j] : 0.0;
        };
        load_leaves(0, l_ix, l_x);
        vals t = zero();
        for (int ew = 0; ew < n_total; ew += W) {
            load_leaves(ew + W, l_ix2, l_x2);
            const int n = n_total - ew < W ? n_total - ew : W;
            vals yv[4], yv2[4];                              // rows of F1 four leaves at a time, one batch ahead
#pragma unroll
            for (int k = 0; k < 4; ++k) yv[k] = row(f1b, __shfl(l_ix, k, W), fs1, f1_lane);      // past the end: row 0, never added
            for (int u0 = 0; u0 < n; u0 += 4) {
                if (u0 + 4 < n) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) yv2[k] = row(f1b, __shfl(l_ix, u0 + 4 + k, W), fs1, f1_lane);
                }
                double xv[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) xv[k] = __shfl(l_x, u0 + k, W);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if (u0 + k < n) {
                        const int pos = ew + u0 + k;
                        if (pos >= next) {                   // the fiber ended (every fiber of a CSF has a leaf): its sum
                            fma_v(t, fv, s[0]);              // times the factor of its level
                            t = zero();
                            ++c;
                            next = next2;
                            fv = fv2;
                            look_ahead();
                            bool up = true;                  // and so for each level above whose node ended with it
#pragma unroll
                            for (int v = 1; v <= U; ++v) {
                                if (up && pos >= endu[v]) {
                                    fma_v(s[v - 1], fvu[v], s[v]);
                                    s[v - 1] = zero();
                                    ++cu[v];
                                    endu[v] = endu2[v];
                                    fvu[v] = fvu2[v];
                                    upper_ahead(v);
                                } else {
                                    up = false;
                                }
                            }
                        }
                        fma_s(xv[k], yv[k], t);
                    }
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) yv[k] = yv2[k];
            }
            l_ix = l_ix2;
            l_x = l_x2;
        }
        fma_v(t, fv, s[0]);
#pragma unroll
        for (int v = 1; v <= U; ++v) fma_v(s[v - 1], fvu[v], s[v]);
    }
    if (!live) return;
    const int64_t row_out = segmented ? unit : (g.scatter_rows ? int64_t(g.idx[0][p]) : p);
    double *dst = (segmented ? g.partial : g.out) + row_out * g.out_block + out_off;
    if constexpr (V == 2) *reinterpret_cast<double2 *>(dst) = make_double2(s[U].v[0], s[U].v[1]);
    else dst[0] = s[U].v[0];
}

template <int W, int U>
static void launch_fused_u(const GenStmt &g, bool pairs, dim3 grid, hipStream_t stream) {
    if (pairs) {
        if (g.fused_small) generic_fused_kernel<W, true, U, 2><<<grid, dim3(256), 0, stream>>>(g);
        else generic_fused_kernel<W, false, U, 2><<<grid, dim3(256), 0, stream>>>(g);
    } else {
        if (g.fused_small) generic_fused_kernel<W, true, U, 1><<<grid, dim3(256), 0, stream>>>(g);
        else generic_fused_kernel<W, false, U, 1><<<grid, dim3(256), 0, stream>>>(g);
    }
}
template <int W>
static void launch_fused(const GenStmt &g, bool pairs, dim3 grid, hipStream_t stream) {
    static_assert(kGenMaxUpper == 2, "one instance per number of inlined levels");
    if (g.fused_upper == 0) launch_fused_u<W, 0>(g, pairs, grid, stream);
    else if (g.fused_upper == 1) launch_fused_u<W, 1>(g, pairs, grid, stream);
    else launch_fused_u<W, 2>(g, pairs, grid, stream);
}

// second pass of a long sum: the partial sums of each result node, added in segment order.  Nodes
// with more than kGenHeavy segments are left to the kernel below.
__global__ void __launch_bounds__(256)
generic_segsum_kernel(GenStmt g) {
    const int64_t gid = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (gid >= g.out_nodes * g.out_block) return;
    const int64_t p = gid / g.out_block, o = gid - p * g.out_block;
    const int64_t s0 = g.seg_ptr[p], s1 = g.seg_ptr[p + 1];
    if (s1 - s0 > kGenHeavy) return;
    double acc = 0.0;
    for (int64_t sg = s0; sg < s1; ++sg) acc += g.partial[sg * g.out_block + o];
    const int64_t row = g.scatter_rows ? int64_t(g.idx[0][p]) : p;
    g.out[row * g.out_block + o] = acc;
}

// One workgroup per node with many segments (a slice of a power-law tensor has thousands): thread
// (s, j) adds every S-th segment's element j, S = 256 / W, then thread (0, j) adds the S sums in
// order.  The order of addition depends on the launch shape only.  kGenHeavyParts workgroups share a
// node, each a contiguous range of its segments; their sums go to `heavy_sums` and a last small kernel
// adds them in order.
constexpr int kGenHeavyParts = 16;
template <int W>
__global__ void __launch_bounds__(256)
generic_segsum_heavy_kernel(GenStmt g) {
    constexpr int S = 256 / W;
    __shared__ double part[256];
    const int64_t p = g.heavy[blockIdx.x];
    const int64_t a0 = g.seg_ptr[p], a1 = g.seg_ptr[p + 1];
    const int64_t s0 = a0 + (a1 - a0) * int64_t(blockIdx.y) / kGenHeavyParts,
                  s1 = a0 + (a1 - a0) * int64_t(blockIdx.y + 1) / kGenHeavyParts;
    const int j = int(threadIdx.x) % W, sl = int(threadIdx.x) / W;
    double *dst = g.heavy_sums + (int64_t(blockIdx.x) * kGenHeavyParts + blockIdx.y) * g.out_block;
    for (int64_t o0 = 0; o0 < g.out_block; o0 += W) {
        const int64_t o = o0 + j;
        double acc = 0.0;
        if (o < g.out_block)
            for (int64_t sg = s0 + sl; sg < s1; sg += S) acc += g.partial[sg * g.out_block + o];
        part[threadIdx.x] = acc;
        __syncthreads();
        if (sl == 0 && o < g.out_block) {
            double sum = 0.0;
#pragma unroll
            for (int k = 0; k < S; ++k) sum += part[k * W + j];
            dst[o] = sum;
        }
        __syncthreads();
    }
}
__global__ void __launch_bounds__(256)
generic_segsum_heavy_final_kernel(GenStmt g) {
    const int64_t gid = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (gid >= g.n_heavy * g.out_block) return;
    const int64_t h = gid / g.out_block, o = gid - h * g.out_block;
    double sum = 0.0;
#pragma unroll
    for (int k = 0; k < kGenHeavyParts; ++k) sum += g.heavy_sums[(h * kGenHeavyParts + k) * g.out_block + o];
    const int64_t p = g.heavy[h];
    const int64_t row = g.scatter_rows ? int64_t(g.idx[0][p]) : p;
    g.out[row * g.out_block + o] = sum;
}

__global__ void generic_heavy_flag_kernel(const int64_t *seg_ptr, int64_t nodes, int64_t *flag) {
    const int64_t p = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (p < nodes) flag[p] = seg_ptr[p + 1] - seg_ptr[p] > kGenHeavy ? 1 : 0;
}
__global__ void generic_heavy_list_kernel(const int64_t *flag, const int64_t *pos, int64_t nodes, int64_t *list) {
    const int64_t p = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (p < nodes && flag[p]) list[pos[p]] = p;
}

// segments of kGenSegment children: how many per result node, then their ranges
__global__ void generic_seg_count_kernel(const int64_t *ptr, int64_t nodes, int64_t roots, int64_t *count) {
    const int64_t p = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (p >= nodes) return;
    const int64_t children = ptr ? ptr[p + 1] - ptr[p] : roots;
    count[p] = (children + kGenSegment - 1) / kGenSegment;
}
__global__ void generic_seg_fill_kernel(const int64_t *ptr, int64_t nodes, int64_t roots, const int64_t *seg_ptr, int64_t *seg) {
    const int64_t p = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (p >= nodes) return;
    const int64_t c0 = ptr ? ptr[p] : 0, c1 = ptr ? ptr[p + 1] : roots;
    int64_t sg = seg_ptr[p];
    for (int64_t c = c0; c < c1; c += kGenSegment, ++sg) {
        seg[3 * sg] = p;
        seg[3 * sg + 1] = c;
        seg[3 * sg + 2] = c + kGenSegment < c1 ? c + kGenSegment : c1;
    }
}

// The same for a statement whose producer is inlined: its work is counted in X's leaves, so the
// leaves below a result node are cut into ranges of kGenLeafSegment, wherever the fibers end.
__global__ void generic_leafseg_count_kernel(const int64_t *out_leaf, int64_t nodes, int64_t leaves, int64_t *count) {
    const int64_t p = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (p >= nodes) return;
    const int64_t e0 = out_leaf ? out_leaf[p] : 0, e1 = out_leaf ? out_leaf[p + 1] : leaves;
    count[p] = (e1 - e0 + kGenLeafSegment - 1) / kGenLeafSegment;
}
__global__ void generic_leafseg_fill_kernel(const int64_t *out_leaf, int64_t nodes, int64_t leaves, const int64_t *seg_ptr, int64_t *seg) {
    const int64_t p = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (p >= nodes) return;
    const int64_t l1 = out_leaf ? out_leaf[p + 1] : leaves;
    int64_t e = out_leaf ? out_leaf[p] : 0;
    for (int64_t sg = seg_ptr[p]; sg < seg_ptr[p + 1]; ++sg, e += kGenLeafSegment) {
        seg[3 * sg] = p;
        seg[3 * sg + 1] = e;
        seg[3 * sg + 2] = e + kGenLeafSegment < l1 ? e + kGenLeafSegment : l1;
    }
}
// first leaf below each node of a level, from the level below: out[x] = below[ptr[x]], x = 0 .. nodes
__global__ void generic_leaf_ptr_kernel(const int64_t *ptr, const int64_t *below, int64_t nodes, int64_t *out) {
    const int64_t x = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (x <= nodes) out[x] = below[ptr[x]];
}

__global__ void __launch_bounds__(256)
generic_node_kernel(GenStmt g) {
    const int64_t gid = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    const int d = g.d_node;
    if (gid >= g.nodes[d - 1] * g.out_threads) return;
    const int64_t node = gid / g.out_threads;
    int64_t rem = gid - node * g.out_threads;
    int64_t anc[CONSTSTN_MAX_ORDER];
    anc[d - 1] = node;
    for (int L = d - 1; L >= 1; --L) anc[L - 1] = parent_of(g.ptr[L - 1], g.nodes[L - 1], anc[L]);
    int64_t in_off = g.d_in > 0 ? anc[g.d_in - 1] * g.in_block : 0;
    int64_t f_off = g.d_f > 0 ? anc[g.d_f - 1] * g.f_block : 0;
    int64_t out_off = 0;
    if (g.d_out > 0) {
        const int64_t row = g.scatter_rows ? int64_t(g.idx[0][anc[0]]) : anc[g.d_out - 1];
        out_off = row * g.out_block;
    }
    for (int L = 0; L < d; ++L) {
        const int64_t x = g.idx[L][anc[L]];
        in_off += x * g.in_level_stride[L];
        f_off += x * g.f_level_stride[L];
        out_off += x * g.out_level_stride[L];
    }
    for (int q = g.n_out - 1; q >= 0; --q) {
        const int64_t o = rem % g.extent[q];
        rem /= g.extent[q];
        in_off += o * g.in_stride[q];
        f_off += o * g.f_stride[q];
        out_off += o * g.out_stride[q];
    }
    double acc = 0.0;
    int64_t cnt[kGenMaxIdx] = {0};
    for (;;) {
        acc = fma(g.in[in_off], g.f[f_off], acc);
        int q = g.n_out + g.n_red - 1;
        for (; q >= g.n_out; --q) {
            in_off += g.in_stride[q];
            f_off += g.f_stride[q];
            if (++cnt[q] < g.extent[q]) break;
            in_off -= g.in_stride[q] * g.extent[q];
            f_off -= g.f_stride[q] * g.extent[q];
            cnt[q] = 0;
        }
        if (q < g.n_out) break;
    }
    if (g.atomic) unsafeAtomicAdd(g.out + (g.copies > 1 ? int64_t(blockIdx.x % unsigned(g.copies)) * g.out_elems : 0) + out_off, acc);
    else g.out[out_off] = acc;
}

// the private copies of an added-into result, summed in copy order
__global__ void __launch_bounds__(256)
generic_copysum_kernel(const double *copies, int n_copies, int64_t elems, double *out) {
    const int64_t x = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (x >= elems) return;
    double acc = 0.0;
    for (int c = 0; c < n_copies; ++c) acc += copies[int64_t(c) * elems + x];
    out[x] = acc;
}

// largest number of depth-d_in nodes below one depth-d_out node (d_out >= 1)
__global__ void generic_span_kernel(GenStmt g, int d_out, int d_in, unsigned long long *result) {
    const int64_t p = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (p >= g.nodes[d_out - 1]) return;
    int64_t lo = p, hi = p + 1;
    for (int L = d_out - 1; L <= d_in - 2; ++L) { lo = g.ptr[L][lo]; hi = g.ptr[L][hi]; }
    atomicMax(result, (unsigned long long)(hi - lo));
}

namespace {

// a tensor on the way from X to the result, or a dense one
struct GenTensor {
    int depth = 0;                        // CSF prefix depth of the storage (0 = stored dense)
    bool leaf = false;                    // X itself
    std::vector<std::string> dense;       // index names in storage order after the prefix (last fastest)
    int operand = -1;                     // dense operand ordinal among ALL operands, or -1
    int buffer = -1;                      // intermediate buffer number, or -1
    bool from_x = false;                  // descends from the CSF operand and is stored by prefix
};

int find_name(const std::vector<std::string> &v, const std::string &n) {
    for (size_t i = 0; i < v.size(); ++i) if (v[i] == n) return int(i);
    return -1;
}

// dense[level-order offset of the leaf's coordinates] = value, one thread per leaf (the array was cleared)
__global__ void densify_csf_kernel(GenStmt g, int order, double *dense) {
    int64_t node = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (node >= g.nodes[order - 1]) return;
    const double v = g.in[node];
    int64_t off = 0, stride = 1;
    for (int l = order - 1; l >= 0; --l) {
        off += int64_t(g.idx[l][node]) * stride;
        stride *= g.extent[l];
        if (l > 0) node = parent_of(g.ptr[l - 1], g.nodes[l - 1], node);
    }
    dense[off] = v;
}

// A tree over several CSF operands (Sec. 3.1's running example has four): the executor walks ONE of them,
// the one with the most nonzeros; the others are spread out into dense arrays in their level order when
// the plan is built (their values are fixed by their handles) and take part as dense operands.  Slow
// and always applicable, within the memory bound; no co-iteration.
static conststn_status densify_other_operands(conststn_plan_s *plan, int keep) {
    Schedule &s = plan->sched;
    const int64_t limit = plan->opt("generic_max_gb", 64) << 30;
    for (size_t o = 0; o < s.operands.size(); ++o) {
        OperandInfo &oi = s.operands[o];
        if (oi.kind != CONSTSTN_OPERAND_CSF || int(o) == keep) continue;
        const conststn_csf_s *c = oi.csf;
        if (!c) { set_error("CSF operand %s has no handle", oi.name.c_str()); return CONSTSTN_EINVAL; }
        if (c->order > kGenMaxIdx) { set_error("CSF operand %s has more levels than the generic executor spreads out", oi.name.c_str()); return CONSTSTN_EUNSUPPORTED; }
        int64_t elems = 1;
        for (int l = 0; l < c->order; ++l) {
            if (oi.dims[l] > 0 && elems > limit / 8 / oi.dims[l]) {
                set_error("a dense copy of CSF operand %s would exceed generic_max_gb", oi.name.c_str());
                return CONSTSTN_EUNSUPPORTED;
            }
            elems *= oi.dims[l];
        }
        plan->gen_densified.emplace_back(new DevBuf<double>());
        DevBuf<double> &buf = *plan->gen_densified.back();
        CST_TRY(buf.alloc(size_t(std::max<int64_t>(elems, 1))));
        CST_HIP(hipMemset(buf.p, 0, size_t(std::max<int64_t>(elems, 1)) * sizeof(double)));
        if (c->nnz > 0) {
            GenStmt g{};
            for (int l = 0; l < c->order; ++l) {
                g.nodes[l] = c->nodes[l];
                g.idx[l] = c->idx[l].p;
                g.ptr[l] = l + 1 < c->order ? c->ptr[l].p : nullptr;
                g.extent[l] = oi.dims[l];
            }
            g.in = c->vals.p;
            densify_csf_kernel<<<dim3(unsigned(div_up(c->nnz, 256))), dim3(256)>>>(g, c->order, buf.p);
            CST_HIP(hipGetLastError());
            CST_HIP(hipDeviceSynchronize());
        }
        oi.kind = CONSTSTN_OPERAND_DENSE;         // from here on a dense operand that the plan owns
        oi.owned = buf.p;
    }
    return CONSTSTN_OK;
}

}  // namespace

conststn_status build_generic(conststn_plan_s *plan) {
    Schedule &s = plan->sched;
    const int m = int(s.stmts.size());
    int xop = -1, n_csf = 0;
    for (size_t o = 0; o < s.operands.size(); ++o)
        if (s.operands[o].kind == CONSTSTN_OPERAND_CSF) {
            ++n_csf;
            // the operand the executor walks: the one with the most nonzeros among those used once
            int uses = 0;
            for (const Stmt &st : s.stmts)
                for (const Ref *r : {&st.a, &st.b})
                    if (r->name == s.operands[o].name) ++uses;
            const conststn_csf_s *c = s.operands[o].csf;
            if (uses == 1 && c && (xop < 0 || c->nnz > s.operands[size_t(xop)].csf->nnz)) xop = int(o);
        }
    if (n_csf > 1) {
        if (plan->opt("generic_densify", 1) != 1) { set_error("the generic executor takes one CSF operand; the schedule has more"); return CONSTSTN_EUNSUPPORTED; }
        if (xop < 0) { set_error("the generic executor needs a CSF operand that is used exactly once"); return CONSTSTN_EUNSUPPORTED; }
        CST_TRY(densify_other_operands(plan, xop));
    } else if (n_csf == 1 && xop < 0) {
        for (size_t o = 0; o < s.operands.size(); ++o)
            if (s.operands[o].kind == CONSTSTN_OPERAND_CSF) xop = int(o);     // reported below: used more than once
    }
    if (xop < 0) { set_error("the generic executor needs a CSF operand"); return CONSTSTN_EUNSUPPORTED; }
    const OperandInfo &X = s.operands[xop];
    const conststn_csf_s *csf = X.csf;
    if (!csf) { set_error("CSF operand %s has no handle", X.name.c_str()); return CONSTSTN_EINVAL; }
    const int n = X.order;
    std::vector<std::string> level_name;          // index name of each CSF level, from X's reference
    int x_uses = 0;
    for (const Stmt &st : s.stmts)
        for (const Ref *r : {&st.a, &st.b})
            if (r->name == X.name) { level_name = r->idx; ++x_uses; }
    if (x_uses != 1) { set_error("the generic executor needs the CSF operand to be used exactly once"); return CONSTSTN_EUNSUPPORTED; }
    auto level_of = [&](const std::string &nm) { return find_name(level_name, nm); };
    // leading names of a result that are CSF levels 0,1,.. in order, at most `limit` of them
    auto front_prefix = [&](const std::vector<std::string> &names, int limit) {
        int d = 0;
        while (d < int(names.size()) && d < limit && names[d] == level_name[d]) ++d;
        return d;
    };
    // does the result keep a level below `limit` that is not part of its front prefix of depth d?
    auto keeps_beyond_prefix = [&](const std::vector<std::string> &names, int d, int limit) {
        for (size_t q = size_t(d); q < names.size(); ++q) {
            const int L = level_of(names[q]);
            if (L >= 0 && L < limit) return true;
        }
        return false;
    };

    // first pass: how deep each statement's result is sparse like X (-1: not at all), from the
    // index names alone; decides which products of dense tensors are computed at X's nodes only
    std::vector<int> xdepth(m, -1);
    auto ref_xdepth = [&](int src, int op) {
        if (src >= 0) return xdepth[src];
        return s.operands[op].kind == CONSTSTN_OPERAND_CSF ? n : -1;
    };
    for (int p = 0; p < m; ++p) {
        const Stmt &st = s.stmts[p];
        const int da = ref_xdepth(st.src_a, st.op_a), db = ref_xdepth(st.src_b, st.op_b);
        const int d_in = std::max(da, db);
        if (d_in < 1) continue;
        const int d = front_prefix(st.out.idx, d_in);
        const bool last = st.consumer < 0;
        if (keeps_beyond_prefix(st.out.idx, d, d_in) || (last && d > 1)) continue;       // stored dense
        xdepth[p] = d >= 1 ? d : -1;
    }

    // one thread summing a whole subtree is fine for short fibers and hopeless for a power-law slice:
    // beyond span_limit nodes below one result node the sum is cut into segments (two passes)
    const int64_t span_limit = plan->opt("generic_span", 4096);
    std::map<std::pair<int, int>, int64_t> span_cache;
    conststn_status span_status = CONSTSTN_OK;
    auto max_span = [&](int d_out, int d_in) -> int64_t {
        if (d_out == 0) return csf->nodes[d_in - 1];
        const auto key = std::make_pair(d_out, d_in);
        auto it = span_cache.find(key);
        if (it != span_cache.end()) return it->second;
        GenStmt g{};
        for (int l = 0; l < n; ++l) { g.nodes[l] = csf->nodes[l]; g.ptr[l] = l + 1 < n ? csf->ptr[l].p : nullptr; }
        DevBuf<unsigned long long> dmax;
        unsigned long long h = 0;
        if (dmax.alloc(1) != CONSTSTN_OK || hipMemset(dmax.p, 0, sizeof(h)) != hipSuccess) { span_status = CONSTSTN_ENOMEM; return 0; }
        if (csf->nodes[d_out - 1] > 0)
            generic_span_kernel<<<dim3(unsigned((csf->nodes[d_out - 1] + 255) / 256)), dim3(256)>>>(g, d_out, d_in, dmax.p);
        if (hipMemcpy(&h, dmax.p, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) { span_status = CONSTSTN_EHIP; return 0; }
        span_cache[key] = int64_t(h);
        return int64_t(h);
    };

    std::vector<GenTensor> result(m);             // the tensor each statement produces
    plan->gen.clear();
    plan->gen_buffers.clear();
    plan->gen_tables.clear();
    plan->gen_leaf_tables.clear();
    plan->gen_zero_out = false;
    std::vector<int64_t> buffer_elems;
    auto tensor_of_ref = [&](const Ref &r, int src, int op, GenTensor &t) {
        if (src >= 0) { t = result[src]; return; }
        const OperandInfo &oi = s.operands[op];
        t = GenTensor();
        if (oi.kind == CONSTSTN_OPERAND_CSF) {
            t.depth = n;
            t.leaf = true;
            t.from_x = true;
        } else {
            t.dense = r.idx;
            t.operand = op;
        }
    };
    // strides of an index list stored row-major in the given order; returns the element count
    auto strides = [&](const std::vector<std::string> &names, std::map<std::string, int64_t> &out) {
        int64_t stride = 1;
        for (int q = int(names.size()) - 1; q >= 0; --q) { out[names[q]] = stride; stride *= s.extent[names[q]]; }
        return stride;
    };

    // first leaf below each node of level L (and the leaf count after the last): X's own pointers for the
    // fibers, composed level by level above them; built when a fused statement asks, kept with the plan
    std::vector<const int64_t *> leaf_ptr_of(size_t(n), nullptr);
    auto leaf_ptr = [&](int L, const int64_t **out) -> conststn_status {
        if (L < 0 || L > n - 2) { set_error("internal: no leaf pointers for level %d", L); return CONSTSTN_EINVAL; }
        leaf_ptr_of[size_t(n - 2)] = csf->ptr[n - 2].p;
        for (int l = n - 3; l >= L; --l) {
            if (leaf_ptr_of[size_t(l)]) continue;
            plan->gen_leaf_tables.emplace_back(new DevBuf<int64_t>());
            DevBuf<int64_t> &t = *plan->gen_leaf_tables.back();
            CST_TRY(t.alloc(size_t(csf->nodes[l] + 1)));
            generic_leaf_ptr_kernel<<<dim3(unsigned((csf->nodes[l] + 256) / 256)), dim3(256)>>>(csf->ptr[l].p, leaf_ptr_of[size_t(l + 1)], csf->nodes[l], t.p);
            CST_HIP(hipGetLastError());
            leaf_ptr_of[size_t(l)] = t.p;
        }
        *out = leaf_ptr_of[size_t(L)];
        return CONSTSTN_OK;
    };
    std::vector<std::vector<std::string>> out_dense_of(static_cast<size_t>(m));     // each statement's dense result indices, in loop order

    for (int p = 0; p < m; ++p) {
        const Stmt &st = s.stmts[p];
        const bool last = st.consumer < 0;
        GenTensor ta, tb;
        tensor_of_ref(st.a, st.src_a, st.op_a, ta);
        tensor_of_ref(st.b, st.src_b, st.op_b, tb);
        if (ta.from_x && tb.from_x) { set_error("statement %d multiplies two tensors that both descend from the CSF operand", p); return CONSTSTN_EUNSUPPORTED; }
        const GenTensor &in = tb.from_x ? tb : ta;            // sparse side (or first dense input)
        const GenTensor &fa = tb.from_x ? ta : tb;            // the other side
        if (!in.from_x && (in.depth > 0 || fa.depth > 0)) { set_error("internal: a tensor stored by prefix meets no sparse partner in statement %d", p); return CONSTSTN_EINVAL; }
        if (fa.depth > in.depth) { set_error("internal: statement %d joins a deeper prefix with a shallower one", p); return CONSTSTN_EINVAL; }

        // which kernel, and how the result is stored
        int kind = 0, d_node = in.from_x ? in.depth : 0, d_out = 0;
        bool out_by_prefix = true;
        if (d_node == 0) {
            // two dense inputs: computed at X's nodes when the consumer's other input is sparse to that depth
            const int d = front_prefix(st.out.idx, n);
            int other = -1;
            if (!last) {
                const Stmt &c = s.stmts[st.consumer];
                other = c.src_a == p ? ref_xdepth(c.src_b, c.op_b) : ref_xdepth(c.src_a, c.op_a);
            }
            if (d >= 1 && other >= d) { kind = 1; d_node = d; d_out = d; }
        } else {
            d_out = front_prefix(st.out.idx, d_node);
            bool f_uses_kept = false;
            for (const auto &nm : fa.dense) { const int L = level_of(nm); if (L >= 0 && L < d_out) f_uses_kept = true; }
            if (keeps_beyond_prefix(st.out.idx, d_out, d_node) || (last && d_out > 1)) { kind = 1; out_by_prefix = false; d_out = 0; }
            else if (fa.depth > 0 || f_uses_kept) kind = 1;
        }
        bool long_sum = kind == 0 && d_node > 0 && d_out < d_node && max_span(d_out, d_node) > span_limit;
        if (span_status != CONSTSTN_OK) { set_error("could not measure the subtree sizes of the CSF operand"); return span_status; }
        auto is_level = [&](const std::string &nm) { const int L = level_of(nm); return L >= 0 && L < d_node; };

        // dense loop indices: the result's first, then the summed ones
        std::vector<std::string> out_dense;
        for (size_t q = out_by_prefix ? size_t(d_out) : 0; q < st.out.idx.size(); ++q)
            if (!is_level(st.out.idx[q])) out_dense.push_back(st.out.idx[q]);
        std::vector<std::string> red;
        auto consider = [&](const std::string &nm) {
            if (is_level(nm)) return;
            if (find_name(out_dense, nm) >= 0 || find_name(red, nm) >= 0) return;
            red.push_back(nm);
        };
        for (const auto &nm : in.dense) consider(nm);
        for (const auto &nm : fa.dense) consider(nm);
        out_dense_of[size_t(p)] = out_dense;
        if (out_dense.size() + red.size() > size_t(kGenMaxIdx)) { set_error("statement %d has more than %d dense indices", p, kGenMaxIdx); return CONSTSTN_EUNSUPPORTED; }

        GenStmt g{};
        g.kind = kind;
        g.d_node = d_node;
        g.d_in = kind == 1 ? in.depth : d_node;
        g.d_f = fa.depth;
        g.d_out = d_out;
        g.atomic = (kind == 1 && d_out != d_node) ? 1 : 0;
        g.in_is_leaf = in.leaf ? 1 : 0;
        g.n_out = int(out_dense.size());
        g.n_red = int(red.size());
        std::vector<std::string> loopn = out_dense;
        loopn.insert(loopn.end(), red.begin(), red.end());
        for (size_t q = 0; q < loopn.size(); ++q) g.extent[q] = s.extent[loopn[q]];
        std::map<std::string, int64_t> sin, sf, sout;
        g.in_block = strides(in.dense, sin);
        g.f_block = strides(fa.dense, sf);
        std::vector<std::string> out_names = out_by_prefix ? std::vector<std::string>(st.out.idx.begin() + d_out, st.out.idx.end())
                                                           : st.out.idx;
        g.out_block = strides(out_names, sout);
        g.out_threads = 1;
        for (size_t q = 0; q < out_dense.size(); ++q) g.out_threads *= g.extent[q];
        for (size_t q = 0; q < loopn.size(); ++q) {
            g.in_stride[q] = sin.count(loopn[q]) ? sin[loopn[q]] : 0;
            g.f_stride[q] = sf.count(loopn[q]) ? sf[loopn[q]] : 0;
            g.out_stride[q] = (q < out_dense.size() && sout.count(loopn[q])) ? sout[loopn[q]] : 0;
        }
        for (int L = 0; L < d_node; ++L) {
            const std::string &nm = level_name[L];
            if (sin.count(nm)) g.in_level_stride[L] = sin[nm];
            if (sf.count(nm)) g.f_level_stride[L] = sf[nm];
            if (sout.count(nm)) g.out_level_stride[L] = sout[nm];
        }
        if (kind == 0 && d_node > 0) {
            // the first kernel knows the other input's level strides only, and only below the result's depth
            for (int L = 0; L < d_node; ++L)
                if (g.in_level_stride[L] || g.out_level_stride[L] || (L < d_out && g.f_level_stride[L])) {
                    set_error("internal: statement %d was given to the subtree kernel with a level-indexed tensor", p);
                    return CONSTSTN_EINVAL;
                }
        }
        // where the inputs live
        g.in_operand = in.operand;
        g.in_buffer = in.buffer;
        g.f_operand = fa.operand;
        g.f_buffer = fa.buffer;
        g.out_nodes = (out_by_prefix && d_out > 0) ? csf->nodes[d_out - 1] : 1;
        g.out_elems = g.out_nodes * g.out_block;
        g.roots = csf->nodes[0];
        for (int l = 0; l < n; ++l) {
            g.nodes[l] = csf->nodes[l];
            g.idx[l] = csf->idx[l].p;
            g.ptr[l] = l + 1 < n ? csf->ptr[l].p : nullptr;
        }
        // Fusion (Sec. 2.2): when this statement consumes a result that the statement before it in the tree forms
        // from X's leaves and a dense operand one level deeper, with the same dense indices, and the
        // schedule fuses the two on the whole prefix, the producer is computed inside this statement's
        // kernel.  The producer may have inlined its own producer the same way: a chain of statements that
        // each sum one more level becomes one kernel, and none of their results is stored.
        {
            const int prod = tb.from_x ? st.src_b : st.src_a;
            if (kind == 0 && prod >= 0 && in.from_x && g.n_red == 0 && d_node - d_out == 1 &&
                plan->opt("generic_fuse", 1) == 1 && s.stmts[prod].fused_depth >= d_node) {
                GenStmt &g1 = plan->gen[size_t(prod)];
                const Stmt &sp = s.stmts[prod];
                const bool chain = g1.fused == 1;
                const Ref *f1ref = nullptr;
                if (sp.op_a >= 0 && sp.op_a == g1.f_operand) f1ref = &sp.a;
                else if (sp.op_b >= 0 && sp.op_b == g1.f_operand) f1ref = &sp.b;
                bool ok = g1.kind == 0 && g1.in_is_leaf && g1.n_red == 0 && g1.d_node == d_node + 1 && g1.d_f == 0 &&
                          g1.d_out == d_node && g1.out_buffer == in.buffer && g1.f_operand >= 0 && f1ref &&
                          g1.n_out == g.n_out && g1.skip == 0;
                if (chain) ok = ok && g1.fused_upper < kGenMaxUpper;
                else ok = ok && d_node == n - 1;
                const std::vector<std::string> &dense1 = out_dense_of[size_t(prod)];
                std::map<std::string, int64_t> sf1;
                if (ok) {
                    strides(f1ref->idx, sf1);
                    // the same dense indices on both results (any order), none of them summed
                    for (size_t q = 0; q < out_dense.size() && ok; ++q)
                        if (find_name(in.dense, out_dense[q]) < 0 || find_name(dense1, out_dense[q]) < 0) ok = false;
                    if (in.dense.size() != out_dense.size() || dense1.size() != out_dense.size()) ok = false;
                    for (const auto &nm : f1ref->idx)
                        if (nm != level_name[d_node] && find_name(out_dense, nm) < 0) ok = false;
                }
                if (ok) {
                    g.fused = 1;
                    // the largest byte offset into a factor, the largest row number and row stride
                    auto within_reach = [&](const int64_t *stride, int64_t level_stride, int64_t level_extent) {
                        int64_t elems = (level_extent - 1) * level_stride;
                        for (size_t q = 0; q < out_dense.size(); ++q) elems += (g.extent[q] - 1) * stride[q];
                        const int64_t lim24 = int64_t(1) << 24, lim31 = int64_t(1) << 31;
                        return elems * 8 + 8 < lim31 && level_extent < lim24 && level_stride * 8 < lim24;
                    };
                    bool small = within_reach(g.f_stride, g.f_level_stride[d_out], s.extent[level_name[d_out]]);
                    int64_t sf1_dense[kGenMaxIdx] = {};
                    for (size_t q = 0; q < out_dense.size(); ++q) sf1_dense[q] = sf1.count(out_dense[q]) ? sf1[out_dense[q]] : 0;
                    const int64_t sf1_level = sf1.count(level_name[d_node]) ? sf1[level_name[d_node]] : 0;
                    small = small && within_reach(sf1_dense, sf1_level, s.extent[level_name[d_node]]);
                    if (!chain) {
                        g.fused_upper = 0;
                        g.f1_operand = g1.f_operand;
                        for (size_t q = 0; q < out_dense.size(); ++q) g.f1_stride[q] = sf1_dense[q];
                        g.f1_level_stride = sf1_level;
                    } else {
                        // what the producer had inlined, its dense indices in this statement's order, then its own factor
                        const int u1 = g1.fused_upper;
                        g.fused_upper = u1 + 1;
                        g.f1_operand = g1.f1_operand;
                        g.f1_level_stride = g1.f1_level_stride;
                        for (int v = 0; v < u1; ++v) {
                            g.fu_operand[v] = g1.fu_operand[v];
                            g.fu_level_stride[v] = g1.fu_level_stride[v];
                        }
                        for (size_t q = 0; q < out_dense.size(); ++q) {
                            const int q1 = find_name(dense1, out_dense[q]);
                            g.f1_stride[q] = g1.f1_stride[q1];
                            for (int v = 0; v < u1; ++v) g.fu_stride[v][q] = g1.fu_stride[v][q1];
                            g.fu_stride[u1][q] = sf1_dense[q];
                        }
                        g.fu_operand[u1] = g1.f_operand;
                        g.fu_level_stride[u1] = sf1_level;
                        small = small && g1.fused_small == 1;
                    }
                    g.fused_small = small ? 1 : 0;
                    {
                        // two adjacent elements of the innermost dense index per lane: stride 1 there, every other stride even
                        const int last_q = g.n_out - 1;
                        auto fits = [&](const int64_t *stride, int64_t level_stride) {
                            if (stride[last_q] != 1 || level_stride % 2 != 0) return false;
                            for (int q = 0; q < last_q; ++q)
                                if (stride[q] % 2 != 0) return false;
                            return true;
                        };
                        bool pairs = last_q >= 0 && g.extent[last_q] % 2 == 0 && g.out_block % 2 == 0 &&
                                     fits(g.f_stride, g.f_level_stride[d_out]) && fits(g.f1_stride, g.f1_level_stride) &&
                                     fits(g.out_stride, 0);
                        for (int v = 0; v < g.fused_upper; ++v) pairs = pairs && fits(g.fu_stride[v], g.fu_level_stride[v]);
                        g.fused_pairs = pairs ? 1 : 0;
                    }
                    for (int v = 1; v <= g.fused_upper; ++v) CST_TRY(leaf_ptr(n - 2 - v, &g.leaf_end[v - 1]));
                    if (d_out > 0) CST_TRY(leaf_ptr(d_out - 1, &g.out_leaf));
                    g.in_is_leaf = 1;                       // reads X's values, not the intermediate
                    g.d_in = n - 1;
                    g.in_operand = -1;
                    g.in_buffer = -1;
                    g1.skip = 1;
                    buffer_elems[size_t(in.buffer)] = 1;    // the intermediate is never stored,
                    if (g1.n_segs > 0) {                    // nor are its partial sums
                        buffer_elems[size_t(g1.partial_buffer)] = 1;
                        buffer_elems[size_t(g1.heavy_buffer)] = 1;
                    }
                    long_sum = max_span(d_out, n) > std::min<int64_t>(span_limit, int64_t(1) << 29);     // work counted in leaves
                }
            }
        }
        if (long_sum) {
            // the children of every result node in segments of kGenSegment
            const int64_t on = g.out_nodes;
            const int64_t *cptr = d_out > 0 ? csf->ptr[d_out - 1].p : nullptr;
            DevBuf<int64_t> count;
            CST_TRY(count.alloc(size_t(on)));
            plan->gen_tables.emplace_back(new DevBuf<int64_t>());
            DevBuf<int64_t> &sptr = *plan->gen_tables.back();
            CST_TRY(sptr.alloc(size_t(on + 1)));
            if (g.fused) generic_leafseg_count_kernel<<<dim3(unsigned((on + 255) / 256)), dim3(256)>>>(g.out_leaf, on, csf->nnz, count.p);
            else generic_seg_count_kernel<<<dim3(unsigned((on + 255) / 256)), dim3(256)>>>(cptr, on, csf->nodes[0], count.p);
            CST_HIP(hipGetLastError());
            int64_t n_segs = 0;
            CST_TRY(exscan(count.p, sptr.p, on, &n_segs));
            CST_HIP(hipMemcpy(sptr.p + on, &n_segs, sizeof(int64_t), hipMemcpyHostToDevice));
            plan->gen_tables.emplace_back(new DevBuf<int64_t>());
            DevBuf<int64_t> &seg = *plan->gen_tables.back();
            CST_TRY(seg.alloc(size_t(3 * n_segs)));
            if (g.fused) generic_leafseg_fill_kernel<<<dim3(unsigned((on + 255) / 256)), dim3(256)>>>(g.out_leaf, on, csf->nnz, sptr.p, seg.p);
            else generic_seg_fill_kernel<<<dim3(unsigned((on + 255) / 256)), dim3(256)>>>(cptr, on, csf->nodes[0], sptr.p, seg.p);
            CST_HIP(hipGetLastError());
            CST_HIP(hipDeviceSynchronize());
            g.n_segs = n_segs;
            g.seg_table = int(plan->gen_tables.size()) - 2;
            {
                // the nodes with many segments, listed for the second pass
                DevBuf<int64_t> flag, pos;
                CST_TRY(flag.alloc(size_t(on)));
                CST_TRY(pos.alloc(size_t(on)));
                generic_heavy_flag_kernel<<<dim3(unsigned((on + 255) / 256)), dim3(256)>>>(sptr.p, on, flag.p);
                CST_HIP(hipGetLastError());
                int64_t n_heavy = 0;
                CST_TRY(exscan(flag.p, pos.p, on, &n_heavy));
                plan->gen_tables.emplace_back(new DevBuf<int64_t>());
                DevBuf<int64_t> &heavy = *plan->gen_tables.back();
                CST_TRY(heavy.alloc(size_t(std::max<int64_t>(n_heavy, 1))));
                generic_heavy_list_kernel<<<dim3(unsigned((on + 255) / 256)), dim3(256)>>>(flag.p, pos.p, on, heavy.p);
                CST_HIP(hipGetLastError());
                CST_HIP(hipDeviceSynchronize());
                g.n_heavy = n_heavy;
                g.heavy_buffer = int(buffer_elems.size());
                buffer_elems.push_back(std::max<int64_t>(n_heavy, 1) * kGenHeavyParts * g.out_block);
            }
            g.partial_buffer = int(buffer_elems.size());
            buffer_elems.push_back(n_segs * g.out_block);
        }
        if (g.atomic) {
            const int64_t bytes = g.out_elems * 8;
            int copies = int(std::min<int64_t>(64, (int64_t(512) << 20) / std::max<int64_t>(bytes, 1)));
            if (copies >= 2 && !(last && out_by_prefix && d_out == 1 && !plan->compact)) {     // rows scattered by root index keep one copy
                g.copies = copies;
                g.copies_buffer = int(buffer_elems.size());
                buffer_elems.push_back(g.out_elems * copies);
            }
        }
        // the result
        GenTensor &res = result[p];
        res.depth = out_by_prefix ? d_out : 0;
        res.from_x = in.from_x && out_by_prefix && d_out > 0;
        res.dense = out_names;
        if (in.from_x && (res.from_x ? res.depth : -1) != xdepth[p]) { set_error("internal: storage of statement %d's result decided two ways", p); return CONSTSTN_EINVAL; }
        if (!last) {
            res.buffer = int(buffer_elems.size());
            buffer_elems.push_back(g.out_elems);
            g.out_buffer = res.buffer;
        } else {
            g.out_buffer = -1;
            const bool rooted = out_by_prefix && d_out == 1;
            g.scatter_rows = (rooted && !plan->compact) ? 1 : 0;
            plan->gen_rooted = rooted;
            plan->row_elems = g.out_block;
            plan->gen_zero_out = g.atomic != 0;
        }
        plan->gen.push_back(g);
    }
    // intermediates, held whole
    int64_t total = 0;
    for (int64_t e : buffer_elems) total += e;
    const int64_t cap = plan->opt("generic_max_gb", 64) << 27;      // doubles
    if (total > cap) {
        set_error("the generic executor would hold %.1f GB of intermediates (limit %lld GB)", double(total) * 8e-9,
                  (long long)(cap >> 27));
        return CONSTSTN_ENOMEM;
    }
    for (size_t b = 0; b < buffer_elems.size(); ++b) {
        plan->gen_buffers.emplace_back(new DevBuf<double>());
        CST_TRY(plan->gen_buffers.back()->alloc(size_t(buffer_elems[b])));
    }
    plan->family = FAM_GENERIC;
    plan->X = csf;
    return CONSTSTN_OK;
}

conststn_status launch_generic(const conststn_plan_s *plan, const double *const *dense, double *out,
                               hipStream_t stream) {
    const Schedule &s = plan->sched;
    const conststn_csf_s *csf = plan->X;
    // rows of root indices that hold no nonzero are never written by a kernel; a result that is
    // added into starts from zero
    if (plan->gen_zero_out || (plan->gen_rooted && !plan->compact && csf->nodes[0] < plan->out_rows))
        CST_TRY(zero_fill(out, plan->out_rows * plan->row_elems, stream));
    ProfScope prof(plan, stream);
    for (const GenStmt &g0 : plan->gen) {
        if (g0.skip) continue;                     // computed inside its consumer's kernel
        GenStmt g = g0;
        auto where = [&](int operand, int buffer) -> const double * {
            if (buffer >= 0) return plan->gen_buffers[size_t(buffer)]->p;
            if (operand >= 0 && s.operands[size_t(operand)].owned) return s.operands[size_t(operand)].owned;
            if (operand >= 0) return dense[s.operands[size_t(operand)].dense_ordinal];
            return nullptr;
        };
        g.in = g.in_is_leaf ? csf->vals.p : where(g.in_operand, g.in_buffer);      // X: the leaf values
        g.f = where(g.f_operand, g.f_buffer);
        if (g.fused) {
            g.f1 = where(g.f1_operand, -1);
            for (int v = 0; v < g.fused_upper; ++v) g.fu[v] = where(g.fu_operand[v], -1);
        }
        g.out = g.out_buffer >= 0 ? plan->gen_buffers[size_t(g.out_buffer)]->p : out;
        if (!g.in || !g.f || !g.out) { set_error("internal: unresolved tensor in the generic executor"); return CONSTSTN_EINVAL; }
        double *final_out = g.out;
        if (g.copies > 1) {
            g.out = plan->gen_buffers[size_t(g.copies_buffer)]->p;
            CST_TRY(zero_fill(g.out, g.out_elems * g.copies, stream));
        } else if (g.atomic && g.out_buffer >= 0) {
            CST_TRY(zero_fill(g.out, g.out_elems, stream));
        }
        if (g.n_segs > 0) {
            g.seg_ptr = plan->gen_tables[size_t(g.seg_table)]->p;
            g.seg = plan->gen_tables[size_t(g.seg_table) + 1]->p;
            g.heavy = plan->gen_tables[size_t(g.seg_table) + 2]->p;
            g.heavy_sums = plan->gen_buffers[size_t(g.heavy_buffer)]->p;
            g.partial = plan->gen_buffers[size_t(g.partial_buffer)]->p;
        }
        // two result elements per lane where the plan found the layouts fit and the caller's arrays begin on 16 bytes
        bool pairs = false;
        if (g.fused && g.fused_pairs) {
            auto on16 = [](const void *q) { return reinterpret_cast<uintptr_t>(q) % 16 == 0; };
            pairs = on16(g.f) && on16(g.f1) && on16(g.out) && (g.n_segs == 0 || on16(g.partial));
            for (int v = 0; v < g.fused_upper; ++v) pairs = pairs && on16(g.fu[v]);
        }
        // lanes that share a result node in the fused kernel: the power of two that holds its elements, 8 to 64
        const int64_t lane_elems = pairs ? g.out_block / 2 : g.out_block;
        int fused_w = 8;
        while (fused_w < 64 && fused_w < lane_elems) fused_w *= 2;
        const int64_t units = g.n_segs > 0 ? g.n_segs : g.out_nodes;
        const int64_t total = g.kind == 1 ? g.nodes[g.d_node - 1] * g.out_threads
                              : g.fused   ? units * ((lane_elems + fused_w - 1) / fused_w) * fused_w
                                          : units * g.out_block;
        if (total > (int64_t(1) << 31) * 256) { set_error("statement result too large for one launch"); return CONSTSTN_EUNSUPPORTED; }
        const dim3 grid(unsigned((total + 255) / 256)), block(256);
        if (total > 0) {
            if (g.kind == 1) generic_node_kernel<<<grid, block, 0, stream>>>(g);
            else if (g.fused && fused_w == 8) launch_fused<8>(g, pairs, grid, stream);
            else if (g.fused && fused_w == 16) launch_fused<16>(g, pairs, grid, stream);
            else if (g.fused && fused_w == 32) launch_fused<32>(g, pairs, grid, stream);
            else if (g.fused) launch_fused<64>(g, pairs, grid, stream);
            else generic_stmt_kernel<<<grid, block, 0, stream>>>(g);
            CST_HIP(hipGetLastError());
        }
        if (g.copies > 1 && g.out_elems > 0) {
            generic_copysum_kernel<<<dim3(unsigned((g.out_elems + 255) / 256)), block, 0, stream>>>(g.out, g.copies, g.out_elems, final_out);
            CST_HIP(hipGetLastError());
        }
        if (g.kind == 0 && g.n_segs > 0 && total > 0) {
            const int64_t t2 = g.out_nodes * g.out_block;
            generic_segsum_kernel<<<dim3(unsigned((t2 + 255) / 256)), block, 0, stream>>>(g);
            CST_HIP(hipGetLastError());
            if (g.n_heavy > 0) {
                const dim3 hg{unsigned(g.n_heavy), unsigned(kGenHeavyParts)};
                if (g.out_block <= 8) generic_segsum_heavy_kernel<8><<<hg, block, 0, stream>>>(g);
                else if (g.out_block <= 32) generic_segsum_heavy_kernel<32><<<hg, block, 0, stream>>>(g);
                else if (g.out_block <= 128) generic_segsum_heavy_kernel<128><<<hg, block, 0, stream>>>(g);
                else generic_segsum_heavy_kernel<256><<<hg, block, 0, stream>>>(g);
                CST_HIP(hipGetLastError());
                generic_segsum_heavy_final_kernel<<<dim3(unsigned(div_up(g.n_heavy * g.out_block, 256))), block, 0, stream>>>(g);
                CST_HIP(hipGetLastError());
            }
        }
    }
    return CONSTSTN_OK;
}

}  // namespace cst
