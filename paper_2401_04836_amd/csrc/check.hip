// Index checking: every array the contraction kernels index through another array is checked
// against the size of what it indexes -- the level arrays of a CSF (conststn_csf_check) and the tables a plan
// holds for the order-3 MTTKRP and TTMc kernels and for the generic executor (conststn_plan_check).  The kernels themselves trust their
// tables (an index out of range there is a memory fault, not an error code); these passes are the
// debugging aid that turns a wrong table into a message.  One thread per entry, violations are OR-ed
// into a word of flags that the host reads.  Not part of the timed path.
#include "plan.hpp"

namespace cst {

namespace {

enum : unsigned {
    kBadIndex = 1u << 0,       // an index outside its mode extent
    kBadPtrStart = 1u << 1,    // a pointer array that does not start at 0
    kBadPtrOrder = 1u << 2,    // a node without children, or pointers that decrease
    kBadPtrEnd = 1u << 3,      // a pointer array that does not end at the next level's node count
    kBadSibling = 1u << 4,     // children of a node (or the roots) not strictly ascending
    kBadChunk = 1u << 5,       // a chunk table entry that does not name the fiber / slice of the chunk's first leaf
    kBadSliceLeaf = 1u << 6,   // slice_leaf differs from the composition of the pointer arrays
    kBadCode = 1u << 7,        // a re-encoded leaf naming an LDS slot or a factor row out of range, or a wrong end mark
    kBadRow = 1u << 8,         // a row descriptor outside the leaves, longer than 16 leaves or with a level-1 index out of range
    kBadKstep = 1u << 9,       // a K-step with no rows, more than four, rows outside the table or a destination out of range
    kBadBatch = 1u << 10,      // workgroup batches not ascending, not covering the K-steps, or ending inside an item
    kBadItem = 1u << 11,       // an item outside its slice or with a destination out of range
    kBadLeafTable = 1u << 12,  // a table of first leaves per node that is not the composition of the pointer arrays
    kBadSegment = 1u << 13,    // segments of a long sum that do not tile the children (or leaves) of their result node in order
    kBadHeavy = 1u << 14,      // the list of result nodes with many segments names a node that is not one, or misses one
};

struct CsfView {
    int order;
    int64_t nodes[CONSTSTN_MAX_ORDER];
    int64_t dim[CONSTSTN_MAX_ORDER];          // extent of the mode at each level
    const int32_t *idx[CONSTSTN_MAX_ORDER];
    const int64_t *ptr[CONSTSTN_MAX_ORDER];
};

CsfView view_of(const conststn_csf_s *c) {
    CsfView v{};
    v.order = c->order;
    for (int l = 0; l < c->order; ++l) {
        v.nodes[l] = c->nodes[l];
        v.dim[l] = c->dims[c->mode_order[l]];
        v.idx[l] = c->idx[l].p;
        v.ptr[l] = l + 1 < c->order ? c->ptr[l].p : nullptr;
    }
    return v;
}

__global__ void __launch_bounds__(256)
check_level_kernel(CsfView v, int l, unsigned *flags) {
    const int64_t p = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (p >= v.nodes[l]) return;
    unsigned bad = 0;
    const int32_t x = v.idx[l][p];
    if (x < 0 || int64_t(x) >= v.dim[l]) bad |= kBadIndex;
    if (l + 1 < v.order) {
        const int64_t a = v.ptr[l][p], b = v.ptr[l][p + 1];
        if (p == 0 && a != 0) bad |= kBadPtrStart;
        if (b <= a) bad |= kBadPtrOrder;
        if (p == v.nodes[l] - 1 && b != v.nodes[l + 1]) bad |= kBadPtrEnd;
    }
    if (p > 0) {
        bool same_parent = true;               // the roots are siblings of each other
        if (l > 0) {
            const int64_t q = parent_of(v.ptr[l - 1], v.nodes[l - 1], p);
            same_parent = q >= 0 && q < v.nodes[l - 1] && p > v.ptr[l - 1][q];
        }
        if (same_parent && v.idx[l][p - 1] >= x) bad |= kBadSibling;
    }
    if (bad) atomicOr(flags, bad);
}

// MTTKRP tables over a CSF given as raw arrays (the caller's tensor or one of the two sub-tensors)
struct MttkrpView {
    int64_t slices, fibers, nnz, q, n_chunks, out_rows, dim1, dim2;
    const int64_t *ptr0, *ptr1, *slice_leaf, *chunk_fiber;
    const int32_t *chunk_slice, *row_of_slice, *idx1;
    const uint32_t *code;                      // re-encoded leaves, or nullptr
    int n_hot, mode;                           // mode 1: every leaf hot, 2: every leaf cold, 0: marked per leaf
};

__global__ void __launch_bounds__(256)
check_mttkrp_kernel(MttkrpView m, unsigned *flags) {
    const int64_t t = int64_t(blockIdx.x) * 256 + threadIdx.x;
    unsigned bad = 0;
    if (t < m.n_chunks) {
        const int64_t leaf = t * m.q, f = m.chunk_fiber[t];
        const int32_t s = m.chunk_slice[t];
        if (f < 0 || f >= m.fibers || m.ptr1[f] > leaf || m.ptr1[f + 1] <= leaf) bad |= kBadChunk;
        else if (s < 0 || s >= m.slices || m.ptr0[s] > f || m.ptr0[s + 1] <= f) bad |= kBadChunk;
    }
    if (t <= m.slices) {
        const int64_t want = t < m.slices ? m.ptr1[m.ptr0[t]] : m.nnz;
        if (m.slice_leaf[t] != want) bad |= kBadSliceLeaf;
        if (t < m.slices && m.row_of_slice && (m.row_of_slice[t] < 0 || m.row_of_slice[t] >= m.out_rows)) bad |= kBadIndex;
    }
    if (t < m.fibers && (m.idx1[t] < 0 || m.idx1[t] >= m.dim1)) bad |= kBadIndex;
    if (m.code && t < m.nnz) {
        const uint32_t cd = m.code[t];
        const bool hot = m.mode == 1 || (m.mode == 0 && (cd & 0x80000000u));
        const int64_t row = cd & 0x0fffffffu;
        if (hot ? row >= m.n_hot : row >= m.dim2) bad |= kBadCode;
        // the marks: this leaf ends its fiber / its slice exactly when the pointer arrays say so
        const int64_t f = parent_of(m.ptr1, m.fibers, t);
        const bool fiber_end = t + 1 == m.ptr1[f + 1];
        const int64_t s = parent_of(m.ptr0, m.slices, f);
        const bool slice_end = fiber_end && f + 1 == m.ptr0[s + 1];
        if (bool(cd & 0x40000000u) != fiber_end || bool(cd & 0x20000000u) != slice_end) bad |= kBadCode;
    }
    if (bad) atomicOr(flags, bad);
}

struct Ttmc3View {
    int64_t nnz, slices, n_rows, n_items, n_ksteps, n_wg, out_blocks, n_partials, dim1;
    const RowDesc *rows;
    const int64_t *slice_row;
    const SliceItem *items;
    const KStepDesc *ksteps;
    const int32_t *wg_kstep;
};

__global__ void __launch_bounds__(256)
check_ttmc3_kernel(Ttmc3View v, unsigned *flags) {
    const int64_t t = int64_t(blockIdx.x) * 256 + threadIdx.x;
    unsigned bad = 0;
    if (t < v.n_rows) {
        const RowDesc r = v.rows[t];
        if (r.leaf < 0 || r.cnt < 1 || r.cnt > kRowLeaves || r.leaf + r.cnt > v.nnz || r.j < 0 || r.j >= v.dim1) bad |= kBadRow;
    }
    if (t <= v.slices && v.slice_row) {
        const int64_t a = v.slice_row[t];
        if (a < 0 || a > v.n_rows || (t == 0 && a != 0) || (t == v.slices && a != v.n_rows) ||
            (t < v.slices && v.slice_row[t + 1] <= a))
            bad |= kBadRow;
    }
    if (t < v.n_items && v.items) {
        const SliceItem it = v.items[t];
        if (it.slice < 0 || it.slice >= v.slices) bad |= kBadItem;
        else if (v.slice_row && (it.begin < v.slice_row[it.slice] || it.end > v.slice_row[it.slice + 1] || it.end <= it.begin)) bad |= kBadItem;
        if (it.dest >= v.n_partials) bad |= kBadItem;
    }
    if (t < v.n_ksteps && v.ksteps) {
        const KStepDesc k = v.ksteps[t];
        const int n = k.meta & 7;
        if (n < 1 || n > 4 || k.row0 < 0 || int64_t(k.row0) + n > v.n_rows) bad |= kBadKstep;
        if (k.meta & 8) {
            if (k.dest >= 0 ? k.dest >= v.out_blocks : ~k.dest >= v.n_partials) bad |= kBadKstep;
        }
    }
    if (t <= v.n_wg && v.wg_kstep) {
        const int64_t a = v.wg_kstep[t];
        if (a < 0 || a > v.n_ksteps || (t == 0 && a != 0) || (t == v.n_wg && a != v.n_ksteps)) bad |= kBadBatch;
        else if (t < v.n_wg) {
            const int64_t b = v.wg_kstep[t + 1];
            if (b < a) bad |= kBadBatch;
            else if (b > a && b <= v.n_ksteps && !(v.ksteps[b - 1].meta & 8)) bad |= kBadBatch;    // a batch holds whole items
        }
    }
    if (bad) atomicOr(flags, bad);
}

// Generic executor, one statement with a long sum: thread t checks segment t against its neighbours and
// its result node, node t's range of segments, and entry t of the heavy list.
struct GenSegView {
    int64_t out_nodes, n_segs, n_heavy, heavy_limit, seg_len;
    int64_t total;                    // children of the (absent) root, or every leaf, when `range` is null
    const int64_t *range;             // [out_nodes + 1] first child (fused: first leaf) of each result node
    const int64_t *seg_ptr, *seg, *heavy;
};
__global__ void __launch_bounds__(256)
check_gen_segments_kernel(GenSegView v, unsigned *flags) {
    const int64_t t = int64_t(blockIdx.x) * 256 + threadIdx.x;
    unsigned bad = 0;
    if (t <= v.out_nodes) {
        const int64_t a = v.seg_ptr[t];
        if (a < 0 || a > v.n_segs || (t == 0 && a != 0) || (t == v.out_nodes && a != v.n_segs)) bad |= kBadSegment;
        else if (t < v.out_nodes) {
            const int64_t b = v.seg_ptr[t + 1];
            const int64_t lo = v.range ? v.range[t] : 0, hi = v.range ? v.range[t + 1] : v.total;
            if (b < a || b > v.n_segs) bad |= kBadSegment;
            else if (b - a != (hi - lo + v.seg_len - 1) / v.seg_len) bad |= kBadSegment;
            else if (b > a && (v.seg[3 * a + 1] != lo || v.seg[3 * (b - 1) + 2] != hi)) bad |= kBadSegment;
            else if (b - a > v.heavy_limit) {                 // then the node is on the heavy list
                int64_t l0 = 0, l1 = v.n_heavy;
                while (l1 - l0 > 1) {
                    const int64_t mid = (l0 + l1) >> 1;
                    if (v.heavy[mid] <= t) l0 = mid; else l1 = mid;
                }
                if (v.n_heavy == 0 || v.heavy[l0] != t) bad |= kBadHeavy;
            }
        }
    }
    if (t < v.n_segs) {
        const int64_t p = v.seg[3 * t], e0 = v.seg[3 * t + 1], e1 = v.seg[3 * t + 2];
        if (p < 0 || p >= v.out_nodes) bad |= kBadSegment;
        else {
            const int64_t a = v.seg_ptr[p], b = v.seg_ptr[p + 1];
            if (t < a || t >= b || e1 <= e0 || e1 - e0 > v.seg_len) bad |= kBadSegment;
            else if (t + 1 < b && v.seg[3 * (t + 1) + 1] != e1) bad |= kBadSegment;
        }
    }
    if (t < v.n_heavy) {
        const int64_t p = v.heavy[t];
        if (p < 0 || p >= v.out_nodes || (t > 0 && v.heavy[t - 1] >= p)) bad |= kBadHeavy;
        else if (v.seg_ptr[p + 1] - v.seg_ptr[p] <= v.heavy_limit) bad |= kBadHeavy;
    }
    if (bad) atomicOr(flags, bad);
}
// table[x] = below[ptr[x]] for x = 0 .. nodes (below = null: the identity, i.e. table = ptr)
__global__ void __launch_bounds__(256)
check_gen_leaf_table_kernel(const int64_t *table, const int64_t *ptr, const int64_t *below, int64_t nodes, unsigned *flags) {
    const int64_t x = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (x > nodes) return;
    const int64_t c = ptr[x];
    if (table[x] != (below ? below[c] : c)) atomicOr(flags, unsigned(kBadLeafTable));
}

// out[x] = below ? below[ptr[x]] : ptr[x]
__global__ void __launch_bounds__(256)
gather_i64_kernel(const int64_t *ptr, const int64_t *below, int64_t count, int64_t *out) {
    const int64_t x = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (x < count) out[x] = below ? below[ptr[x]] : ptr[x];
}

conststn_status report(unsigned bits, const char *what) {
    if (!bits) return CONSTSTN_OK;
    static const char *const names[] = {"an index outside its extent", "a pointer array that does not start at 0",
                                        "a node without children or decreasing pointers",
                                        "a pointer array that does not end at the next level's node count",
                                        "siblings that are not strictly ascending", "a chunk table entry off its leaf",
                                        "slice_leaf off the pointer arrays", "a re-encoded leaf out of range or with a wrong end mark",
                                        "a row descriptor out of range", "a K-step out of range", "workgroup batches that are not whole items in order",
                                        "an item outside its slice", "a first-leaf table off the pointer arrays",
                                        "segments that do not tile their result node", "a wrong list of nodes with many segments"};
    std::string msg;
    for (int b = 0; b < 15; ++b)
        if (bits & (1u << b)) { if (!msg.empty()) msg += "; "; msg += names[b]; }
    set_error("%s: %s", what, msg.c_str());
    return CONSTSTN_EINVAL;
}

conststn_status run_csf_check(const conststn_csf_s *c, unsigned *dflags) {
    const CsfView v = view_of(c);
    for (int l = 0; l < c->order; ++l) {
        if (c->nodes[l] == 0) continue;
        check_level_kernel<<<dim3(unsigned(div_up(c->nodes[l], 256))), dim3(256)>>>(v, l, dflags);
        CST_HIP(hipGetLastError());
    }
    return CONSTSTN_OK;
}

// The tables of a generic plan: per statement with a long sum the segment table and the list of nodes
// with many segments; per fused statement the first-leaf tables of the levels it walks.
conststn_status check_generic_tables(const conststn_plan_s *plan, unsigned *dflags) {
    const conststn_csf_s *X = plan->X;
    const int n = X->order;
    for (const GenStmt &g : plan->gen) {
        if (g.skip) continue;
        if (g.fused) {
            // (table, level): the result's nodes and the levels between the summed level and the fibers
            std::vector<std::pair<const int64_t *, int>> tables;
            if (g.out_leaf) tables.push_back({g.out_leaf, g.d_out - 1});
            for (int v = 1; v <= g.fused_upper; ++v) tables.push_back({g.leaf_end[v - 1], n - 2 - v});
            for (const auto &tl : tables) {
                const int L = tl.second;
                if (L < 0 || L > n - 2 || !tl.first) { set_error("plan tables: a first-leaf table for level %d of an order-%d tensor", L, n); return CONSTSTN_EINVAL; }
                // compare with the composition from the fibers upwards, one level at a time through scratch tables
                DevBuf<int64_t> scratch[2];
                int which = 0;
                const int64_t *cur = nullptr;                         // first leaves of level l + 1 (null: the leaves themselves)
                for (int l = n - 2; l >= L; --l) {
                    if (l == L) {
                        check_gen_leaf_table_kernel<<<dim3(unsigned(div_up(X->nodes[l] + 1, 256))), dim3(256)>>>(
                            tl.first, X->ptr[l].p, cur, X->nodes[l], dflags);
                        CST_HIP(hipGetLastError());
                        break;
                    }
                    DevBuf<int64_t> &mine = scratch[which];
                    which ^= 1;
                    CST_TRY(mine.alloc(size_t(X->nodes[l] + 1)));
                    gather_i64_kernel<<<dim3(unsigned(div_up(X->nodes[l] + 1, 256))), dim3(256)>>>(X->ptr[l].p, cur, X->nodes[l] + 1, mine.p);
                    CST_HIP(hipGetLastError());
                    CST_HIP(hipDeviceSynchronize());                     // the other buffer may be released at the next turn
                    cur = mine.p;
                }
                CST_HIP(hipDeviceSynchronize());
            }
        }
        if (g.n_segs > 0) {
            GenSegView v{};
            v.out_nodes = g.out_nodes;
            v.n_segs = g.n_segs;
            v.n_heavy = g.n_heavy;
            v.heavy_limit = kGenHeavy;
            v.seg_len = g.fused ? kGenLeafSegment : kGenSegment;
            v.total = g.fused ? X->nnz : X->nodes[0];
            v.range = g.fused ? g.out_leaf : (g.d_out > 0 ? X->ptr[g.d_out - 1].p : nullptr);
            v.seg_ptr = plan->gen_tables[size_t(g.seg_table)]->p;
            v.seg = plan->gen_tables[size_t(g.seg_table) + 1]->p;
            v.heavy = plan->gen_tables[size_t(g.seg_table) + 2]->p;
            const int64_t threads = std::max(std::max(v.out_nodes + 1, v.n_segs), v.n_heavy);
            check_gen_segments_kernel<<<dim3(unsigned(div_up(threads, 256))), dim3(256)>>>(v, dflags);
            CST_HIP(hipGetLastError());
        }
    }
    CST_HIP(hipDeviceSynchronize());
    return CONSTSTN_OK;
}

}  // namespace

}  // namespace cst

using namespace cst;

extern "C" conststn_status conststn_csf_check(const conststn_csf_t *csf) {
    clear_error();
    if (!csf) { set_error("null argument"); return CONSTSTN_EINVAL; }
    for (int l = 0; l + 1 < csf->order; ++l)
        if ((csf->nodes[l] == 0) != (csf->nodes[l + 1] == 0)) { set_error("CSF: a level is empty and the next is not"); return CONSTSTN_EINVAL; }
    if (csf->order > 0 && csf->nodes[csf->order - 1] != csf->nnz) { set_error("CSF: the leaf level does not hold nnz nodes"); return CONSTSTN_EINVAL; }
    DevBuf<unsigned> flags;
    CST_TRY(flags.alloc(1));
    CST_HIP(hipMemset(flags.p, 0, sizeof(unsigned)));
    CST_TRY(run_csf_check(csf, flags.p));
    unsigned h = 0;
    CST_HIP(hipMemcpy(&h, flags.p, sizeof(h), hipMemcpyDeviceToHost));
    return report(h, "CSF");
}

extern "C" conststn_status conststn_plan_check(const conststn_plan_t *plan) {
    clear_error();
    if (!plan) { set_error("null argument"); return CONSTSTN_EINVAL; }
    const conststn_csf_s *X = plan->X;
    if (!X || (plan->family != FAM_MTTKRP3 && plan->family != FAM_TTMC3 && plan->family != FAM_GENERIC)) {
        set_error("the table check covers the order-3 MTTKRP and TTMc plans and those of the generic executor");
        return CONSTSTN_EUNSUPPORTED;
    }
    DevBuf<unsigned> flags;
    CST_TRY(flags.alloc(1));
    CST_HIP(hipMemset(flags.p, 0, sizeof(unsigned)));
    CST_TRY(run_csf_check(X, flags.p));                    // the tensor the kernels walk (the private copy, if one was made)
    if (plan->family == FAM_GENERIC) {
        CST_TRY(check_generic_tables(plan, flags.p));
        unsigned hg = 0;
        CST_HIP(hipMemcpy(&hg, flags.p, sizeof(hg), hipMemcpyDeviceToHost));
        return report(hg, "plan tables");
    }
    const int64_t dim1 = X->dims[X->mode_order[1]], dim2 = X->dims[X->mode_order[2]];
    if (X->nnz > 0 && plan->family == FAM_MTTKRP3) {
        auto launch = [&](const MttkrpView &m) -> conststn_status {
            const int64_t n = std::max(std::max(m.n_chunks, m.slices + 1), std::max(m.fibers, m.code ? m.nnz : 0));
            check_mttkrp_kernel<<<dim3(unsigned(div_up(n, 256))), dim3(256)>>>(m, flags.p);
            CST_HIP(hipGetLastError());
            return CONSTSTN_OK;
        };
        if (plan->split) {
            for (int part = 0; part < 2; ++part) {
                const MttkrpPart &P = plan->part[part];
                if (P.nnz == 0) continue;
                MttkrpView m{P.slices, P.fibers, P.nnz, P.chunk_q, P.n_chunks, plan->out_rows, dim1, dim2,
                             P.ptr0.p, P.ptr1.p, P.slice_leaf.p, P.chunk_fiber.p, P.chunk_slice.p, P.row_of_slice.p,
                             P.idx1.p, P.code.p, plan->n_hot, part == 0 ? 1 : 2};
                CST_TRY(launch(m));
            }
        } else {
            MttkrpView m{X->nodes[0], X->nodes[1], X->nnz, plan->chunk_q, plan->n_chunks, plan->out_rows, dim1, dim2,
                         X->ptr[0].p, X->ptr[1].p, plan->slice_leaf.p, plan->chunk_fiber.p, plan->chunk_slice.p, nullptr,
                         X->idx[1].p, plan->leaf_code.p, plan->n_hot, 0};
            CST_TRY(launch(m));
        }
    }
    if (X->nnz > 0 && plan->family == FAM_TTMC3 && plan->use_rows) {
        Ttmc3View v{X->nnz, X->nodes[0], plan->n_rows_tab, plan->n_items, plan->use_stream ? plan->n_ksteps : 0,
                    plan->use_stream ? plan->n_stream_wg : 0, plan->out_rows, plan->n_partials, dim1,
                    plan->rows.p, plan->slice_row.p, plan->items.p, plan->use_stream ? plan->ksteps.p : nullptr,
                    plan->use_stream ? plan->wg_kstep.p : nullptr};
        const int64_t n = std::max(std::max(v.n_rows, v.slices + 1), std::max(std::max(v.n_items, v.n_ksteps), v.n_wg + 1));
        check_ttmc3_kernel<<<dim3(unsigned(div_up(n, 256))), dim3(256)>>>(v, flags.p);
        CST_HIP(hipGetLastError());
    }
    unsigned h = 0;
    CST_HIP(hipMemcpy(&h, flags.p, sizeof(h), hipMemcpyDeviceToHost));
    return report(h, "plan tables");
}
