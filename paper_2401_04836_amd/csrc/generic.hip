// Generic executor for contraction trees over ONE CSF tensor and dense operands -- any order,
// any rank extents, any legal loop order and fusion choice (Sec. 2.2 / 4.2: a schedule is a tree
// of binary contractions; fusion changes the size of the intermediates, never their values).
//
// Supported shape of a tree: the CSF operand X is contracted from its innermost level upwards.
// Every tensor on the path from X to the result is indexed by a PREFIX of X's CSF levels plus
// dense indices, so it is stored as one dense block per CSF node of that depth ("sparse like
// X above, dense below" -- the sparsity structure the paper's Sec. 2.1 assigns to a contraction
// result, restricted to prefixes).  A statement
//        out[x_0..x_{d'-1}, O...] = in[x_0..x_{d-1}, I...] * F[...]        (d' <= d)
// sums over the CSF levels d'..d-1 and over the dense indices that are in `in` or F but not in
// `out`.  F is a dense operand or the result of a dense-only subtree, and may be indexed by the
// contracted level indices and by dense indices.  Statements whose two inputs are both dense are
// handled by the same kernel with an empty prefix.
//
// One thread per output element walks the CSF subtree below its node and the contracted dense
// indices in a fixed order: deterministic, no atomics, intermediates held whole in device
// memory.  This is the slow, always-applicable path; the tuned kernels of the other files take
// the schedules they match.
#include <algorithm>
#include <set>

#include "plan.hpp"

namespace cst {

__global__ void __launch_bounds__(256)
generic_stmt_kernel(GenStmt g) {
    const int64_t gid = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (gid >= g.out_nodes * g.out_block) return;
    const int64_t p = gid / g.out_block;
    int64_t rem = gid - p * g.out_block;
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
    } else {
        int64_t cur[CONSTSTN_MAX_ORDER], end[CONSTSTN_MAX_ORDER], foff[CONSTSTN_MAX_ORDER];
        int l = 0;
        if (g.d_out == 0) { cur[0] = 0; end[0] = g.roots; }
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
    const int64_t row = g.scatter_rows ? int64_t(g.idx[0][p]) : p;
    g.out[row * g.out_block + out_off] = acc;
}

namespace {

// a tensor on the way from X to the result, or a dense one
struct GenTensor {
    int depth = 0;                        // CSF prefix depth (0 = dense)
    bool leaf = false;                    // X itself
    std::vector<std::string> dense;       // dense index names in storage order (last fastest)
    int operand = -1;                     // dense operand ordinal among ALL operands, or -1
    int buffer = -1;                      // intermediate buffer number, or -1
    bool from_x = false;                  // descends from the CSF operand
};

int find_name(const std::vector<std::string> &v, const std::string &n) {
    for (size_t i = 0; i < v.size(); ++i) if (v[i] == n) return int(i);
    return -1;
}

}  // namespace

conststn_status build_generic(conststn_plan_s *plan) {
    Schedule &s = plan->sched;
    const int m = int(s.stmts.size());
    int xop = -1;
    for (size_t o = 0; o < s.operands.size(); ++o)
        if (s.operands[o].kind == CONSTSTN_OPERAND_CSF) {
            if (xop >= 0) { set_error("the generic executor takes one CSF operand; the schedule has more"); return CONSTSTN_EUNSUPPORTED; }
            xop = int(o);
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

    std::vector<GenTensor> result(m);             // the tensor each statement produces
    plan->gen.clear();
    plan->gen_buffers.clear();
    std::vector<int64_t> buffer_elems;
    auto tensor_of_ref = [&](const Ref &r, int src, int op, GenTensor &t) -> conststn_status {
        if (src >= 0) { t = result[src]; return CONSTSTN_OK; }
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
        return CONSTSTN_OK;
    };

    for (int p = 0; p < m; ++p) {
        const Stmt &st = s.stmts[p];
        GenTensor ta, tb;
        CST_TRY(tensor_of_ref(st.a, st.src_a, st.op_a, ta));
        CST_TRY(tensor_of_ref(st.b, st.src_b, st.op_b, tb));
        if (ta.from_x && tb.from_x) { set_error("statement %d multiplies two tensors that both descend from the CSF operand", p); return CONSTSTN_EUNSUPPORTED; }
        const GenTensor &in = tb.from_x ? tb : ta;            // sparse side (or first dense input)
        const GenTensor &fa = tb.from_x ? ta : tb;            // dense side
        if (fa.from_x) { set_error("internal: dense side descends from the CSF operand"); return CONSTSTN_EINVAL; }
        const int d_in = in.from_x ? in.depth : 0;

        // output: leading CSF level names (a prefix, in level order), then dense names
        int d_out = 0;
        while (d_out < int(st.out.idx.size()) && d_out < d_in && st.out.idx[d_out] == level_name[d_out]) ++d_out;
        std::vector<std::string> out_dense(st.out.idx.begin() + d_out, st.out.idx.end());
        for (const auto &nm : out_dense)
            if (in.from_x && level_of(nm) >= 0 && level_of(nm) < d_in) {
                set_error("statement %d: result %s keeps CSF index %s without the levels above it; the generic "
                          "executor stores results by CSF prefix only", p, st.out.name.c_str(), nm.c_str());
                return CONSTSTN_EUNSUPPORTED;
            }
        // dense loop indices
        std::vector<std::string> red;
        auto consider = [&](const std::string &nm) {
            if (in.from_x && level_of(nm) >= 0 && level_of(nm) < d_in) return;        // a CSF level
            if (find_name(out_dense, nm) >= 0 || find_name(red, nm) >= 0) return;
            red.push_back(nm);
        };
        for (const auto &nm : in.dense) consider(nm);
        for (const auto &nm : fa.dense) consider(nm);
        if (out_dense.size() + red.size() > size_t(kGenMaxIdx)) { set_error("statement %d has more than %d dense indices", p, kGenMaxIdx); return CONSTSTN_EUNSUPPORTED; }

        GenStmt g{};
        g.d_in = d_in;
        g.d_out = d_out;
        g.in_is_leaf = in.leaf ? 1 : 0;
        g.n_out = int(out_dense.size());
        g.n_red = int(red.size());
        std::vector<std::string> loopn = out_dense;
        loopn.insert(loopn.end(), red.begin(), red.end());
        for (size_t q = 0; q < loopn.size(); ++q) g.extent[q] = s.extent[loopn[q]];
        // strides of a dense index list stored row-major in the given order
        auto strides = [&](const std::vector<std::string> &names, std::map<std::string, int64_t> &out) {
            int64_t stride = 1;
            for (int q = int(names.size()) - 1; q >= 0; --q) { out[names[q]] = stride; stride *= s.extent[names[q]]; }
            return stride;
        };
        std::map<std::string, int64_t> sin, sf, sout;
        g.in_block = strides(in.dense, sin);
        strides(fa.dense, sf);
        g.out_block = strides(out_dense, sout);
        for (size_t q = 0; q < loopn.size(); ++q) {
            g.in_stride[q] = sin.count(loopn[q]) ? sin[loopn[q]] : 0;
            g.f_stride[q] = sf.count(loopn[q]) ? sf[loopn[q]] : 0;
            g.out_stride[q] = q < out_dense.size() ? sout[loopn[q]] : 0;
        }
        for (const auto &nm : fa.dense) {
            const int L = in.from_x ? level_of(nm) : -1;
            if (L < 0 || L >= d_in) continue;
            if (L < d_out) {
                set_error("statement %d: dense input is indexed by CSF index %s that the result keeps; not implemented "
                          "in the generic executor", p, nm.c_str());
                return CONSTSTN_EUNSUPPORTED;
            }
            g.f_level_stride[L] = sf[nm];
        }
        // where the inputs live
        g.in_operand = in.operand;
        g.in_buffer = in.buffer;
        g.f_operand = fa.operand;
        g.f_buffer = fa.buffer;
        g.out_nodes = d_out == 0 ? 1 : csf->nodes[d_out - 1];
        g.roots = csf->nodes[0];
        for (int l = 0; l < n; ++l) {
            g.idx[l] = csf->idx[l].p;
            g.ptr[l] = l + 1 < n ? csf->ptr[l].p : nullptr;
        }
        // the result
        GenTensor &res = result[p];
        res.depth = d_out;
        res.from_x = in.from_x;
        res.dense = out_dense;
        if (st.consumer >= 0) {
            res.buffer = int(buffer_elems.size());
            buffer_elems.push_back(g.out_nodes * g.out_block);
            g.out_buffer = res.buffer;
        } else {
            if (res.from_x && d_out > 1) {
                set_error("the result keeps %d CSF indices; the generic executor writes dense results or one "
                          "row block per root index", d_out);
                return CONSTSTN_EUNSUPPORTED;
            }
            g.out_buffer = -1;
            g.scatter_rows = (d_out == 1 && !plan->compact) ? 1 : 0;
            plan->gen_rooted = d_out == 1;
            plan->row_elems = g.out_block;
        }
        plan->gen.push_back(g);
    }
    // intermediates, held whole
    int64_t total = 0;
    for (int64_t e : buffer_elems) total += e;
    const int64_t cap = env_int("CONSTSTN_GENERIC_MAX_GB", 64) << 27;      // doubles
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
    // rows of root indices that hold no nonzero are never written by a kernel
    if (plan->gen_rooted && !plan->compact && csf->nodes[0] < plan->out_rows)
        CST_TRY(zero_fill(out, plan->out_rows * plan->row_elems, stream));
    ProfScope prof(plan, stream);
    for (const GenStmt &g0 : plan->gen) {
        GenStmt g = g0;
        auto where = [&](int operand, int buffer) -> const double * {
            if (buffer >= 0) return plan->gen_buffers[size_t(buffer)]->p;
            if (operand >= 0) return dense[s.operands[size_t(operand)].dense_ordinal];
            return nullptr;
        };
        g.in = g.in_is_leaf ? csf->vals.p : where(g.in_operand, g.in_buffer);      // X: the leaf values
        g.f = where(g.f_operand, g.f_buffer);
        g.out = g.out_buffer >= 0 ? plan->gen_buffers[size_t(g.out_buffer)]->p : out;
        if (!g.in || !g.f || !g.out) { set_error("internal: unresolved tensor in the generic executor"); return CONSTSTN_EINVAL; }
        const int64_t total = g.out_nodes * g.out_block;
        if (total == 0) continue;
        if (total > (int64_t(1) << 31) * 256) { set_error("statement result too large for one launch"); return CONSTSTN_EUNSUPPORTED; }
        generic_stmt_kernel<<<dim3(unsigned((total + 255) / 256)), dim3(256), 0, stream>>>(g);
        CST_HIP(hipGetLastError());
    }
    return CONSTSTN_OK;
}

}  // namespace cst
