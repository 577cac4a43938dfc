// The C ABI of the conststn library: argument checking, handle lifetime, kernel-family
// matching of a validated schedule, and dispatch.  See include/conststn.h for the contract.
#include <algorithm>
#include <cstring>
#include <set>
#include <new>

#include "plan.hpp"

namespace cst {

static thread_local std::string g_error;

void set_error(const char *fmt, ...) {
    char buf[1024];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    g_error = buf;
}
const char *get_error() { return g_error.c_str(); }
void clear_error() { g_error.clear(); }

// ---- kernel-family matching -------------------------------------------------------------
//
// "Chain" families (TTMc, MTTKRP): one CSF operand X with levels x0 > x1 > ... > x_{n-1};
// statement p contracts the innermost remaining sparse index x_{n-1-p} with a dense factor
// F[x, r]; every producer is fused with its consumer on all remaining sparse indices.
static conststn_status match_chain(conststn_plan_s *plan) {
    Schedule &s = plan->sched;
    const int m = int(s.stmts.size());
    const Stmt &s0 = s.stmts[0];
    int xop = -1;
    const Ref *xref = nullptr;
    if (s0.op_a >= 0 && s.operands[s0.op_a].kind == CONSTSTN_OPERAND_CSF) { xop = s0.op_a; xref = &s0.a; }
    else if (s0.op_b >= 0 && s.operands[s0.op_b].kind == CONSTSTN_OPERAND_CSF) { xop = s0.op_b; xref = &s0.b; }
    if (xop < 0) return CONSTSTN_EUNSUPPORTED;
    const OperandInfo &X = s.operands[xop];
    const int n = X.order;
    if (m != n - 1 || n < 3 || n > 4) return CONSTSTN_EUNSUPPORTED;
    if (!X.csf) { set_error("CSF operand %s has no handle", X.name.c_str()); return CONSTSTN_EINVAL; }
    const std::vector<std::string> &x = xref->idx;
    std::vector<std::string> ranks;          // rank index introduced by statement p
    for (int p = 0; p < m; ++p) {
        const Stmt &st = s.stmts[p];
        // which input is the factor, which the running tensor
        const Ref *fac = nullptr, *run = nullptr;
        int fop = -1;
        if (p == 0) {
            run = xref;
            fac = (xref == &st.a) ? &st.b : &st.a;
            fop = (xref == &st.a) ? st.op_b : st.op_a;
        } else {
            if (st.src_a == p - 1) { run = &st.a; fac = &st.b; fop = st.op_b; }
            else if (st.src_b == p - 1) { run = &st.b; fac = &st.a; fop = st.op_a; }
            else return CONSTSTN_EUNSUPPORTED;
        }
        (void)run;
        if (fop < 0 || s.operands[fop].kind != CONSTSTN_OPERAND_DENSE || s.operands[fop].order != 2)
            return CONSTSTN_EUNSUPPORTED;
        const int level = n - 1 - p;
        if (fac->idx[0] != x[level]) return CONSTSTN_EUNSUPPORTED;      // F[x_level, r], row-major
        ranks.push_back(fac->idx[1]);
        for (int l = 0; l < n; ++l) if (fac->idx[1] == x[l]) return CONSTSTN_EUNSUPPORTED;
        plan->factor_of_level[level] = s.operands[fop].dense_ordinal;
        plan->rank_of_level[level] = int(s.operands[fop].dims[1]);
        // result holds the remaining sparse indices and the rank indices so far
        std::set<std::string> want(x.begin(), x.begin() + level);
        want.insert(ranks.begin(), ranks.end());
        std::set<std::string> got(st.out.idx.begin(), st.out.idx.end());
        if (want != got) return CONSTSTN_EUNSUPPORTED;
        // loops: remaining sparse indices in level order first
        for (int l = 0; l <= level; ++l)
            if (st.loops[l] != x[l]) return CONSTSTN_EUNSUPPORTED;
        if (p + 1 < m && st.fused_depth != level) {
            set_error("statement %d is fused to depth %d; the TTMc/MTTKRP kernels need the full sparse prefix (%d)",
                      p, st.fused_depth, level);
            return CONSTSTN_EUNSUPPORTED;
        }
    }
    bool all_same = true, all_distinct = true;
    for (int p = 1; p < m; ++p) {
        if (ranks[p] != ranks[0]) all_same = false;
        for (int q = 0; q < p; ++q) if (ranks[p] == ranks[q]) all_distinct = false;
    }
    const Stmt &last = s.stmts[m - 1];
    if (all_same && m > 1) {
        // MTTKRP: batch index r; output M[x0, r]
        if (n != 3) { set_error("MTTKRP kernels exist for order-3 tensors only"); return CONSTSTN_EUNSUPPORTED; }
        if (last.out.idx.size() != 2 || last.out.idx[0] != x[0] || last.out.idx[1] != ranks[0]) return CONSTSTN_EUNSUPPORTED;
        for (int l = 2; l < n; ++l)
            if (plan->rank_of_level[l] != plan->rank_of_level[1]) { set_error("batch index with two extents"); return CONSTSTN_ESCHED; }
        plan->family = FAM_MTTKRP3;
        plan->row_elems = plan->rank_of_level[1];
    } else if (all_distinct) {
        // TTMc: output Y[x0, r(level 1), r(level 2), ...]
        if (int(last.out.idx.size()) != n || last.out.idx[0] != x[0]) return CONSTSTN_EUNSUPPORTED;
        for (int l = 1; l < n; ++l)
            if (last.out.idx[l] != ranks[n - 1 - l]) {
                set_error("TTMc output must list the rank indices in CSF level order after the root index");
                return CONSTSTN_EUNSUPPORTED;
            }
        plan->family = n == 3 ? FAM_TTMC3 : FAM_TTMC4;
        plan->row_elems = 1;
        for (int l = 1; l < n; ++l) plan->row_elems *= plan->rank_of_level[l];
    } else {
        return CONSTSTN_EUNSUPPORTED;
    }
    plan->X = X.csf;
    return CONSTSTN_OK;
}

// Three-tensor network  T[i,k,l] = U[i,k,j] V[j,l] ; Z[i,m] = T[i,k,l] W[k,l,m], fused on i,k.
static conststn_status match_sptn3(conststn_plan_s *plan) {
    Schedule &s = plan->sched;
    if (s.stmts.size() != 2) return CONSTSTN_EUNSUPPORTED;
    const Stmt &p0 = s.stmts[0], &p1 = s.stmts[1];
    const Ref *u = nullptr, *v = nullptr;
    int uop = -1, vop = -1;
    if (p0.op_a >= 0 && s.operands[p0.op_a].kind == CONSTSTN_OPERAND_CSF) { u = &p0.a; uop = p0.op_a; v = &p0.b; vop = p0.op_b; }
    else if (p0.op_b >= 0 && s.operands[p0.op_b].kind == CONSTSTN_OPERAND_CSF) { u = &p0.b; uop = p0.op_b; v = &p0.a; vop = p0.op_a; }
    if (uop < 0 || vop < 0 || s.operands[vop].kind != CONSTSTN_OPERAND_DENSE) return CONSTSTN_EUNSUPPORTED;
    if (s.operands[uop].order != 3 || s.operands[vop].order != 2) return CONSTSTN_EUNSUPPORTED;
    const Ref *t = nullptr, *w = nullptr;
    int wop = -1;
    if (p1.src_a == 0) { t = &p1.a; w = &p1.b; wop = p1.op_b; }
    else if (p1.src_b == 0) { t = &p1.b; w = &p1.a; wop = p1.op_a; }
    if (!t || wop < 0 || s.operands[wop].kind != CONSTSTN_OPERAND_CSF || s.operands[wop].order != 3) return CONSTSTN_EUNSUPPORTED;
    const std::string &i = u->idx[0], &k = u->idx[1], &j = u->idx[2];
    if (v->idx[0] != j) return CONSTSTN_EUNSUPPORTED;
    const std::string &l = v->idx[1];
    if (w->idx[0] != k || w->idx[1] != l) return CONSTSTN_EUNSUPPORTED;
    const std::string &mm = w->idx[2];
    std::set<std::string> tset(p0.out.idx.begin(), p0.out.idx.end());
    if (tset != std::set<std::string>{i, k, l}) return CONSTSTN_EUNSUPPORTED;
    if (p1.out.idx.size() != 2 || p1.out.idx[0] != i || p1.out.idx[1] != mm) return CONSTSTN_EUNSUPPORTED;
    if (std::set<std::string>{i, j, k, l, mm}.size() != 5) return CONSTSTN_EUNSUPPORTED;
    if (p0.fused_depth != 2) {
        set_error("the three-tensor kernel needs producer and consumer fused on the two outer loops (depth 2), got %d",
                  p0.fused_depth);
        return CONSTSTN_EUNSUPPORTED;
    }
    if (!s.operands[uop].csf || !s.operands[wop].csf) { set_error("CSF operand without handle"); return CONSTSTN_EINVAL; }
    plan->family = FAM_SPTN3;
    plan->X = s.operands[uop].csf;
    plan->W = s.operands[wop].csf;
    plan->row_elems = s.extent[mm];
    plan->factor_of_level[0] = s.operands[vop].dense_ordinal;
    return CONSTSTN_OK;
}

// Chain of three sparse tensors with a sparse result (Sec. 5.1):
//   T[K,i,v] = I[K,u,v] * C[i,u] ; E[K,i,m] = T[K,i,v] * P[m,v]                      (unrestricted)
//   T[K,i,v] = I[K,u,v] * C[i,u] ; F[K,i,v] = T[K,i,v] * L[K,i] ; E[K,i,m] = F[K,i,v] * P[m,v]
// every operand a CSF tensor whose reference lists its indices in level order.
static conststn_status match_spchain3(conststn_plan_s *plan) {
    Schedule &s = plan->sched;
    const size_t m = s.stmts.size();
    if (m != 2 && m != 3) return CONSTSTN_EUNSUPPORTED;
    for (const auto &o : s.operands) if (o.kind != CONSTSTN_OPERAND_CSF) return CONSTSTN_EUNSUPPORTED;
    if (s.operands.size() != m + 1) return CONSTSTN_EUNSUPPORTED;
    const Stmt &p0 = s.stmts[0];
    if (p0.op_a < 0 || p0.op_b < 0) return CONSTSTN_EUNSUPPORTED;
    const Ref *ri = &p0.a, *rc = &p0.b;
    int iop = p0.op_a, cop = p0.op_b;
    if (s.operands[iop].order != 3) { std::swap(ri, rc); std::swap(iop, cop); }
    if (s.operands[iop].order != 3 || s.operands[cop].order != 2) return CONSTSTN_EUNSUPPORTED;
    const std::string &K = ri->idx[0], &u = ri->idx[1], &v = ri->idx[2];
    const std::string &i = rc->idx[0];
    if (rc->idx[1] != u) return CONSTSTN_EUNSUPPORTED;
    if (std::set<std::string>(p0.out.idx.begin(), p0.out.idx.end()) != std::set<std::string>{K, i, v}) return CONSTSTN_EUNSUPPORTED;
    // the other input of a later statement, which must be an operand
    auto partner = [&](const Stmt &st, int src, const Ref *&r, int &op) {
        if (st.src_a == src && st.op_b >= 0) { r = &st.b; op = st.op_b; return true; }
        if (st.src_b == src && st.op_a >= 0) { r = &st.a; op = st.op_a; return true; }
        return false;
    };
    const Ref *rl = nullptr, *rp = nullptr;
    int lop = -1, pop = -1;
    if (m == 3) {
        const Stmt &p1 = s.stmts[1];
        if (!partner(p1, 0, rl, lop) || s.operands[lop].order != 2) return CONSTSTN_EUNSUPPORTED;
        if (rl->idx[0] != K || rl->idx[1] != i) return CONSTSTN_EUNSUPPORTED;
        if (std::set<std::string>(p1.out.idx.begin(), p1.out.idx.end()) != std::set<std::string>{K, i, v}) return CONSTSTN_EUNSUPPORTED;
    }
    const Stmt &pe = s.stmts[m - 1];
    if (!partner(pe, int(m) - 2, rp, pop) || s.operands[pop].order != 2) return CONSTSTN_EUNSUPPORTED;
    const std::string &mm = rp->idx[0];
    if (rp->idx[1] != v) return CONSTSTN_EUNSUPPORTED;
    if (pe.out.idx != std::vector<std::string>{K, i, mm}) return CONSTSTN_EUNSUPPORTED;
    if (std::set<std::string>{K, i, u, v, mm}.size() != 5) return CONSTSTN_EUNSUPPORTED;
    for (size_t p = 0; p + 1 < m; ++p)
        if (s.stmts[p].fused_depth != 2) {
            set_error("the sparse-chain kernel needs every producer fused with its consumer on the two outer loops "
                      "(depth 2); statement %zu has depth %d", p, s.stmts[p].fused_depth);
            return CONSTSTN_EUNSUPPORTED;
        }
    if (plan->compact) { set_error("the result of the sparse chain is sparse; the compact-rows flag does not apply"); return CONSTSTN_EINVAL; }
    plan->family = FAM_SPCHAIN3;
    plan->X = s.operands[iop].csf;
    plan->sc_C = s.operands[cop].csf;
    plan->sc_P = s.operands[pop].csf;
    plan->sc_L = lop >= 0 ? s.operands[lop].csf : nullptr;
    if (!plan->X || !plan->sc_C || !plan->sc_P || (lop >= 0 && !plan->sc_L)) { set_error("CSF operand without handle"); return CONSTSTN_EINVAL; }
    return CONSTSTN_OK;
}

// Four-index product of Sec. 5.1: one statement V[i,j,m,n] = Ea[i,K,m] * Eb[j,K,n], both operands CSF
// tensors of order 3 referenced in level order, sparse result.
static conststn_status match_sppair4(conststn_plan_s *plan) {
    Schedule &s = plan->sched;
    if (s.stmts.size() != 1 || s.operands.size() != 2) return CONSTSTN_EUNSUPPORTED;
    const Stmt &p0 = s.stmts[0];
    if (p0.op_a < 0 || p0.op_b < 0 || p0.op_a == p0.op_b) return CONSTSTN_EUNSUPPORTED;
    const OperandInfo &oa = s.operands[p0.op_a], &ob = s.operands[p0.op_b];
    if (oa.kind != CONSTSTN_OPERAND_CSF || ob.kind != CONSTSTN_OPERAND_CSF || oa.order != 3 || ob.order != 3) return CONSTSTN_EUNSUPPORTED;
    if (p0.a.idx[1] != p0.b.idx[1]) return CONSTSTN_EUNSUPPORTED;
    if (p0.out.idx != std::vector<std::string>{p0.a.idx[0], p0.b.idx[0], p0.a.idx[2], p0.b.idx[2]}) return CONSTSTN_EUNSUPPORTED;
    if (std::set<std::string>{p0.a.idx[0], p0.a.idx[1], p0.a.idx[2], p0.b.idx[0], p0.b.idx[2]}.size() != 5) return CONSTSTN_EUNSUPPORTED;
    if (plan->compact) { set_error("the result of the sparse product is sparse; the compact-rows flag does not apply"); return CONSTSTN_EINVAL; }
    if (!oa.csf || !ob.csf) { set_error("CSF operand without handle"); return CONSTSTN_EINVAL; }
    plan->family = FAM_SPPAIR4;
    plan->X = oa.csf;
    plan->W = ob.csf;
    return CONSTSTN_OK;
}

// Order-3 MTTKRP or TTMc whose result is indexed by a level of X other than the root, written as any
// legal two-statement tree (the factor of the leaf level first, or the two dense factors first, ...):
//      MTTKRP   M[x_m, r]      = X[x_0,x_1,x_2] . Fa[x_a, r]  . Fb[x_b, r]
//      TTMc     Y[x_m, ra, rb] = X[x_0,x_1,x_2] . Fa[x_a, ra] . Fb[x_b, rb]          {m, a, b} = {0, 1, 2}, m != 0
// The value does not depend on the tree (Sec. 2.2), so the plan re-sorts a private copy of X with level m
// at the root and hands it to the kernels of the root-mode case.
static conststn_status match_rerooted(conststn_plan_s *plan) {
    Schedule &s = plan->sched;
    if (s.stmts.size() != 2 || s.operands.size() != 3) return CONSTSTN_EUNSUPPORTED;
    int xop = -1;
    for (size_t o = 0; o < s.operands.size(); ++o)
        if (s.operands[o].kind == CONSTSTN_OPERAND_CSF) { if (xop >= 0) return CONSTSTN_EUNSUPPORTED; xop = int(o); }
    if (xop < 0 || s.operands[xop].order != 3 || !s.operands[xop].csf) return CONSTSTN_EUNSUPPORTED;
    // references to the operands, and what each statement's other input still holds when a factor joins
    const Ref *xref = nullptr;
    struct Fac { int level = -1; int ordinal = -1; std::string rank; int extent = 0; };
    std::vector<Fac> facs;
    std::vector<std::pair<const Ref *, const Ref *>> joins;       // (factor reference, the other input)
    for (const Stmt &st : s.stmts) {
        const Ref *refs[2] = {&st.a, &st.b};
        const int ops[2] = {st.op_a, st.op_b};
        for (int side = 0; side < 2; ++side) {
            if (ops[side] < 0) continue;
            if (ops[side] == xop) { if (xref) return CONSTSTN_EUNSUPPORTED; xref = refs[side]; continue; }
            const OperandInfo &o = s.operands[ops[side]];
            if (o.kind != CONSTSTN_OPERAND_DENSE || o.order != 2) return CONSTSTN_EUNSUPPORTED;
            joins.push_back({refs[side], refs[1 - side]});
        }
    }
    if (!xref || joins.size() != 2) return CONSTSTN_EUNSUPPORTED;
    const std::vector<std::string> &x = xref->idx;
    for (const auto &jn : joins) {
        const Ref *f = jn.first;
        Fac fc;
        for (int l = 0; l < 3; ++l) if (f->idx[0] == x[l]) fc.level = l;       // F[x_l, r], row-major
        if (fc.level < 0) return CONSTSTN_EUNSUPPORTED;
        fc.rank = f->idx[1];
        for (int l = 0; l < 3; ++l) if (fc.rank == x[l]) return CONSTSTN_EUNSUPPORTED;
        for (const auto &o : s.operands)
            if (o.name == f->name) { fc.ordinal = o.dense_ordinal; fc.extent = int(o.dims[1]); }
        facs.push_back(fc);
    }
    if (facs[0].level == facs[1].level || facs[0].ordinal == facs[1].ordinal) return CONSTSTN_EUNSUPPORTED;
    const int m = 3 - facs[0].level - facs[1].level;
    if (m == 0) return CONSTSTN_EUNSUPPORTED;           // the root-mode kernels take that, without a copy
    // the tree must be this network: every statement keeps x_m and the rank indices, and a level's index is
    // summed only by the statement that joins its factor (with X or the other intermediate) or after it
    const Stmt &first = s.stmts[0], &last = s.stmts[1];
    if (first.consumer != 1) return CONSTSTN_EUNSUPPORTED;
    auto holds = [](const Ref &r, const std::string &i) { return std::find(r.idx.begin(), r.idx.end(), i) != r.idx.end(); };
    const bool x_first = first.op_a == xop || first.op_b == xop;
    for (const Fac &fc : facs) {
        // where does this factor join?
        const bool in_first = (first.op_a >= 0 && s.operands[first.op_a].dense_ordinal == fc.ordinal && first.op_a != xop) ||
                              (first.op_b >= 0 && s.operands[first.op_b].dense_ordinal == fc.ordinal && first.op_b != xop);
        if (!holds(first.out, fc.rank) && in_first) return CONSTSTN_EUNSUPPORTED;          // a rank index summed away
        if (in_first && x_first) continue;                    // joined with X itself: x_l is there
        if (in_first && !x_first) {                           // the two factors first: both level indices must survive
            if (!holds(first.out, x[fc.level])) return CONSTSTN_EUNSUPPORTED;
            continue;
        }
        // joined by the last statement: the intermediate must still hold x_l (when X came first) -- or X itself does
        if (x_first && !holds(first.out, x[fc.level])) return CONSTSTN_EUNSUPPORTED;
    }
    if (x_first && !holds(first.out, x[m])) return CONSTSTN_EUNSUPPORTED;
    const bool mttkrp = facs[0].rank == facs[1].rank;
    // order of the two other levels in the copy: for TTMc the result lists the ranks in level order
    int a = facs[0].level < facs[1].level ? 0 : 1, b = 1 - a;
    if (mttkrp) {
        if (last.out.idx != std::vector<std::string>{x[m], facs[0].rank}) return CONSTSTN_EUNSUPPORTED;
        if (facs[0].extent != facs[1].extent) { set_error("batch index with two extents"); return CONSTSTN_ESCHED; }
    } else {
        if (last.out.idx.size() != 3 || last.out.idx[0] != x[m]) return CONSTSTN_EUNSUPPORTED;
        if (last.out.idx[1] == facs[b].rank && last.out.idx[2] == facs[a].rank) std::swap(a, b);
        else if (!(last.out.idx[1] == facs[a].rank && last.out.idx[2] == facs[b].rank)) return CONSTSTN_EUNSUPPORTED;
    }
    const int new_levels[3] = {m, facs[a].level, facs[b].level};
    std::unique_ptr<conststn_csf_s> copy(new (std::nothrow) conststn_csf_s());
    if (!copy) { set_error("host allocation failed"); return CONSTSTN_ENOMEM; }
    CST_TRY(reroot_csf3(s.operands[xop].csf, new_levels, copy.get()));
    plan->rerooted_x = std::move(copy);
    plan->rerooted_level = m;
    plan->X = plan->rerooted_x.get();
    plan->factor_of_level[1] = facs[a].ordinal;
    plan->rank_of_level[1] = facs[a].extent;
    plan->factor_of_level[2] = facs[b].ordinal;
    plan->rank_of_level[2] = facs[b].extent;
    plan->family = mttkrp ? FAM_MTTKRP3 : FAM_TTMC3;
    plan->row_elems = mttkrp ? facs[a].extent : int64_t(facs[a].extent) * facs[b].extent;
    return CONSTSTN_OK;
}

// rank extents the tuned kernels are built for
static bool tuned_kernel_fits(const conststn_plan_s *plan) {
    switch (plan->family) {
        case FAM_MTTKRP3: return plan->rank_of_level[1] <= 128;
        case FAM_TTMC3: return plan->rank_of_level[1] <= 64 && plan->rank_of_level[2] <= 64;
        case FAM_TTMC4: return plan->rank_of_level[1] <= 16 && plan->rank_of_level[2] <= 16 && plan->rank_of_level[3] <= 16;
        default: return true;
    }
}

static const char *family_name(Family f) {
    switch (f) {
        case FAM_TTMC3: return "ttmc3";
        case FAM_TTMC4: return "ttmc4";
        case FAM_MTTKRP3: return "mttkrp3";
        case FAM_SPTN3: return "sptn3";
        case FAM_GENERIC: return "generic";
        case FAM_SPCHAIN3: return "spchain3";
        case FAM_SPPAIR4: return "sppair4";
        default: return "none";
    }
}

}  // namespace cst

using namespace cst;

extern "C" {

const char *conststn_last_error(void) { return get_error(); }
const char *conststn_version(void) { return "conststn 0.1 (gfx950)"; }

conststn_status conststn_build_csf(int order, const int64_t *dims, int64_t nnz,
                                   const int32_t *const *coords, const double *vals,
                                   const int *mode_order, unsigned flags, conststn_stream stream,
                                   conststn_csf_t **out) {
    clear_error();
    if (!out) { set_error("out is null"); return CONSTSTN_EINVAL; }
    *out = nullptr;
    if (order < 1 || order > CONSTSTN_MAX_ORDER) { set_error("order %d outside 1..%d", order, CONSTSTN_MAX_ORDER); return CONSTSTN_EINVAL; }
    if (!dims || !mode_order || !coords) { set_error("null argument"); return CONSTSTN_EINVAL; }
    if (nnz < 0) { set_error("nnz is negative"); return CONSTSTN_EINVAL; }
    if (nnz >= (int64_t(1) << 31)) { set_error("nnz of 2^31 or more is not implemented"); return CONSTSTN_EUNSUPPORTED; }
    if (flags & ~CONSTSTN_COALESCE_DUPS) { set_error("unknown flag bits"); return CONSTSTN_EINVAL; }
    bool seen[CONSTSTN_MAX_ORDER] = {false};
    for (int l = 0; l < order; ++l) {
        if (dims[l] < 1 || dims[l] > 0x7fffffffll) { set_error("extent of mode %d outside 1..2^31-1", l); return CONSTSTN_EINVAL; }
        const int m = mode_order[l];
        if (m < 0 || m >= order || seen[m]) { set_error("mode_order is not a permutation of 0..%d", order - 1); return CONSTSTN_EINVAL; }
        seen[m] = true;
        if (nnz > 0 && !coords[l]) { set_error("coords[%d] is null", l); return CONSTSTN_EINVAL; }
    }
    if (nnz > 0 && !vals) { set_error("vals is null"); return CONSTSTN_EINVAL; }
    conststn_csf_s *csf = new (std::nothrow) conststn_csf_s();
    if (!csf) { set_error("host allocation failed"); return CONSTSTN_ENOMEM; }
    const conststn_status st = build_csf_device(order, dims, nnz, coords, vals, mode_order, flags,
                                                static_cast<hipStream_t>(stream), csf);
    if (st != CONSTSTN_OK) { delete csf; return st; }
    *out = csf;
    return CONSTSTN_OK;
}

conststn_status conststn_csf_info(const conststn_csf_t *csf, int *order, int64_t *dims, int *mode_order, int64_t *nnz) {
    clear_error();
    if (!csf) { set_error("csf is null"); return CONSTSTN_EINVAL; }
    if (order) *order = csf->order;
    if (nnz) *nnz = csf->nnz;
    for (int l = 0; l < csf->order; ++l) {
        if (dims) dims[l] = csf->dims[l];
        if (mode_order) mode_order[l] = csf->mode_order[l];
    }
    return CONSTSTN_OK;
}

conststn_status conststn_csf_export(const conststn_csf_t *csf, int level, const int32_t **idx,
                                    const int64_t **ptr, int64_t *nodes, const double **vals) {
    clear_error();
    if (!csf) { set_error("csf is null"); return CONSTSTN_EINVAL; }
    if (level < 0 || level >= csf->order) { set_error("level %d outside 0..%d", level, csf->order - 1); return CONSTSTN_EINVAL; }
    if (idx) *idx = csf->idx[level].p;
    if (ptr) *ptr = level < csf->order - 1 ? csf->ptr[level].p : nullptr;
    if (nodes) *nodes = csf->nodes[level];
    if (vals) *vals = level == csf->order - 1 ? csf->vals.p : nullptr;
    return CONSTSTN_OK;
}

void conststn_csf_destroy(conststn_csf_t *csf) { delete csf; }

conststn_status conststn_schedule_check(const char *schedule, const int *fusion, int n_operands,
                                        const conststn_operand_desc *operands, char *buf, size_t len,
                                        int *reduced_orders) {
    clear_error();
    Schedule s;
    CST_TRY(parse_schedule(schedule, s));
    CST_TRY(validate_schedule(s, fusion, n_operands, operands));
    if (buf && len > 0) {
        std::strncpy(buf, s.lowered.c_str(), len - 1);
        buf[len - 1] = 0;
    }
    if (reduced_orders)
        for (size_t p = 0; p < s.stmts.size(); ++p) reduced_orders[p] = s.stmts[p].reduced_order;
    return CONSTSTN_OK;
}

conststn_status conststn_schedule_search(const char *tree, int n_operands, const conststn_operand_desc *operands,
                                         unsigned flags, int max_order, char *buf, size_t len, int *order_found,
                                         int *level_modes) {
    clear_error();
    if (!tree) { set_error("tree is null"); return CONSTSTN_EINVAL; }
    if (flags & ~CONSTSTN_SEARCH_KEEP_LAYOUT) { set_error("unknown flag bits"); return CONSTSTN_EINVAL; }
    for (int o = 0; o < n_operands; ++o)
        if (operands[o].kind == CONSTSTN_OPERAND_CSF && operands[o].csf) {
            set_error("describe CSF operands by structure (csf = NULL, order, extents in the order of the reference)");
            return CONSTSTN_EINVAL;
        }
    Schedule found;
    std::vector<std::vector<int>> modes;
    int l = 0;
    CST_TRY(search_schedule(tree, n_operands, operands, (flags & CONSTSTN_SEARCH_KEEP_LAYOUT) != 0, max_order, found, &l, modes));
    const std::string text = schedule_text(found);
    // the result must pass the same checks as any schedule handed to conststn_plan
    std::vector<conststn_operand_desc> permuted(operands, operands + n_operands);
    for (int o = 0; o < n_operands; ++o)
        for (int d = 0; d < operands[o].order; ++d) permuted[size_t(o)].dims[d] = operands[o].dims[modes[size_t(o)][size_t(d)]];
    Schedule check;
    CST_TRY(parse_schedule(text.c_str(), check));
    conststn_status st = validate_schedule(check, nullptr, n_operands, permuted.data());
    if (st != CONSTSTN_OK) {
        std::string why = get_error();
        set_error("internal: the schedule found (%s) fails the legality check: %s", text.c_str(), why.c_str());
        return CONSTSTN_EINVAL;
    }
    for (size_t p = 0; p + 1 < check.stmts.size(); ++p)
        if (check.stmts[p].reduced_order > l) { set_error("internal: the schedule found leaves an intermediate of order %d > %d", check.stmts[p].reduced_order, l); return CONSTSTN_EINVAL; }
    if (buf && len > 0) {
        if (text.size() + 1 > len) { set_error("buffer of %zu bytes is too small for the schedule (%zu)", len, text.size() + 1); return CONSTSTN_EINVAL; }
        std::strncpy(buf, text.c_str(), len - 1);
        buf[len - 1] = 0;
    }
    if (order_found) *order_found = l;
    if (level_modes)
        for (int o = 0; o < n_operands; ++o)
            for (int d = 0; d < CONSTSTN_MAX_ORDER; ++d)
                level_modes[o * CONSTSTN_MAX_ORDER + d] = d < operands[o].order ? modes[size_t(o)][size_t(d)] : -1;
    return CONSTSTN_OK;
}

conststn_status conststn_plan(const char *schedule, const int *fusion, int n_operands,
                              const conststn_operand_desc *operands, unsigned flags,
                              conststn_plan_t **out) {
    return conststn_plan_options(schedule, fusion, n_operands, operands, flags, nullptr, out);
}

// Every plan option with the values it takes: a range, or (lo > hi) the listed values only.
struct PlanOptionRange { const char *name; int64_t lo, hi; int64_t listed[5]; };
static const PlanOptionRange kPlanOptions[] = {
    {"force_generic", 0, 1, {}},       {"generic_max_gb", 1, 4096, {}},   {"generic_span", 1, int64_t(1) << 30, {}},
    {"generic_fuse", 0, 1, {}},        {"generic_densify", 0, 1, {}},     {"reroot", 0, 1, {}},
    {"mttkrp_split", 0, 1, {}},        {"mttkrp_dual", 1, 0, {0, 35, 44, 53, 88}},
    {"mttkrp_hot", 1, int64_t(1) << 20, {}},                              {"mttkrp_chunk", 0, int64_t(1) << 24, {}},
    {"ttmc3_mfma", 0, 1, {}},          {"ttmc3_stream", 0, 1, {}},        {"ttmc3_producers", 1, 0, {2, 3, 4, 6, 8}},
    {"ttmc3_batch", 1, int64_t(1) << 30, {}},                             {"ttmc3_itemcost", 0, int64_t(1) << 20, {}},
    {"ttmc3_qn", 1, 0, {1, 2, 4, 4, 4}},
    {"ttmc3_split", 1, int64_t(1) << 40, {}},                             {"ttmc3_rowsplit", 1, int64_t(1) << 40, {}},
    {"ttmc4_mfma", 0, 1, {}},          {"ttmc4_split", 1, int64_t(1) << 40, {}},
    {"ttmc4_ksplit", 1, int64_t(1) << 40, {}},
    {"sptn3_tiled", 0, 2, {}},         {"sptn3_waves", 1, 2, {}},         {"sptn3_wgs", 1, int64_t(1) << 24, {}},
    {"sptn3_xcd", 0, 1, {}},
    {"spchain3_form", 1, 2, {}},       {"spchain3_order", 0, 1, {}},      {"spchain3_local_kb", 1, 160, {}},
    {"spchain3_pk_gb", 0, 4096, {}},
    {"sppair4_keep", 1, 2, {}},        {"sppair4_keep_gb", 0, 4096, {}},  {"sppair4_rows", 1, 2, {}},
    {"sppair4_rows_gb", 0, 4096, {}},  {"sppair4_buffers", 1, 2, {}},     {"sppair4_xcd", 0, 2, {}}};

// 0: no such option; 1: the value is one it takes; -1: it is not, and `takes` says which are
static int check_plan_option(const std::string &name, int64_t value, std::string &takes) {
    for (const PlanOptionRange &o : kPlanOptions) {
        if (name != o.name) continue;
        char b[96];
        if (o.lo <= o.hi) {
            if (value >= o.lo && value <= o.hi) return 1;
            snprintf(b, sizeof(b), "%lld to %lld", (long long)o.lo, (long long)o.hi);
            takes = b;
            return -1;
        }
        takes.clear();
        for (int k = 0; k < 5; ++k) {
            if (value == o.listed[k]) return 1;
            if (k > 0 && o.listed[k] == o.listed[k - 1]) continue;
            snprintf(b, sizeof(b), "%s%lld", k ? ", " : "", (long long)o.listed[k]);
            takes += b;
        }
        return -1;
    }
    return 0;
}

// "name=value,name=value" (spaces allowed around the separators) into the plan's option table
static conststn_status parse_plan_options(const char *text, conststn_plan_s *plan) {
    if (!text) return CONSTSTN_OK;
    std::string s(text), item;
    size_t pos = 0;
    while (pos <= s.size()) {
        const size_t end = std::min(s.find(',', pos), s.size());
        item = s.substr(pos, end - pos);
        pos = end + 1;
        item.erase(std::remove(item.begin(), item.end(), ' '), item.end());
        if (item.empty()) continue;
        const size_t eq = item.find('=');
        if (eq == std::string::npos || eq == 0 || eq + 1 == item.size()) { set_error("plan option '%s' is not of the form name=value", item.c_str()); return CONSTSTN_EINVAL; }
        const std::string name = item.substr(0, eq);
        char *stop = nullptr;
        const long long v = std::strtoll(item.c_str() + eq + 1, &stop, 10);
        if (!stop || *stop != 0 || v < 0) { set_error("plan option '%s': the value must be a non-negative integer", item.c_str()); return CONSTSTN_EINVAL; }
        std::string takes;
        const int known = check_plan_option(name, int64_t(v), takes);
        if (known == 0) { set_error("unknown plan option '%s'", name.c_str()); return CONSTSTN_EINVAL; }
        if (known < 0) { set_error("plan option '%s': %s takes %s", item.c_str(), name.c_str(), takes.c_str()); return CONSTSTN_EINVAL; }
        plan->options[name] = int64_t(v);
    }
    return CONSTSTN_OK;
}

conststn_status conststn_plan_options(const char *schedule, const int *fusion, int n_operands,
                                      const conststn_operand_desc *operands, unsigned flags,
                                      const char *options, conststn_plan_t **out) {
    clear_error();
    if (!out) { set_error("out is null"); return CONSTSTN_EINVAL; }
    *out = nullptr;
    if (flags & ~CONSTSTN_OUT_COMPACT) { set_error("unknown flag bits"); return CONSTSTN_EINVAL; }
    conststn_plan_s *plan = new (std::nothrow) conststn_plan_s();
    if (!plan) { set_error("host allocation failed"); return CONSTSTN_ENOMEM; }
    struct Guard { conststn_plan_s *p; ~Guard() { delete p; } } guard{plan};
    plan->flags = flags;
    plan->compact = (flags & CONSTSTN_OUT_COMPACT) != 0;
    CST_TRY(parse_plan_options(options, plan));
    {
        int dev = 0;
        CST_HIP(hipGetDevice(&dev));
        CST_HIP(hipDeviceGetAttribute(&plan->n_cus, hipDeviceAttributeMultiprocessorCount, dev));
        const int64_t qn = plan->opt("ttmc3_qn", 2);
        plan->ttmc3_qn = (qn == 1 || qn == 2 || qn == 4) ? int(qn) : 2;
    }
    CST_TRY(parse_schedule(schedule, plan->sched));
    CST_TRY(validate_schedule(plan->sched, fusion, n_operands, operands));
    for (const auto &o : plan->sched.operands)
        if (o.kind == CONSTSTN_OPERAND_CSF && !o.csf) { set_error("CSF operand %s has no handle", o.name.c_str()); return CONSTSTN_EINVAL; }
    for (const auto &o : plan->sched.operands) if (o.kind == CONSTSTN_OPERAND_DENSE) plan->n_dense++;

    clear_error();
    conststn_status st = match_chain(plan);
    if (st == CONSTSTN_EUNSUPPORTED && plan->family == FAM_NONE) {
        std::string why = get_error();
        clear_error();
        st = match_sptn3(plan);
        if (st == CONSTSTN_EUNSUPPORTED && !*get_error() && !why.empty()) set_error("%s", why.c_str());
    }
    if (st == CONSTSTN_EUNSUPPORTED && plan->family == FAM_NONE) {
        std::string why = get_error();
        clear_error();
        st = match_spchain3(plan);
        if (st == CONSTSTN_EUNSUPPORTED && !*get_error() && !why.empty()) set_error("%s", why.c_str());
    }
    if (st == CONSTSTN_EUNSUPPORTED && plan->family == FAM_NONE) {
        std::string why = get_error();
        clear_error();
        st = match_sppair4(plan);
        if (st == CONSTSTN_EUNSUPPORTED && !*get_error() && !why.empty()) set_error("%s", why.c_str());
    }
    if (st == CONSTSTN_EUNSUPPORTED && plan->family == FAM_NONE && plan->opt("reroot", 1) == 1) {
        std::string why = get_error();
        clear_error();
        st = match_rerooted(plan);
        if (st == CONSTSTN_EUNSUPPORTED && !*get_error() && !why.empty()) set_error("%s", why.c_str());
    }
    // tuned kernels have rank limits; beyond them, and for every other tree over one CSF operand,
    // the generic executor takes over
    if (st == CONSTSTN_OK && !tuned_kernel_fits(plan)) st = CONSTSTN_EUNSUPPORTED;
    if (st == CONSTSTN_OK && plan->opt("force_generic", 0) == 1 && plan->family != FAM_SPTN3 &&
        plan->family != FAM_SPCHAIN3 && plan->family != FAM_SPPAIR4)
        st = CONSTSTN_EUNSUPPORTED;
    if (st == CONSTSTN_EUNSUPPORTED) {
        std::string why = get_error();
        clear_error();
        plan->family = FAM_NONE;
        plan->rerooted_x.reset();
        plan->rerooted_level = -1;
        plan->X = nullptr;
        st = build_generic(plan);
        if (st == CONSTSTN_EUNSUPPORTED) {
            std::string why2 = get_error();
            set_error("the schedule is legal but no kernel takes it.  Tuned families (TTMc order 3/4, MTTKRP order 3, "
                      "(U.V).W): %s.  Generic executor: %s", why.empty() ? "no match" : why.c_str(),
                      why2.empty() ? "no match" : why2.c_str());
        }
    }
    CST_TRY(st);

    const conststn_csf_s *X = plan->X;
    plan->out_rows = plan->compact ? X->nodes[0] : X->dims[X->mode_order[0]];
    if (plan->family == FAM_GENERIC && !plan->gen_rooted) plan->out_rows = 1;    // fully contracted sparse modes
    switch (plan->family) {
        case FAM_MTTKRP3: CST_TRY(build_mttkrp3_tables(plan)); break;
        case FAM_TTMC3:
        case FAM_TTMC4: CST_TRY(build_ttmc_tables(plan)); break;
        case FAM_SPTN3: CST_TRY(build_sptn3_tables(plan)); break;
        case FAM_SPCHAIN3: CST_TRY(build_spchain3_tables(plan)); break;
        case FAM_SPPAIR4: CST_TRY(build_sppair4_tables(plan)); break;
        default: break;
    }
    char head[256];
    snprintf(head, sizeof(head), "family=%s rows=%lld row_elems=%lld compact=%d", family_name(plan->family),
             (long long)plan->out_rows, (long long)plan->row_elems, plan->compact ? 1 : 0);
    plan->description = head;
    if (plan->rerooted_level >= 0) {
        char b[96];
        snprintf(b, sizeof(b), " private copy of the tensor with level %d at the root", plan->rerooted_level);
        plan->description += b;
    }
    if (plan->family == FAM_SPTN3) {
        char b[96];
        if (plan->w_tiled)
            snprintf(b, sizeof(b), " kernel=tiled %s k chunks %d w tiles %lld", plan->sp_two_waves ? "two waves per SIMD" : "one wave per SIMD",
                     plan->sp_kc, (long long)plan->n_w_tiles);
        else
            snprintf(b, sizeof(b), " kernel=baseline");
        plan->description += b;
    }
    if (plan->family == FAM_TTMC3 && plan->use_rows) {
        char b[128];
        if (plan->use_stream)
            // mfma = matrix instructions one execute issues: K-steps x (R2/16) x (R3/16) tiles
            snprintf(b, sizeof(b), " kernel=stream producers %d batches %lld ksteps %lld mfma=%lld", plan->stream_producers,
                     (long long)plan->n_stream_wg, (long long)plan->n_ksteps,
                     (long long)(plan->n_ksteps * (plan->rank_of_level[1] / 16) * (plan->rank_of_level[2] / 16)));
        else
            snprintf(b, sizeof(b), " kernel=rows");
        plan->description += b;
    }
    if (plan->family == FAM_TTMC3 || plan->family == FAM_TTMC4) {
        char b[64];
        snprintf(b, sizeof(b), " partial_blocks=%lld", (long long)plan->n_partials);
        plan->description += b;
    }
    if (plan->family == FAM_GENERIC) {
        int fused = 0, pairs = 0;
        for (const GenStmt &g : plan->gen) { fused += g.skip; pairs += (g.fused && !g.skip && g.fused_pairs) ? 1 : 0; }
        char b[96];
        snprintf(b, sizeof(b), " kernels=%d inlined_producers=%d", int(plan->gen.size()) - fused, fused);
        plan->description += b;
        snprintf(b, sizeof(b), " two_elements_per_lane=%d", pairs);
        plan->description += b;
        if (!plan->gen_densified.empty()) {
            snprintf(b, sizeof(b), " dense_copies_of_csf_operands=%d", int(plan->gen_densified.size()));
            plan->description += b;
        }
    }
    if (plan->family == FAM_SPCHAIN3) {
        char b[96];
        if (plan->sc_local)
            snprintf(b, sizeof(b), " kernel=block-local lds %d P blocks %.1f MB", plan->sc_local_lds, double(plan->sc_pk_doubles) * 8e-6);
        else snprintf(b, sizeof(b), " kernel=general lds %d", plan->sc_lds_bytes);
        plan->description += b;
    }
    if (plan->family == FAM_SPPAIR4) {
        char b[96];
        snprintf(b, sizeof(b), " kernel=%s lds %d", plan->p4_dense ? "dense rows" : plan->p4_stored ? "leaf lists kept" : "nothing kept",
                 plan->p4_layout.empty() ? 0 : plan->p4_layout.back());
        plan->description += b;
    }
    for (size_t p = 0; p + 1 < plan->sched.stmts.size(); ++p) {
        char b[128];
        snprintf(b, sizeof(b), " %s:order%d", plan->sched.stmts[p].out.name.c_str(), plan->sched.stmts[p].reduced_order);
        plan->description += b;
    }
    plan->description += " | " + plan->sched.lowered;
    guard.p = nullptr;
    *out = plan;
    return CONSTSTN_OK;
}

conststn_status conststn_plan_output_size(const conststn_plan_t *plan, int64_t *n_rows, int64_t *row_elems) {
    clear_error();
    if (!plan) { set_error("plan is null"); return CONSTSTN_EINVAL; }
    if (n_rows) *n_rows = plan->out_rows;
    if (row_elems) *row_elems = plan->row_elems;
    return CONSTSTN_OK;
}

conststn_status conststn_plan_output_rows(const conststn_plan_t *plan, const int32_t **rows, int64_t *n_rows) {
    clear_error();
    if (!plan) { set_error("plan is null"); return CONSTSTN_EINVAL; }
    if (!plan->compact) { set_error("the plan's output is not compact"); return CONSTSTN_EINVAL; }
    if (rows) *rows = plan->X->idx[0].p;
    if (n_rows) *n_rows = plan->X->nodes[0];
    return CONSTSTN_OK;
}

conststn_status conststn_plan_output_csf(const conststn_plan_t *plan, const conststn_csf_t **structure) {
    clear_error();
    if (!plan || !structure) { set_error("null argument"); return CONSTSTN_EINVAL; }
    if (!plan->sc_E) { set_error("the plan's result is dense"); return CONSTSTN_EINVAL; }
    *structure = plan->sc_E.get();
    return CONSTSTN_OK;
}

conststn_status conststn_plan_describe(const conststn_plan_t *plan, char *buf, size_t len) {
    clear_error();
    if (!plan || !buf || len == 0) { set_error("null argument"); return CONSTSTN_EINVAL; }
    std::strncpy(buf, plan->description.c_str(), len - 1);
    buf[len - 1] = 0;
    return CONSTSTN_OK;
}

void conststn_plan_destroy(conststn_plan_t *plan) { delete plan; }

conststn_status conststn_plan_profile(conststn_plan_t *plan, int capacity) {
    clear_error();
    if (!plan || capacity < 0 || capacity > 4096) { set_error("bad argument"); return CONSTSTN_EINVAL; }
    for (hipEvent_t e : plan->prof_start) (void)hipEventDestroy(e);
    for (hipEvent_t e : plan->prof_stop) (void)hipEventDestroy(e);
    plan->prof_start.clear();
    plan->prof_stop.clear();
    plan->prof_count = 0;
    for (int i = 0; i < capacity; ++i) {
        hipEvent_t a, b;
        CST_HIP(hipEventCreate(&a));
        plan->prof_start.push_back(a);
        CST_HIP(hipEventCreate(&b));
        plan->prof_stop.push_back(b);
    }
    return CONSTSTN_OK;
}

conststn_status conststn_plan_kernel_times(conststn_plan_t *plan, float *ms, int max_n, int *n) {
    clear_error();
    if (!plan || !n || (max_n > 0 && !ms)) { set_error("null argument"); return CONSTSTN_EINVAL; }
    const int64_t cap = int64_t(plan->prof_start.size());
    const int64_t have = std::min<int64_t>(plan->prof_count, cap);
    const int64_t first = plan->prof_count - have;
    int written = 0;
    for (int64_t i = first; i < plan->prof_count && written < max_n; ++i) {
        const int slot = int(i % cap);
        CST_HIP(hipEventSynchronize(plan->prof_stop[slot]));
        CST_HIP(hipEventElapsedTime(&ms[written], plan->prof_start[slot], plan->prof_stop[slot]));
        ++written;
    }
    *n = written;
    plan->prof_count = 0;
    return CONSTSTN_OK;
}

conststn_status conststn_execute(const conststn_plan_t *plan, const double *const *dense_factors,
                                 double *out, conststn_stream stream) {
    clear_error();
    if (!plan) { set_error("plan is null"); return CONSTSTN_EINVAL; }
    if (!out && plan->out_rows * plan->row_elems > 0) { set_error("out is null"); return CONSTSTN_EINVAL; }
    if (plan->n_dense > 0 && !dense_factors) { set_error("dense_factors is null"); return CONSTSTN_EINVAL; }
    for (int d = 0; d < plan->n_dense; ++d)
        if (!dense_factors[d]) { set_error("dense_factors[%d] is null", d); return CONSTSTN_EINVAL; }
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (plan->family) {
        case FAM_MTTKRP3: return launch_mttkrp3(plan, dense_factors, out, st);
        case FAM_TTMC3: return launch_ttmc3(plan, dense_factors, out, st);
        case FAM_TTMC4: return launch_ttmc4(plan, dense_factors, out, st);
        case FAM_SPTN3: return launch_sptn3(plan, dense_factors, out, st);
        case FAM_SPCHAIN3: return launch_spchain3(plan, out, st);
        case FAM_SPPAIR4: return launch_sppair4(plan, out, st);
        case FAM_GENERIC: return launch_generic(plan, dense_factors, out, st);
        default: set_error("plan has no kernel family"); return CONSTSTN_EINVAL;
    }
}

conststn_status conststn_execute_static(const conststn_plan_t *plan, const double *const *dense_factors,
                                        double *out, conststn_stream stream) {
    clear_error();
    if (!plan) { set_error("plan is null"); return CONSTSTN_EINVAL; }
    if (plan->family != FAM_TTMC3) {
        set_error("conststn_execute_static takes plans of the order-3 TTMc kernels only (this one is %s)", family_name(plan->family));
        return CONSTSTN_EUNSUPPORTED;
    }
    if (!out && plan->out_rows * plan->row_elems > 0) { set_error("out is null"); return CONSTSTN_EINVAL; }
    if (!dense_factors) { set_error("dense_factors is null"); return CONSTSTN_EINVAL; }
    for (int d = 0; d < plan->n_dense; ++d)
        if (!dense_factors[d]) { set_error("dense_factors[%d] is null", d); return CONSTSTN_EINVAL; }
    return launch_ttmc3_static(plan, dense_factors, out, static_cast<hipStream_t>(stream));
}

}  // extern "C"
