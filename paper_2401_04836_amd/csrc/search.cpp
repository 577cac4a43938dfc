// Schedule search (host only): the question of Sec. 3 -- for a given contraction tree, is there
// an order of the assignments, a loop order per assignment and a level order per sparse tensor
// such that every intermediate has order at most l after fusion? -- asked for l = 1, 2, ...
// until the answer is yes.  The paper hands the constraints of Sec. 3.2 to an SMT solver; trees
// of a few contractions are small enough to enumerate, so this file walks the space directly:
//
//   ap   every topological order of the tree's statements ("Ordering of assignments"),
//   lp   for each statement, in that order, every permutation of its indices ("Ordering of loops"),
//        cut as soon as a constraint that only involves statements already placed fails,
//   dp   the level order of a sparse tensor is read off the loop order of the one statement that
//        references it ("Consistency between mode order and loop order" then holds by
//        construction); a tensor whose layout the caller fixes instead constrains that loop order.
//
// For producer q with result order n and consumer c the constraints are those of "Producer-consumer
// pairs": the outermost n - l loops of q are indices of its result, c has the same loops in the
// same positions, and so has every statement placed between the two.
//
// Among the solutions for the smallest l the search prefers fewer statements whose summed index is
// the innermost loop (a summed innermost loop makes the intermediate a scalar and every sparse
// operand below it an intersection), then smaller intermediates (sum of the orders after taking the
// longest legal fused prefix), then the first one found; the walk stops after a bounded number of
// complete solutions, so the preference is over those seen.
#include <algorithm>
#include <set>

#include "schedule.hpp"

namespace cst {

namespace {

struct Node {
    std::vector<std::string> all;                         // indices of the statement, sorted
    std::vector<std::pair<std::string, std::string>> before;   // fixed layouts: first must be outside second
    std::vector<int> children;                            // producers consumed here
    int parent = -1;
    int out_order = 0;
};

int pos_of(const std::vector<std::string> &v, const std::string &x) {
    auto it = std::find(v.begin(), v.end(), x);
    return it == v.end() ? -1 : int(it - v.begin());
}

bool has(const std::vector<std::string> &v, const std::string &x) { return pos_of(v, x) >= 0; }

struct Walk {
    const Schedule &s;
    const std::vector<Node> &nodes;
    int m, l;
    std::vector<int> order, place;                        // order[k] = statement at position k; place = inverse
    std::vector<std::vector<std::string>> loops;          // per statement
    std::vector<int> need;                                // per statement: loops it must share with its consumer
    // best so far
    bool found = false;
    long score[2] = {0, 0};
    std::vector<int> best_order;
    std::vector<std::vector<std::string>> best_loops;
    long leaves = 0, leaf_cap = 20000;

    Walk(const Schedule &sched, const std::vector<Node> &n, int l_) : s(sched), nodes(n), m(int(n.size())), l(l_) {
        loops.resize(size_t(m));
        need.assign(size_t(m), 0);
        for (int p = 0; p < m; ++p)
            if (nodes[size_t(p)].parent >= 0) need[size_t(p)] = std::max(0, nodes[size_t(p)].out_order - l);
    }

    // constraints that involve statement st (placed at position k) and statements placed before it
    bool admissible(int st, int k) const {
        const Node &nd = nodes[size_t(st)];
        const auto &lp = loops[size_t(st)];
        for (const auto &pr : nd.before)
            if (pos_of(lp, pr.first) > pos_of(lp, pr.second)) return false;
        const auto &out = s.stmts[size_t(st)].out.idx;
        for (int d = 0; d < need[size_t(st)]; ++d)
            if (d >= int(lp.size()) || !has(out, lp[size_t(d)])) return false;          // producer constraints
        for (int q = 0; q < m; ++q) {
            if (q == st || place[size_t(q)] < 0 || place[size_t(q)] >= k) continue;     // placed earlier only
            const int c = nodes[size_t(q)].parent;
            if (c < 0) continue;
            const bool is_consumer = c == st;
            const bool between = !is_consumer && (place[size_t(c)] < 0 || place[size_t(c)] > k);
            if (!is_consumer && !between) continue;
            const auto &lq = loops[size_t(q)];
            for (int d = 0; d < need[size_t(q)]; ++d)
                if (d >= int(lp.size()) || lp[size_t(d)] != lq[size_t(d)]) return false;  // consumer / in-between
        }
        return true;
    }

    // longest legal fused prefix of producer p in the complete assignment
    int fused_depth(int p) const {
        const int c = nodes[size_t(p)].parent;
        const auto &lp = loops[size_t(p)], &lc = loops[size_t(c)];
        const auto &out = s.stmts[size_t(p)].out.idx;
        int d = 0;
        for (;; ++d) {
            if (d >= int(lp.size()) || d >= int(lc.size()) || !has(out, lp[size_t(d)]) || lc[size_t(d)] != lp[size_t(d)]) break;
            bool ok = true;
            for (int k = place[size_t(p)] + 1; k < place[size_t(c)] && ok; ++k) {
                const auto &lr = loops[size_t(order[size_t(k)])];
                ok = d < int(lr.size()) && lr[size_t(d)] == lp[size_t(d)];
            }
            if (!ok) break;
        }
        return d;
    }

    void leaf() {
        ++leaves;
        long sum = 0, inner = 0;
        for (int p = 0; p < m; ++p) {
            if (nodes[size_t(p)].parent >= 0) sum += nodes[size_t(p)].out_order - fused_depth(p);
            const Stmt &st = s.stmts[size_t(p)];
            if (!loops[size_t(p)].empty() && !has(st.out.idx, loops[size_t(p)].back())) ++inner;   // a summed index innermost
        }
        if (!found || inner < score[0] || (inner == score[0] && sum < score[1])) {
            found = true;
            score[0] = inner;
            score[1] = sum;
            best_order = order;
            best_loops = loops;
        }
    }

    void place_from(int k) {
        if (leaves >= leaf_cap) return;
        if (k == m) { leaf(); return; }
        const int st = order[size_t(k)];
        std::vector<std::string> perm = nodes[size_t(st)].all;
        do {
            loops[size_t(st)] = perm;
            if (admissible(st, k)) place_from(k + 1);
            if (leaves >= leaf_cap) return;
        } while (std::next_permutation(perm.begin(), perm.end()));
    }

    // every topological order: statement placed after all of its children
    void orders_from(int k) {
        if (leaves >= leaf_cap) return;
        if (k == m) {
            place_from(0);
            return;
        }
        for (int st = 0; st < m; ++st) {
            if (place[size_t(st)] >= 0) continue;
            bool ready = true;
            for (int ch : nodes[size_t(st)].children) ready = ready && place[size_t(ch)] >= 0;
            if (!ready) continue;
            place[size_t(st)] = k;
            order[size_t(k)] = st;
            orders_from(k + 1);
            place[size_t(st)] = -1;
        }
    }

    void run() {
        order.assign(size_t(m), -1);
        place.assign(size_t(m), -1);
        orders_from(0);
    }
};

}  // namespace

conststn_status search_schedule(const char *tree, int n_operands, const conststn_operand_desc *ops, bool keep_layout,
                                int max_order, Schedule &result, int *order_found,
                                std::vector<std::vector<int>> &level_modes) {
    Schedule s;
    CST_TRY(parse_schedule(tree, s));
    const int m = int(s.stmts.size());
    if (m > 6) { set_error("the search enumerates trees of at most 6 contractions; this one has %d", m); return CONSTSTN_EUNSUPPORTED; }
    if (n_operands < 0 || (n_operands > 0 && !ops)) { set_error("bad operand list"); return CONSTSTN_EINVAL; }
    auto find_operand = [&](const std::string &n) {
        for (int o = 0; o < n_operands; ++o) if (ops[o].name && n == ops[o].name) return o;
        return -1;
    };
    auto find_stmt = [&](const std::string &n) {
        for (int q = 0; q < m; ++q) if (s.stmts[size_t(q)].out.name == n) return q;
        return -1;
    };
    std::vector<Node> nodes(static_cast<size_t>(m));
    std::vector<int> uses(static_cast<size_t>(std::max(n_operands, 1)), 0);
    std::map<std::string, int64_t> extent;
    for (int p = 0; p < m; ++p) {
        Stmt &st = s.stmts[size_t(p)];
        if (!st.loops.empty()) { set_error("statement %d already has a loop order; the search chooses them", p); return CONSTSTN_EINVAL; }
        Node &nd = nodes[size_t(p)];
        std::set<std::string> all(st.a.idx.begin(), st.a.idx.end());
        all.insert(st.b.idx.begin(), st.b.idx.end());
        if (all.size() > 8) { set_error("statement %d has %zu indices; the search enumerates at most 8", p, all.size()); return CONSTSTN_EUNSUPPORTED; }
        for (const auto &x : st.out.idx)
            if (!all.count(x)) { set_error("statement %d: output index %s appears in no input", p, x.c_str()); return CONSTSTN_EINVAL; }
        nd.all.assign(all.begin(), all.end());
        nd.out_order = int(st.out.idx.size());
        for (const Ref *r : {&st.a, &st.b}) {
            std::set<std::string> seen(r->idx.begin(), r->idx.end());
            if (seen.size() != r->idx.size()) { set_error("statement %d repeats an index inside a reference", p); return CONSTSTN_EINVAL; }
            const int o = find_operand(r->name);
            if (o >= 0) {
                if (++uses[size_t(o)] > 1) { set_error("operand %s is referenced twice; the search takes trees whose leaves are distinct tensors", r->name.c_str()); return CONSTSTN_EUNSUPPORTED; }
                if (int(r->idx.size()) != ops[o].order) { set_error("statement %d: %s has %zu indices, the operand has order %d", p, r->name.c_str(), r->idx.size(), ops[o].order); return CONSTSTN_EINVAL; }
                for (size_t d = 0; d < r->idx.size(); ++d) {
                    auto it = extent.find(r->idx[d]);
                    if (it != extent.end() && it->second != ops[o].dims[d]) { set_error("index %s has two extents", r->idx[d].c_str()); return CONSTSTN_ESCHED; }
                    extent[r->idx[d]] = ops[o].dims[d];
                }
                if (ops[o].kind == CONSTSTN_OPERAND_CSF && keep_layout)
                    for (size_t d = 0; d + 1 < r->idx.size(); ++d) nd.before.emplace_back(r->idx[d], r->idx[d + 1]);
                continue;
            }
            const int q = find_stmt(r->name);
            if (q < 0 || q == p) { set_error("statement %d uses unknown tensor %s", p, r->name.c_str()); return CONSTSTN_EINVAL; }
            if (nodes[size_t(q)].parent >= 0) { set_error("intermediate %s is consumed twice: the contractions do not form a tree", r->name.c_str()); return CONSTSTN_ESCHED; }
            std::set<std::string> pi(s.stmts[size_t(q)].out.idx.begin(), s.stmts[size_t(q)].out.idx.end());
            if (pi != seen) { set_error("statement %d refers to %s with indices that differ from its producer's", p, r->name.c_str()); return CONSTSTN_EINVAL; }
            nodes[size_t(q)].parent = p;
            nd.children.push_back(q);
        }
    }
    int roots = 0, lmax = 1;
    for (int p = 0; p < m; ++p) {
        if (nodes[size_t(p)].parent < 0) ++roots;
        else lmax = std::max(lmax, nodes[size_t(p)].out_order);
    }
    if (roots != 1) { set_error("%d statements are never consumed: the contractions do not form a tree", roots); return CONSTSTN_ESCHED; }
    if (max_order > 0) lmax = std::min(lmax, max_order);

    for (int l = 1; l <= lmax; ++l) {
        Walk w(s, nodes, l);
        w.run();
        if (!w.found) continue;
        // assemble: statements in the chosen order, sparse references rewritten in level order
        result = Schedule();
        level_modes.assign(size_t(n_operands), std::vector<int>());
        for (int k = 0; k < m; ++k) {
            const int p = w.best_order[size_t(k)];
            Stmt st = s.stmts[size_t(p)];
            st.loops = w.best_loops[size_t(p)];
            for (Ref *r : {&st.a, &st.b}) {
                const int o = find_operand(r->name);
                if (o < 0) continue;
                std::vector<int> perm(r->idx.size());
                for (size_t d = 0; d < perm.size(); ++d) perm[d] = int(d);
                if (ops[o].kind == CONSTSTN_OPERAND_CSF && !keep_layout)
                    std::stable_sort(perm.begin(), perm.end(), [&](int x, int y) {
                        return pos_of(st.loops, r->idx[size_t(x)]) < pos_of(st.loops, r->idx[size_t(y)]);
                    });
                std::vector<std::string> idx;
                for (int d : perm) idx.push_back(r->idx[size_t(d)]);
                r->idx = idx;
                level_modes[size_t(o)] = perm;
            }
            result.stmts.push_back(st);
        }
        for (int o = 0; o < n_operands; ++o)
            if (level_modes[size_t(o)].empty()) {
                level_modes[size_t(o)].resize(size_t(ops[o].order));
                for (int d = 0; d < ops[o].order; ++d) level_modes[size_t(o)][size_t(d)] = d;
            }
        if (order_found) *order_found = l;
        return CONSTSTN_OK;
    }
    set_error("no schedule with intermediates of order <= %d satisfies the layouts that were fixed", lmax);
    return CONSTSTN_ESCHED;
}

std::string schedule_text(const Schedule &s) {
    std::string t;
    auto ref = [](const Ref &r) {
        std::string x = r.name + "[";
        for (size_t i = 0; i < r.idx.size(); ++i) x += (i ? "," : "") + r.idx[i];
        return x + "]";
    };
    for (size_t p = 0; p < s.stmts.size(); ++p) {
        const Stmt &st = s.stmts[p];
        if (p) t += " ; ";
        t += ref(st.out) + " = " + ref(st.a) + " * " + ref(st.b) + " | ";
        for (size_t i = 0; i < st.loops.size(); ++i) t += (i ? "," : "") + st.loops[i];
    }
    return t;
}

}  // namespace cst
