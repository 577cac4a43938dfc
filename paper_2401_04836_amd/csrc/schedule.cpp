// Parsing, legality checking and lowering of schedules (host only).
//
// A schedule is the paper's sequence S of pairs <A, pi> in execution order (Sec. 4.2): A is
// the assignment of one binary contraction, pi the order of its surrounding loops.  The
// checks are the constraints of Sec. 3.2 evaluated on a GIVEN solution instead of being
// handed to a solver: assignment order is a topological order of the tree, every pi is a
// permutation, CSF level order implies loop order, and producer / consumer / in-between
// statements share the fused loop prefix.
#include "schedule.hpp"

#include <algorithm>
#include <cctype>
#include <set>

namespace cst {

// ---- parsing -----------------------------------------------------------------------------

namespace {

struct Cursor {
    const char *s;
    size_t i = 0;
    void skip() { while (s[i] && std::isspace(static_cast<unsigned char>(s[i]))) ++i; }
    bool eat(char c) { skip(); if (s[i] == c) { ++i; return true; } return false; }
    bool ident(std::string &out) {
        skip();
        size_t b = i;
        while (s[i] && (std::isalnum(static_cast<unsigned char>(s[i])) || s[i] == '_')) ++i;
        if (i == b) return false;
        out.assign(s + b, i - b);
        return true;
    }
    bool at_end() { skip(); return s[i] == 0; }
};

bool parse_ref(Cursor &c, Ref &r) {
    if (!c.ident(r.name)) return false;
    if (!c.eat('[')) return false;
    r.idx.clear();
    if (c.eat(']')) return true;               // order-0 reference
    for (;;) {
        std::string id;
        if (!c.ident(id)) return false;
        r.idx.push_back(id);
        if (c.eat(']')) return true;
        if (!c.eat(',')) return false;
    }
}

std::string ref_text(const Ref &r, char open, char close) {
    std::string t = r.name;
    t.push_back(open);
    for (size_t i = 0; i < r.idx.size(); ++i) {
        if (i) t += ", ";
        t += r.idx[i];
    }
    t.push_back(close);
    return t;
}

bool contains(const std::vector<std::string> &v, const std::string &x) {
    return std::find(v.begin(), v.end(), x) != v.end();
}

int position(const std::vector<std::string> &v, const std::string &x) {
    auto it = std::find(v.begin(), v.end(), x);
    return it == v.end() ? -1 : int(it - v.begin());
}

}  // namespace

conststn_status parse_schedule(const char *text, Schedule &sched) {
    if (!text) { set_error("schedule text is null"); return CONSTSTN_EINVAL; }
    Cursor c{text};
    sched.stmts.clear();
    while (!c.at_end()) {
        Stmt st;
        if (!parse_ref(c, st.out) || !c.eat('=') || !parse_ref(c, st.a) || !c.eat('*') || !parse_ref(c, st.b)) {
            set_error("malformed statement %zu near offset %zu: expected OUT[..] = A[..] * B[..] | loops",
                      sched.stmts.size(), c.i);
            return CONSTSTN_EINVAL;
        }
        // the loop order may be left out (a contraction tree handed to the schedule search)
        if (c.eat('|'))
            for (;;) {
                std::string id;
                if (!c.ident(id)) {
                    if (st.loops.empty() && (c.at_end() || text[c.i] == ';')) break;   // no loops
                    set_error("malformed loop order in statement %zu", sched.stmts.size());
                    return CONSTSTN_EINVAL;
                }
                st.loops.push_back(id);
                if (!c.eat(',')) break;
            }
        sched.stmts.push_back(st);
        if (!c.eat(';')) break;
    }
    if (!c.at_end()) {
        set_error("unexpected text after statement %zu at offset %zu", sched.stmts.size() - 1, c.i);
        return CONSTSTN_EINVAL;
    }
    if (sched.stmts.empty()) { set_error("schedule has no statement"); return CONSTSTN_EINVAL; }
    return CONSTSTN_OK;
}

// ---- validation ----------------------------------------------------------------------------

static conststn_status set_extent(Schedule &s, const std::string &idx, int64_t n, const char *where) {
    auto it = s.extent.find(idx);
    if (it == s.extent.end()) { s.extent[idx] = n; return CONSTSTN_OK; }
    if (it->second != n) {
        set_error("index %s has extent %lld in %s but %lld elsewhere", idx.c_str(), (long long)n,
                  where, (long long)it->second);
        return CONSTSTN_ESCHED;
    }
    return CONSTSTN_OK;
}

conststn_status validate_schedule(Schedule &s, const int *fusion, int n_operands,
                                  const conststn_operand_desc *ops) {
    if (n_operands < 0 || (n_operands > 0 && !ops)) { set_error("bad operand list"); return CONSTSTN_EINVAL; }
    s.operands.clear();
    s.extent.clear();
    int dense_count = 0;
    for (int o = 0; o < n_operands; ++o) {
        OperandInfo oi;
        if (!ops[o].name) { set_error("operand %d has no name", o); return CONSTSTN_EINVAL; }
        oi.name = ops[o].name;
        for (const auto &prev : s.operands)
            if (prev.name == oi.name) { set_error("operand %s listed twice", oi.name.c_str()); return CONSTSTN_EINVAL; }
        oi.kind = ops[o].kind;
        if (oi.kind == CONSTSTN_OPERAND_CSF) {
            oi.csf = ops[o].csf;
            if (oi.csf) {
                oi.order = oi.csf->order;
                for (int l = 0; l < oi.order; ++l) oi.dims[l] = oi.csf->dims[oi.csf->mode_order[l]];
            } else {                      // structure-only description: extents in level order
                oi.order = ops[o].order;
                if (oi.order < 1 || oi.order > CONSTSTN_MAX_ORDER) { set_error("operand %s: bad order", oi.name.c_str()); return CONSTSTN_EINVAL; }
                for (int l = 0; l < oi.order; ++l) oi.dims[l] = ops[o].dims[l];
            }
        } else if (oi.kind == CONSTSTN_OPERAND_DENSE) {
            oi.order = ops[o].order;
            if (oi.order < 0 || oi.order > CONSTSTN_MAX_ORDER) { set_error("operand %s: bad order", oi.name.c_str()); return CONSTSTN_EINVAL; }
            for (int l = 0; l < oi.order; ++l) oi.dims[l] = ops[o].dims[l];
            oi.dense_ordinal = dense_count++;
        } else {
            set_error("operand %s: unknown kind %d", oi.name.c_str(), oi.kind);
            return CONSTSTN_EINVAL;
        }
        for (int l = 0; l < oi.order; ++l)
            if (oi.dims[l] < 1) { set_error("operand %s: extent %d is not positive", oi.name.c_str(), l); return CONSTSTN_EINVAL; }
        s.operands.push_back(oi);
    }

    const int m = int(s.stmts.size());
    auto find_operand = [&](const std::string &n) {
        for (size_t o = 0; o < s.operands.size(); ++o) if (s.operands[o].name == n) return int(o);
        return -1;
    };
    auto find_stmt = [&](const std::string &n) {
        for (int q = 0; q < m; ++q) if (s.stmts[q].out.name == n) return q;
        return -1;
    };

    // names, distinct indices inside a reference
    for (int p = 0; p < m; ++p) {
        Stmt &st = s.stmts[p];
        for (const Ref *r : {&st.out, &st.a, &st.b}) {
            std::set<std::string> seen(r->idx.begin(), r->idx.end());
            if (seen.size() != r->idx.size()) {
                set_error("statement %d: reference %s repeats an index", p, ref_text(*r, '[', ']').c_str());
                return CONSTSTN_EINVAL;
            }
        }
        if (find_operand(st.out.name) >= 0) { set_error("statement %d assigns to input operand %s", p, st.out.name.c_str()); return CONSTSTN_EINVAL; }
        for (int q = 0; q < p; ++q)
            if (s.stmts[q].out.name == st.out.name) { set_error("tensor %s is assigned twice", st.out.name.c_str()); return CONSTSTN_EINVAL; }
    }

    // producers and consumers: the assignment order must be a topological order of a tree
    for (int p = 0; p < m; ++p) {
        Stmt &st = s.stmts[p];
        int *srcs[2] = {&st.src_a, &st.src_b};
        int *opsn[2] = {&st.op_a, &st.op_b};
        const Ref *refs[2] = {&st.a, &st.b};
        for (int t = 0; t < 2; ++t) {
            const Ref &r = *refs[t];
            *srcs[t] = -1;
            *opsn[t] = find_operand(r.name);
            if (*opsn[t] >= 0) {
                const OperandInfo &oi = s.operands[*opsn[t]];
                if (int(r.idx.size()) != oi.order) {
                    set_error("statement %d: %s has %zu indices but operand order is %d", p,
                              ref_text(r, '[', ']').c_str(), r.idx.size(), oi.order);
                    return CONSTSTN_EINVAL;
                }
                for (int l = 0; l < oi.order; ++l) CST_TRY(set_extent(s, r.idx[l], oi.dims[l], r.name.c_str()));
                continue;
            }
            const int q = find_stmt(r.name);
            if (q < 0) { set_error("statement %d uses unknown tensor %s", p, r.name.c_str()); return CONSTSTN_EINVAL; }
            if (q >= p) {
                set_error("statement %d consumes %s before statement %d produces it: the assignment "
                          "order is not a topological order of the contraction tree", p, r.name.c_str(), q);
                return CONSTSTN_ESCHED;
            }
            if (s.stmts[q].consumer >= 0) {
                set_error("intermediate %s is consumed twice: the contractions do not form a tree", r.name.c_str());
                return CONSTSTN_ESCHED;
            }
            std::set<std::string> pi(s.stmts[q].out.idx.begin(), s.stmts[q].out.idx.end());
            std::set<std::string> ci(r.idx.begin(), r.idx.end());
            if (pi != ci) {
                set_error("statement %d refers to %s with indices that differ from its producer's", p, r.name.c_str());
                return CONSTSTN_EINVAL;
            }
            s.stmts[q].consumer = p;
            *srcs[t] = q;
        }
    }
    for (int p = 0; p + 1 < m; ++p)
        if (s.stmts[p].consumer < 0) {
            set_error("result of statement %d (%s) is never consumed: the contractions do not form a tree",
                      p, s.stmts[p].out.name.c_str());
            return CONSTSTN_ESCHED;
        }

    // loop orders are permutations of the statement's indices; external indices come from the inputs
    for (int p = 0; p < m; ++p) {
        Stmt &st = s.stmts[p];
        std::set<std::string> all(st.a.idx.begin(), st.a.idx.end());
        all.insert(st.b.idx.begin(), st.b.idx.end());
        for (const auto &x : st.out.idx)
            if (!all.count(x)) { set_error("statement %d: output index %s appears in no input", p, x.c_str()); return CONSTSTN_EINVAL; }
        std::set<std::string> lp(st.loops.begin(), st.loops.end());
        if (lp.size() != st.loops.size() || lp != all) {
            set_error("statement %d: the loop order is not a permutation of the statement's indices", p);
            return CONSTSTN_ESCHED;
        }
        for (const auto &x : all)
            if (!s.extent.count(x)) { set_error("statement %d: extent of index %s is unknown", p, x.c_str()); return CONSTSTN_EINVAL; }
    }

    // CSF level order implies loop order (dense operands and workspace intermediates are exempt)
    for (int p = 0; p < m; ++p) {
        Stmt &st = s.stmts[p];
        const Ref *refs[2] = {&st.a, &st.b};
        const int opsn[2] = {st.op_a, st.op_b};
        for (int t = 0; t < 2; ++t) {
            if (opsn[t] < 0 || s.operands[opsn[t]].kind != CONSTSTN_OPERAND_CSF) continue;
            const Ref &r = *refs[t];
            for (size_t l = 0; l + 1 < r.idx.size(); ++l)
                if (position(st.loops, r.idx[l]) > position(st.loops, r.idx[l + 1])) {
                    set_error("statement %d: loop %s is outside loop %s but CSF operand %s stores %s above %s "
                              "(mode order and loop order are inconsistent)", p, r.idx[l + 1].c_str(),
                              r.idx[l].c_str(), r.name.c_str(), r.idx[l].c_str(), r.idx[l + 1].c_str());
                    return CONSTSTN_ESCHED;
                }
        }
    }

    // producer / consumer / in-between prefix rules and fusion depths
    for (int p = 0; p < m; ++p) {
        Stmt &st = s.stmts[p];
        st.fused_depth = 0;
        st.reduced_order = int(st.out.idx.size());
        if (st.consumer < 0) continue;
        const Stmt &co = s.stmts[st.consumer];
        const int want = fusion ? fusion[p] : -1;
        if (want < -1) { set_error("fusion[%d] = %d is invalid", p, want); return CONSTSTN_EINVAL; }
        const int limit = want < 0 ? int(st.loops.size()) : want;
        int d = 0;
        for (; d < limit; ++d) {
            const char *why = nullptr;
            int who = -1;
            if (d >= int(st.loops.size()) || !contains(st.out.idx, st.loops[d])) {
                why = "producer rule: an outermost fused loop of the producer is not an index of its result";
            } else if (d >= int(co.loops.size()) || co.loops[d] != st.loops[d]) {
                why = "consumer rule: the consumer's outermost loops differ from the producer's";
            } else {
                for (int r = p + 1; r < st.consumer; ++r)
                    if (d >= int(s.stmts[r].loops.size()) || s.stmts[r].loops[d] != st.loops[d]) {
                        why = "in-between rule: a statement between producer and consumer does not share the fused loops";
                        who = r;
                        break;
                    }
            }
            if (!why) continue;
            if (want < 0) break;                       // longest legal prefix found
            if (who >= 0)
                set_error("statement %d -> %d, fused loop %d: %s (statement %d)", p, st.consumer, d, why, who);
            else
                set_error("statement %d -> %d, fused loop %d: %s", p, st.consumer, d, why);
            return CONSTSTN_ESCHED;
        }
        st.fused_depth = d;
        st.reduced_order = int(st.out.idx.size()) - d;
    }
    s.lowered = lower_schedule(s);
    return CONSTSTN_OK;
}

// ---- lowering to forall / where (Sec. 4.2, Algorithm 1) -------------------------------------
//
// Work list entries carry the assignment with its current (already reduced) references and
// the part of pi not yet turned into loops.  One level of recursion: walk the list, open a new
// group whenever the leading loop index differs from the previous entry's (an entry with no
// loops left is a group of its own); one group => emit forall (or the assignment itself);
// several => the last group consumes what the earlier ones produce => where(last, rest).

namespace {

struct Item {
    int stmt;
    Ref out, a, b;
    std::vector<std::string> loops;
};

std::string assignment_text(const Item &it) {
    return ref_text(it.out, '(', ')') + " = " + ref_text(it.a, '(', ')') + " * " + ref_text(it.b, '(', ')');
}

void strip(Ref &r, const std::string &idx) {
    auto it = std::find(r.idx.begin(), r.idx.end(), idx);
    if (it != r.idx.end()) r.idx.erase(it);
}

std::string generate(const Schedule &s, const std::vector<Item> &list) {
    struct Group { bool is_index; std::string index; std::vector<Item> items; };
    std::vector<Group> groups;
    for (const Item &it : list) {
        if (it.loops.empty()) {
            groups.push_back(Group{false, "", {it}});
        } else {
            const std::string &i = it.loops.front();
            if (groups.empty() || !groups.back().is_index || groups.back().index != i)
                groups.push_back(Group{true, i, {}});
            groups.back().items.push_back(it);
        }
    }
    if (groups.size() == 1) {
        Group &g = groups[0];
        if (!g.is_index) return assignment_text(g.items[0]);
        // open loop g.index around the group: drop it from every pi, and from every
        // intermediate whose producer and consumer both sit inside the group
        std::set<int> inside;
        for (const Item &it : g.items) inside.insert(it.stmt);
        std::vector<Item> body = g.items;
        for (Item &it : body) {
            it.loops.erase(it.loops.begin());
            const Stmt &st = s.stmts[it.stmt];
            if (st.consumer >= 0 && inside.count(st.consumer)) strip(it.out, g.index);
            if (st.src_a >= 0 && inside.count(st.src_a)) strip(it.a, g.index);
            if (st.src_b >= 0 && inside.count(st.src_b)) strip(it.b, g.index);
        }
        return "forall(" + g.index + ", " + generate(s, body) + ")";
    }
    std::vector<Item> rest;
    for (size_t gi = 0; gi + 1 < groups.size(); ++gi)
        rest.insert(rest.end(), groups[gi].items.begin(), groups[gi].items.end());
    return "where(" + generate(s, groups.back().items) + ", " + generate(s, rest) + ")";
}

}  // namespace

std::string lower_schedule(const Schedule &s) {
    std::vector<Item> list;
    for (size_t p = 0; p < s.stmts.size(); ++p)
        list.push_back(Item{int(p), s.stmts[p].out, s.stmts[p].a, s.stmts[p].b, s.stmts[p].loops});
    return generate(s, list);
}

}  // namespace cst
