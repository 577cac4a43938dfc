// Host-side representation of a schedule: the paper's sequence S of pairs <A, pi>
// (Sec. 4.2) plus the operand table, after parsing and legality checking (Sec. 3.2).
#pragma once

#include <map>
#include <string>
#include <vector>

#include "common.hpp"

namespace cst {

struct Ref {
    std::string name;
    std::vector<std::string> idx;
};

struct Stmt {
    Ref out, a, b;
    std::vector<std::string> loops;      // pi: outermost first
    // filled by validation
    int src_a = -1, src_b = -1;          // producing statement of each input, -1 = an operand
    int op_a = -1, op_b = -1;            // operand ordinal when the input is an operand
    int consumer = -1;                   // statement that consumes out, -1 = result
    int fused_depth = 0;                 // loops shared with the consumer
    int reduced_order = 0;               // order of out after fusion
};

struct OperandInfo {
    std::string name;
    int kind = CONSTSTN_OPERAND_DENSE;
    const conststn_csf_s *csf = nullptr;
    int order = 0;
    int64_t dims[CONSTSTN_MAX_ORDER] = {0};   // CSF: extents in LEVEL order; dense: storage order
    int dense_ordinal = -1;                   // position among the dense operands
    const double *owned = nullptr;            // dense copy kept by the plan (a CSF operand the generic executor spread out)
};

struct Schedule {
    std::vector<Stmt> stmts;
    std::vector<OperandInfo> operands;
    std::map<std::string, int64_t> extent;   // index name -> extent
    std::string lowered;                     // forall/where text of the fused loop tree
};

// Parse `text` into sched.stmts.  CONSTSTN_EINVAL on malformed text.
conststn_status parse_schedule(const char *text, Schedule &sched);

// Bind operands, resolve producers/consumers, check every legality rule, resolve fusion
// depths (fusion may be null), and lower to forall/where text.
conststn_status validate_schedule(Schedule &sched, const int *fusion, int n_operands,
                                  const conststn_operand_desc *operands);

// Schedule search (search.cpp): the smallest l for which the tree given in `tree` (statements without
// loop orders) has a legal schedule with every intermediate of order <= l, and one such schedule.
// keep_layout: references to CSF operands are level orders to keep; otherwise they list the modes
// and the level order is chosen.  level_modes[o][level] = position in the tree's reference.
conststn_status search_schedule(const char *tree, int n_operands, const conststn_operand_desc *operands,
                                bool keep_layout, int max_order, Schedule &result, int *order_found,
                                std::vector<std::vector<int>> &level_modes);

// "OUT[..] = A[..] * B[..] | loops ; ..." of a schedule
std::string schedule_text(const Schedule &s);

// Lowering of a sequence of <A, pi> into nested forall / where text (Sec. 4.2, Algorithm 1).
std::string lower_schedule(const Schedule &sched);

}  // namespace cst
