// Host planner: queries -> operator-level frontiers (Sec. 4.1) + index arrays (Sec. 4.2).
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "ngdb.h"

namespace ngdb {

struct HostPlan {
    int32_t n_queries = 0, n_groups = 0, n_levels = 0, n_slots = 0, n_anchor = 0;
    int32_t n_proj = 0, n_inter = 0, n_neg = 0, n_int_rows = 0, n_roots = 0;
    int32_t max_branch = 0;          // largest number of conjunctive branches of a query
    int32_t peak_live = 0;           // most operator outputs alive at once under eager reference counting
    std::vector<int32_t> lvl_off;
    std::vector<int32_t> g_level, g_type, g_nin, g_n, g_out_base, g_mlp_base, g_ref_off, g_rel_off;
    std::vector<int32_t> in_ref, in_gslot, rel;
    std::vector<int32_t> root_off, root_slot;
    std::vector<int32_t> anchor_ent, pos;
    std::vector<int32_t> r_uniq, r_seg_off, r_src;
    // forward-only passes with eager reference counting (Sec. 4.3): storage row of every output
    // slot when a row is reused once the output's consumer has run, the number of rows that takes
    // (= peak_live), and per type (projection, intersection, negation) the most MLP rows of one step
    std::vector<int32_t> f_row;
    int32_t n_f_rows = 0;
    int32_t f_step_rows[3] = {0, 0, 0};
};

// Returns NGDB_OK or an error code; `err` receives the reason.
int build_plan(const ngdb_query_batch& qb, int32_t n_entities, int32_t n_relations, int32_t schedule,
               int32_t b_max, HostPlan& out, std::string& err);

}  // namespace ngdb
