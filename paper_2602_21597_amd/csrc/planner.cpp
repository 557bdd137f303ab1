// Host planner.  Turns a batch of query trees into the paper's operator pools
// (Sec. 4.1) resolved ahead of time into a sequence of execution steps.  Two
// schedules: level-synchronous -- at every depth, the operators of one type
// (and, for intersections, one input count: the classes C_k of Sec. 4.3) from
// all queries form one group, all groups of a depth are one step; and the
// paper's Max-Fillness loop (Sec. 4.1 "Dynamic Scheduling", Alg. 1) -- ready
// operators wait in one pool per class, every step runs up to B_max operators
// of the fullest pool.  All gather / scatter positions are resolved here, ahead
// of the step (Sec. 4.2 "Efficient Tensor Indexing").  The numbering rules are
// stated in ngdb.h (ngdb_plan_view).
#include "planner.h"

#include <algorithm>
#include <functional>
#include <queue>
#include <climits>
#include <numeric>

namespace ngdb {
namespace {

struct Tree {          // node of a union-free branch (no heap: at most NGDB_MAX_CARD inputs)
    int32_t type, arg, n_kids;
    int32_t kids[NGDB_MAX_CARD];
};

struct Expander {
    const ngdb_query_batch& qb;
    int32_t base;                 // first node of the current query
    int32_t n_local;
    std::vector<Tree>& pool;
    std::string& err;
    int code = NGDB_OK;

    int32_t make(int32_t type, int32_t arg, const int32_t* kids, int32_t n_kids) {
        Tree t;
        t.type = type; t.arg = arg; t.n_kids = n_kids;
        for (int32_t k = 0; k < n_kids; ++k) t.kids[k] = kids[k];
        pool.push_back(t);
        return (int32_t)pool.size() - 1;
    }

    // Appends the conjunctive branches of the sub-query rooted at local node j to `out`.
    void expand(int32_t j, int depth, std::vector<int32_t>& out) {
        if (code != NGDB_OK) return;
        if (depth > NGDB_MAX_LEVELS + 1) {
            code = NGDB_ERR_UNSUPPORTED;
            err = "query deeper than NGDB_MAX_LEVELS";
            return;
        }
        const int32_t n = base + j;
        const int32_t lo = qb.in_off[n], hi = qb.in_off[n + 1];
        const int op = qb.op[n];
        const size_t first = out.size();
        switch (op) {
            case NGDB_OP_ANCHOR:
                out.push_back(make(NGDB_OP_ANCHOR, qb.arg[n], nullptr, 0));
                break;
            case NGDB_OP_PROJ: {
                expand(qb.in_idx[lo], depth + 1, out);          // one projection on top of every branch of the input
                for (size_t i = first; i < out.size() && code == NGDB_OK; ++i) {
                    const int32_t kid = out[i];
                    out[i] = make(NGDB_OP_PROJ, qb.arg[n], &kid, 1);
                }
                break;
            }
            case NGDB_OP_UNION: {
                for (int32_t k = lo; k < hi; ++k) expand(qb.in_idx[k], depth + 1, out);
                break;
            }
            default: {   // INTER, NEG: every input must be union-free
                int32_t kids[NGDB_MAX_CARD];
                int32_t n_kids = 0;
                for (int32_t k = lo; k < hi; ++k) {
                    const size_t before = out.size();
                    expand(qb.in_idx[k], depth + 1, out);
                    if (code != NGDB_OK) return;
                    if (out.size() != before + 1) {
                        code = NGDB_ERR_UNSUPPORTED;
                        err = "union below an intersection or a negation";
                        return;
                    }
                    kids[n_kids++] = out.back();                // validate() bounds the input count
                    out.pop_back();
                }
                out.push_back(make(op, 0, kids, n_kids));
            }
        }
        if (out.size() - first > (size_t)NGDB_MAX_BRANCH && code == NGDB_OK) {
            code = NGDB_ERR_UNSUPPORTED;
            err = "query has more than NGDB_MAX_BRANCH conjunctive branches";
        }
    }
};

struct Flat {   // all nodes of the batch after DNF, by global id
    std::vector<int32_t> type, arg, level, in_off, in;
    int32_t add(int32_t t, int32_t a, int32_t lvl, const int32_t* ins, int32_t n_ins) {
        type.push_back(t);
        arg.push_back(a);
        level.push_back(lvl);
        in.insert(in.end(), ins, ins + n_ins);
        in_off.push_back((int32_t)in.size());
        return (int32_t)type.size() - 1;
    }
    int32_t nin(int32_t g) const { return in_off[g + 1] - in_off[g]; }
};

int32_t number_postorder(const std::vector<Tree>& pool, int32_t t, Flat& flat) {
    const Tree& node = pool[t];
    int32_t ins[NGDB_MAX_CARD];
    int32_t lvl = 0;
    for (int32_t k = 0; k < node.n_kids; ++k) {
        ins[k] = number_postorder(pool, node.kids[k], flat);
        lvl = std::max(lvl, flat.level[ins[k]] + 1);
    }
    return flat.add(node.type, node.arg, lvl, ins, node.n_kids);
}

// Max-Fillness schedule (Alg. 1 without the gradient nodes, which mirror it): returns the step
// (1-based) in which every operator node runs.  One pool per class (type, input count), in
// the order PROJ < INTER by input count < NEG.  A cycle files the newly ready operators into
// their pools in node order, picks the pool with the most entries (fillness = entries / B_max
// with one B_max for all classes; ties to the first class), and runs its first min(size,
// B_max) entries; consumers whose inputs are all done become ready for the next cycle.  The
// loop runs until every pool is empty (the printed loop condition, "ready set not empty",
// would strand the remainder of a pool that was cut at B_max).  Also returns the largest
// number of operator outputs alive at once under eager reference counting (Sec. 4.3): an
// output dies when its consumer has run; the outputs of roots stay for scoring.
void max_fillness_steps(const Flat& flat, int32_t b_max, std::vector<int32_t>& step, int32_t& peak_live) {
    const int32_t n = (int32_t)flat.type.size();
    auto cls = [&](int32_t g) {
        const int32_t t = flat.type[g];
        return t == NGDB_OP_PROJ ? 0 : (t == NGDB_OP_INTER ? flat.nin(g) - 1 : NGDB_MAX_CARD);   // 0, 1..7, 8
    };
    constexpr int N_CLS = NGDB_MAX_CARD + 1;
    std::vector<int32_t> consumer(n, -1), waiting(n, 0);
    for (int32_t g = 0; g < n; ++g)
        for (int32_t k = flat.in_off[g]; k < flat.in_off[g + 1]; ++k) {
            consumer[flat.in[k]] = g;
            if (flat.type[flat.in[k]] != NGDB_OP_ANCHOR) ++waiting[g];
        }
    std::vector<std::vector<int32_t>> pool(N_CLS);
    std::vector<size_t> head(N_CLS, 0);
    std::vector<int32_t> ready;
    for (int32_t g = 0; g < n; ++g)
        if (flat.type[g] != NGDB_OP_ANCHOR && waiting[g] == 0) ready.push_back(g);
    step.assign(n, 0);
    int32_t s = 0, live = 0;
    peak_live = 0;
    for (;;) {
        std::sort(ready.begin(), ready.end());
        for (int32_t g : ready) pool[cls(g)].push_back(g);
        ready.clear();
        int best = -1;
        size_t best_n = 0;
        for (int c = 0; c < N_CLS; ++c) {
            const size_t cnt = pool[c].size() - head[c];
            if (cnt > best_n) { best_n = cnt; best = c; }
        }
        if (best < 0) break;
        const size_t take = b_max > 0 ? std::min<size_t>(best_n, (size_t)b_max) : best_n;
        ++s;
        live += (int32_t)take;                       // outputs of this step exist next to their inputs
        peak_live = std::max(peak_live, live);
        for (size_t i = 0; i < take; ++i) {
            const int32_t g = pool[best][head[best] + i];
            step[g] = s;
            for (int32_t k = flat.in_off[g]; k < flat.in_off[g + 1]; ++k)
                if (flat.type[flat.in[k]] != NGDB_OP_ANCHOR) --live;   // its only consumer has run
            const int32_t c = consumer[g];
            if (c >= 0 && --waiting[c] == 0) ready.push_back(c);
        }
        head[best] += take;
    }
}

int validate(const ngdb_query_batch& qb, int32_t N, int32_t R, std::string& err) {
    if (qb.n_queries < 0) { err = "n_queries < 0"; return NGDB_ERR_ARG; }
    if (qb.n_queries == 0) return NGDB_OK;
    if (!qb.node_off || !qb.op || !qb.arg || !qb.in_off || !qb.pos) {
        err = "null array in query batch";
        return NGDB_ERR_ARG;
    }
    if (qb.node_off[0] != 0 || qb.in_off[0] != 0) { err = "offsets must start at 0"; return NGDB_ERR_ARG; }
    for (int32_t q = 0; q < qb.n_queries; ++q) {
        const int32_t lo = qb.node_off[q], hi = qb.node_off[q + 1];
        if (hi <= lo) { err = "query without nodes"; return NGDB_ERR_ARG; }
        if (qb.pos[q] < 0 || qb.pos[q] >= N) { err = "positive entity id out of range"; return NGDB_ERR_RANGE; }
        for (int32_t n = lo; n < hi; ++n) {
            const int32_t a = qb.in_off[n], b = qb.in_off[n + 1];
            if (b < a) { err = "in_off not monotone"; return NGDB_ERR_ARG; }
            const int32_t nin = b - a;
            if (nin > 0 && !qb.in_idx) { err = "null in_idx"; return NGDB_ERR_ARG; }
            for (int32_t k = a; k < b; ++k)
                if (qb.in_idx[k] < 0 || qb.in_idx[k] >= n - lo) {
                    err = "input must be an earlier node of the same query";
                    return NGDB_ERR_ARG;
                }
            switch (qb.op[n]) {
                case NGDB_OP_ANCHOR:
                    if (nin != 0) { err = "anchor with inputs"; return NGDB_ERR_ARG; }
                    if (qb.arg[n] < 0 || qb.arg[n] >= N) { err = "anchor entity id out of range"; return NGDB_ERR_RANGE; }
                    break;
                case NGDB_OP_PROJ:
                    if (nin != 1) { err = "projection needs one input"; return NGDB_ERR_ARG; }
                    if (qb.arg[n] < 0 || qb.arg[n] >= R) { err = "relation id out of range"; return NGDB_ERR_RANGE; }
                    break;
                case NGDB_OP_NEG:
                    if (nin != 1) { err = "negation needs one input"; return NGDB_ERR_ARG; }
                    break;
                case NGDB_OP_INTER:
                    if (nin < 2) { err = "intersection needs at least two inputs"; return NGDB_ERR_ARG; }
                    if (nin > NGDB_MAX_CARD) { err = "intersection with more than NGDB_MAX_CARD inputs"; return NGDB_ERR_UNSUPPORTED; }
                    break;
                case NGDB_OP_UNION:
                    if (nin < 1) { err = "union without inputs"; return NGDB_ERR_ARG; }
                    break;
                default:
                    err = "unknown operator code";
                    return NGDB_ERR_ARG;
            }
        }
    }
    return NGDB_OK;
}

// order = positions 0..n-1 sorted stably by key[position], keys in [0, key_bound): a counting
// sort where the key range allows it (the keys here are small composites), else a merge sort.
void stable_order_by_key(const std::vector<int32_t>& key, int64_t key_bound, std::vector<int32_t>& order) {
    const size_t n = key.size();
    order.resize(n);
    if (key_bound <= (int64_t)(4 * n + 1024)) {
        std::vector<int32_t> start((size_t)key_bound + 1, 0);
        for (size_t i = 0; i < n; ++i) ++start[key[i] + 1];
        for (int64_t k = 0; k < key_bound; ++k) start[k + 1] += start[k];
        for (size_t i = 0; i < n; ++i) order[start[key[i]]++] = (int32_t)i;
        return;
    }
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return key[a] < key[b]; });
}

// Stable grouping of `keys` (values < n_keys): unique keys ascending, segment
// offsets, and the permutation that lists each segment's members in input order.
void segment_index(const std::vector<int32_t>& keys, int32_t n_keys, std::vector<int32_t>& uniq,
                   std::vector<int32_t>& seg_off, std::vector<int32_t>& order) {
    stable_order_by_key(keys, n_keys, order);
    uniq.clear();
    seg_off.clear();
    for (size_t i = 0; i < order.size(); ++i)
        if (i == 0 || keys[order[i]] != keys[order[i - 1]]) {
            uniq.push_back(keys[order[i]]);
            seg_off.push_back((int32_t)i);
        }
    seg_off.push_back((int32_t)order.size());
}

}  // namespace

int build_plan(const ngdb_query_batch& qb, int32_t N, int32_t R, int32_t schedule, int32_t b_max, HostPlan& P,
               std::string& err) {
    if ((schedule != NGDB_SCHED_LEVEL && schedule != NGDB_SCHED_MAX_FILL) || b_max < 0) {
        err = "unknown schedule or negative b_max";
        return NGDB_ERR_ARG;
    }
    int rc = validate(qb, N, R, err);
    if (rc != NGDB_OK) return rc;
    P = HostPlan{};
    const int32_t B = qb.n_queries;
    P.n_queries = B;
    P.pos.assign(qb.pos, qb.pos + B);

    // 1. DNF + global numbering
    Flat flat;
    flat.in_off.push_back(0);
    std::vector<std::vector<int32_t>> roots(B);
    std::vector<Tree> pool;
    std::vector<int32_t> branches;
    for (int32_t q = 0; q < B; ++q) {
        pool.clear();
        Expander ex{qb, qb.node_off[q], qb.node_off[q + 1] - qb.node_off[q], pool, err};
        branches.clear();
        ex.expand(ex.n_local - 1, 0, branches);
        if (ex.code != NGDB_OK) return ex.code;
        for (int32_t b : branches) {
            if (pool[b].type == NGDB_OP_ANCHOR) {
                err = "a query must contain at least one operator";
                return NGDB_ERR_UNSUPPORTED;
            }
            int32_t g = number_postorder(pool, b, flat);
            if (flat.level[g] > NGDB_MAX_LEVELS) {
                err = "query deeper than NGDB_MAX_LEVELS";
                return NGDB_ERR_UNSUPPORTED;
            }
            roots[q].push_back(g);
        }
        P.max_branch = std::max<int32_t>(P.max_branch, (int32_t)branches.size());
    }
    const int32_t n_nodes = (int32_t)flat.type.size();

    // 1b. execution step of every operator: its depth, or its Max-Fillness step.  From here
    // on "level" means execution step.  The eager-reclamation peak of the level-synchronous
    // order is computed the same way: outputs of a step appear, then their inputs die.
    if (schedule == NGDB_SCHED_MAX_FILL) {
        std::vector<int32_t> step;
        max_fillness_steps(flat, b_max, step, P.peak_live);
        flat.level = step;
    } else {
        int32_t max_level = 0;
        for (int32_t g = 0; g < n_nodes; ++g) max_level = std::max(max_level, flat.level[g]);
        std::vector<int32_t> born(max_level + 2, 0), dead(max_level + 2, 0);
        for (int32_t g = 0; g < n_nodes; ++g) {
            if (flat.type[g] == NGDB_OP_ANCHOR) continue;
            ++born[flat.level[g]];
            for (int32_t k = flat.in_off[g]; k < flat.in_off[g + 1]; ++k)
                if (flat.type[flat.in[k]] != NGDB_OP_ANCHOR) ++dead[flat.level[g]];
        }
        int32_t live = 0;
        for (int32_t l = 1; l <= max_level; ++l) {
            live += born[l];
            P.peak_live = std::max(P.peak_live, live);
            live -= dead[l];
        }
    }

    // 2. anchors and operator nodes
    std::vector<int32_t> ops, anchor_idx(n_nodes, -1);
    for (int32_t g = 0; g < n_nodes; ++g) {
        if (flat.type[g] == NGDB_OP_ANCHOR) {
            anchor_idx[g] = (int32_t)P.anchor_ent.size();
            P.anchor_ent.push_back(flat.arg[g]);
        } else {
            ops.push_back(g);
        }
    }
    P.n_anchor = (int32_t)P.anchor_ent.size();
    P.n_slots = (int32_t)ops.size();

    // 3. slots: type-major, then level, input count, node id
    auto type_rank = [](int32_t t) { return t == NGDB_OP_PROJ ? 0 : (t == NGDB_OP_INTER ? 1 : 2); };
    int32_t top_level = 0;
    for (int32_t g : ops) top_level = std::max(top_level, flat.level[g]);
    const int64_t n_lvl = (int64_t)top_level + 1, n_card = NGDB_MAX_CARD + 1;
    std::vector<int32_t> key(ops.size()), order;
    std::vector<int32_t> by_slot(ops.size());
    if (3 * n_lvl * n_card > INT32_MAX) {
        err = "too many execution steps";
        return NGDB_ERR_UNSUPPORTED;
    }
    for (size_t i = 0; i < ops.size(); ++i)
        key[i] = (int32_t)((type_rank(flat.type[ops[i]]) * n_lvl + flat.level[ops[i]]) * n_card + flat.nin(ops[i]));
    stable_order_by_key(key, 3 * n_lvl * n_card, order);
    for (size_t i = 0; i < ops.size(); ++i) by_slot[i] = ops[order[i]];
    std::vector<int32_t> slot(n_nodes, -1);
    for (int32_t s = 0; s < P.n_slots; ++s) {
        slot[by_slot[s]] = s;
        const int32_t t = flat.type[by_slot[s]];
        if (t == NGDB_OP_PROJ) ++P.n_proj;
        else if (t == NGDB_OP_INTER) ++P.n_inter;
        else ++P.n_neg;
    }
    const int32_t type_base[3] = {0, P.n_proj, P.n_proj + P.n_inter};
    auto grad_row = [&](int32_t g) { return slot[g] >= 0 ? slot[g] : P.n_slots + anchor_idx[g]; };

    // 4. groups: level, type, input count; members in node order
    std::vector<int32_t> by_group(ops.size());
    for (size_t i = 0; i < ops.size(); ++i)
        key[i] = (int32_t)((flat.level[ops[i]] * 3 + type_rank(flat.type[ops[i]])) * n_card + flat.nin(ops[i]));
    stable_order_by_key(key, 3 * n_lvl * n_card, order);
    for (size_t i = 0; i < ops.size(); ++i) by_group[i] = ops[order[i]];
    size_t i = 0;
    while (i < by_group.size()) {
        const int32_t g0 = by_group[i];
        size_t j = i;
        while (j < by_group.size() && flat.level[by_group[j]] == flat.level[g0] &&
               flat.type[by_group[j]] == flat.type[g0] && flat.nin(by_group[j]) == flat.nin(g0))
            ++j;
        const int32_t n = (int32_t)(j - i), nin = flat.nin(g0), t = flat.type[g0];
        P.g_level.push_back(flat.level[g0]);
        P.g_type.push_back(t);
        P.g_nin.push_back(nin);
        P.g_n.push_back(n);
        P.g_out_base.push_back(slot[g0]);
        P.g_ref_off.push_back((int32_t)P.in_ref.size());
        if (t == NGDB_OP_INTER) {
            P.g_mlp_base.push_back(P.n_int_rows);
            P.n_int_rows += n * nin;
        } else {
            P.g_mlp_base.push_back(slot[g0] - type_base[type_rank(t)]);
        }
        P.g_rel_off.push_back(t == NGDB_OP_PROJ ? (int32_t)P.rel.size() : -1);
        for (int32_t k = 0; k < nin; ++k)
            for (size_t m = i; m < j; ++m) {
                const int32_t c = flat.in[flat.in_off[by_group[m]] + k];
                P.in_ref.push_back(slot[c] >= 0 ? slot[c] : -1 - flat.arg[c]);
                P.in_gslot.push_back(grad_row(c));
            }
        if (t == NGDB_OP_PROJ)
            for (size_t m = i; m < j; ++m) P.rel.push_back(flat.arg[by_group[m]]);
        i = j;
    }
    P.n_groups = (int32_t)P.g_level.size();
    P.n_levels = P.n_groups ? P.g_level.back() : 0;
    P.lvl_off.assign(P.n_levels + 2, 0);
    for (int32_t l : P.g_level) P.lvl_off[l + 1] += 1;
    for (size_t l = 1; l < P.lvl_off.size(); ++l) P.lvl_off[l] += P.lvl_off[l - 1];

    // 5. roots
    P.root_off.push_back(0);
    for (int32_t q = 0; q < B; ++q) {
        for (int32_t g : roots[q]) P.root_slot.push_back(slot[g]);
        P.root_off.push_back((int32_t)P.root_slot.size());
    }
    P.n_roots = (int32_t)P.root_slot.size();

    // 6. relation gradient index over the projections in slot order
    std::vector<int32_t> rkeys(P.n_proj), rsrc(P.n_proj);
    for (int32_t s = 0; s < P.n_proj; ++s) {
        const int32_t g = by_slot[s];
        rkeys[s] = flat.arg[g];
        rsrc[s] = grad_row(flat.in[flat.in_off[g]]);
    }
    segment_index(rkeys, R, P.r_uniq, P.r_seg_off, order);
    P.r_src.resize(P.n_proj);
    for (int32_t s = 0; s < P.n_proj; ++s) P.r_src[s] = rsrc[order[s]];

    // 7. rows of a forward-only pass under eager reference counting (Sec. 4.3, Reclaim(T); Alg. 1,
    // DecrementRefCounts): the steps in order; every output of a step takes, in group and member
    // order, the lowest free row (a new one if none is free); when the step has run, the rows of
    // the outputs it consumed are free again.  Every output has one consumer (queries are trees);
    // roots have none and keep their rows.
    P.f_row.assign(P.n_slots, -1);
    std::priority_queue<int32_t, std::vector<int32_t>, std::greater<int32_t>> free_rows;
    P.n_f_rows = 0;
    for (int32_t l = 1; l <= P.n_levels; ++l) {
        int32_t rows_now[3] = {0, 0, 0};
        for (int32_t g = P.lvl_off[l]; g < P.lvl_off[l + 1]; ++g) {
            const int32_t t = P.g_type[g];
            rows_now[t == NGDB_OP_PROJ ? 0 : (t == NGDB_OP_INTER ? 1 : 2)] += P.g_n[g] * (t == NGDB_OP_INTER ? P.g_nin[g] : 1);
            for (int32_t m = 0; m < P.g_n[g]; ++m) {
                int32_t row;
                if (!free_rows.empty()) {
                    row = free_rows.top();
                    free_rows.pop();
                } else {
                    row = P.n_f_rows++;
                }
                P.f_row[P.g_out_base[g] + m] = row;
            }
        }
        for (int32_t g = P.lvl_off[l]; g < P.lvl_off[l + 1]; ++g) {
            const int32_t n_ref = P.g_n[g] * P.g_nin[g];
            for (int32_t k = 0; k < n_ref; ++k) {
                const int32_t ref = P.in_ref[P.g_ref_off[g] + k];
                if (ref >= 0) free_rows.push(P.f_row[ref]);
            }
        }
        for (int k = 0; k < 3; ++k) P.f_step_rows[k] = std::max(P.f_step_rows[k], rows_now[k]);
    }
    return NGDB_OK;
}

}  // namespace ngdb
