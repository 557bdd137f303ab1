// Online query sampler (App. "Stochastic Online Query Sampling"): batches of
// first-order-logic queries are synthesised on the fly from the graph instead
// of being read from a pre-computed set.  A query is a template (one of the 14
// patterns of Sec. 3.1) instantiated by a restricted random walk that runs
// backwards from the answer -- a projection reaching entity v takes a uniform
// in-edge of v, the children of an intersection all reach v, a negated or a
// second union branch is grown toward an unrelated entity -- followed by
// rejection: walks that hit an entity without in-edges, intersections with two
// identical children, and queries whose end point is not an answer (it may lie
// in a negated branch) are drawn again, so every query has a non-empty answer
// set that contains its positive.  Host only, C++ threads; every query draws
// from its own counter-based random stream (seed, batch number, query number),
// so a batch does not depend on the number of threads.
#include <algorithm>
#include <condition_variable>
#include <cstring>
#include <functional>
#include <mutex>
#include <new>
#include <numeric>
#include <memory>
#include <string>
#include <thread>
#include <vector>

#include "ngdb.h"

namespace {

// ---------------------------------------------------------------- random stream
struct Rng {   // splitmix64 over a per-query counter
    uint64_t s;
    Rng(uint64_t seed, uint64_t batch, uint64_t query) {
        s = seed ^ (batch * 0x9E3779B97F4A7C15ull) ^ (query * 0xC2B2AE3D27D4EB4Full + 0x165667B19E3779F9ull);
        next();
        next();
    }
    uint64_t next() {
        uint64_t z = (s += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    // uniform in [0, n), n > 0 (multiply-shift with rejection of the biased tail)
    uint64_t below(uint64_t n) {
        for (;;) {
            const uint64_t x = next();
            const unsigned __int128 m = (unsigned __int128)x * n;
            if ((uint64_t)m >= (uint64_t)(-n) % n) return (uint64_t)(m >> 64);
        }
    }
    double unit() { return (double)(next() >> 11) * (1.0 / 9007199254740992.0); }
    // two uniform draws in [0, n), n < 2^31, from one 64-bit word (each half: multiply-shift,
    // redrawn together if either falls into the biased tail)
    void below32x2(uint32_t n, int32_t* out) {
        const uint32_t tail = (uint32_t)(-n) % n;
        for (;;) {
            const uint64_t x = next();
            const uint64_t a = (uint64_t)(uint32_t)x * n, b = (x >> 32) * n;
            if ((uint32_t)a >= tail && (uint32_t)b >= tail) {
                out[0] = (int32_t)(a >> 32);
                out[1] = (int32_t)(b >> 32);
                return;
            }
        }
    }
};

// Worker threads that live as long as the sampler: a call hands them a function of the
// worker number and waits for all of them.
class Workers {
public:
    explicit Workers(int n) {
        for (int i = 0; i < n; ++i) threads_.emplace_back([this, i] { loop(i); });
    }
    ~Workers() {
        {
            std::lock_guard<std::mutex> lk(mu_);
            stop_ = true;
            ++round_;
        }
        cv_.notify_all();
        for (std::thread& t : threads_) t.join();
    }
    int size() const { return (int)threads_.size(); }
    // fn must stay alive until wait() has returned
    void start(const std::function<void(int)>& fn) {
        {
            std::lock_guard<std::mutex> lk(mu_);
            fn_ = &fn;
            pending_ = (int)threads_.size();
            ++round_;
        }
        cv_.notify_all();
    }
    void wait() {
        std::unique_lock<std::mutex> lk(mu_);
        done_.wait(lk, [this] { return pending_ == 0; });
    }

private:
    void loop(int i) {
        uint64_t seen = 0;
        for (;;) {
            const std::function<void(int)>* fn;
            {
                std::unique_lock<std::mutex> lk(mu_);
                cv_.wait(lk, [&] { return round_ != seen; });
                seen = round_;
                if (stop_) return;
                fn = fn_;
            }
            (*fn)(i);
            {
                std::lock_guard<std::mutex> lk(mu_);
                if (--pending_ == 0) done_.notify_one();
            }
        }
    }
    std::vector<std::thread> threads_;
    std::mutex mu_;
    std::condition_variable cv_, done_;
    const std::function<void(int)>* fn_ = nullptr;
    uint64_t round_ = 0;
    int pending_ = 0;
    bool stop_ = false;
};

// ---------------------------------------------------------------- graph
struct Graph {
    int32_t N = 0, R = 0;
    int64_t T = 0;
    std::vector<int64_t> in_off, out_off;          // [N+1]
    std::vector<int32_t> in_head, in_rel;          // in-edges of every entity, any fixed order
    std::vector<int32_t> out_rel, out_tail;        // out-edges sorted by (relation, tail)
    std::vector<int32_t> tails;                    // tail of every triple (answers are drawn from it)

    bool has_triple(int32_t h, int32_t r, int32_t t) const {
        int64_t lo = out_off[h], hi = out_off[h + 1];
        while (lo < hi) {
            const int64_t mid = (lo + hi) >> 1;
            if (out_rel[mid] < r || (out_rel[mid] == r && out_tail[mid] < t)) lo = mid + 1; else hi = mid;
        }
        return lo < out_off[h + 1] && out_rel[lo] == r && out_tail[lo] == t;
    }
};

// ---------------------------------------------------------------- templates
struct Tmpl {            // node of a template tree
    char kind;           // 'e' 'p' 'i' 'n' 'u'
    std::vector<int> kids;
};
struct Template {
    std::string name;
    std::vector<Tmpl> nodes;   // root last
};

// shapes in a small prefix notation: e, p(x), i(x,..), n(x), u(x,..)
int parse(const char*& s, std::vector<Tmpl>& out) {
    Tmpl t;
    t.kind = *s++;
    if (t.kind != 'e') {
        ++s;   // '('
        for (;;) {
            t.kids.push_back(parse(s, out));
            if (*s == ',') { ++s; continue; }
            ++s;   // ')'
            break;
        }
    }
    out.push_back(t);
    return (int)out.size() - 1;
}

const char* shape_of(const std::string& name) {
    static const char* const table[][2] = {
        {"1p", "p(e)"}, {"2p", "p(p(e))"}, {"3p", "p(p(p(e)))"}, {"2i", "i(p(e),p(e))"}, {"3i", "i(p(e),p(e),p(e))"},
        {"ip", "p(i(p(e),p(e)))"}, {"pi", "i(p(p(e)),p(e))"}, {"2u", "u(p(e),p(e))"}, {"up", "p(u(p(e),p(e)))"},
        {"2in", "i(p(e),n(p(e)))"}, {"3in", "i(p(e),p(e),n(p(e)))"}, {"inp", "p(i(p(e),n(p(e))))"},
        {"pin", "i(p(p(e)),n(p(e)))"}, {"pni", "i(n(p(p(e))),p(e))"}};
    for (const auto& row : table)
        if (name == row[0]) return row[1];
    return nullptr;
}

// ---------------------------------------------------------------- one query
struct Query {           // nodes in post-order, root last
    std::vector<uint8_t> op;
    std::vector<int32_t> arg, in_off, in_idx;
    void clear() { op.clear(); arg.clear(); in_idx.clear(); in_off.assign(1, 0); }
    int add(uint8_t o, int32_t a, const int* ins, int n) {
        op.push_back(o);
        arg.push_back(a);
        in_idx.insert(in_idx.end(), ins, ins + n);
        in_off.push_back((int32_t)in_idx.size());
        return (int)op.size() - 1;
    }
    void truncate(size_t n_nodes) {
        op.resize(n_nodes);
        arg.resize(n_nodes);
        in_off.resize(n_nodes + 1);
        in_idx.resize(in_off.back());
    }
};

struct Builder {
    const Graph& g;
    const Template& tp;
    Rng& rng;
    Query& q;
    long budget = 0;     // membership tests: edge visits left

    // Is v an answer of the sub-query rooted at node n?  Exact, by walking in-edges; gives
    // up (treated as "cannot tell") when the budget runs out.
    int contains(int n, int32_t v) {
        const uint8_t o = q.op[n];
        const int32_t* ins = q.in_idx.data() + q.in_off[n];
        const int nin = q.in_off[n + 1] - q.in_off[n];
        if (o == NGDB_OP_ANCHOR) return q.arg[n] == v;
        if (o == NGDB_OP_NEG) {
            const int c = contains(ins[0], v);
            return c < 0 ? c : !c;
        }
        if (o == NGDB_OP_INTER || o == NGDB_OP_UNION) {
            for (int k = 0; k < nin; ++k) {
                const int c = contains(ins[k], v);
                if (c < 0) return c;
                if (o == NGDB_OP_INTER && !c) return 0;
                if (o == NGDB_OP_UNION && c) return 1;
            }
            return o == NGDB_OP_INTER;
        }
        // projection by relation r: some m with (m, r, v) in the graph and m an answer of the input
        const int32_t r = q.arg[n];
        if (q.op[ins[0]] == NGDB_OP_ANCHOR) return g.has_triple(q.arg[ins[0]], r, v);
        for (int64_t j = g.in_off[v]; j < g.in_off[v + 1]; ++j) {
            if (--budget < 0) return -1;
            if (g.in_rel[j] != r) continue;
            const int c = contains(ins[0], g.in_head[j]);
            if (c) return c;
        }
        return 0;
    }

    bool same_subtree(size_t a0, size_t a1, size_t b0, size_t b1) const {
        if (a1 - a0 != b1 - b0) return false;
        for (size_t i = 0; i < a1 - a0; ++i) {
            if (q.op[a0 + i] != q.op[b0 + i] || q.arg[a0 + i] != q.arg[b0 + i]) return false;
            const int na = q.in_off[a0 + i + 1] - q.in_off[a0 + i], nb = q.in_off[b0 + i + 1] - q.in_off[b0 + i];
            if (na != nb) return false;
            for (int k = 0; k < na; ++k)
                if (q.in_idx[q.in_off[a0 + i] + k] - (int32_t)a0 != q.in_idx[q.in_off[b0 + i] + k] - (int32_t)b0)
                    return false;
        }
        return true;
    }

    int32_t random_tail() { return g.tails[rng.below((uint64_t)g.T)]; }

    // instantiate template node t so that v is one of its answers; -1 = draw the query again
    int grow(int t, int32_t v) {
        const Tmpl& node = tp.nodes[t];
        switch (node.kind) {
            case 'e':
                return q.add(NGDB_OP_ANCHOR, v, nullptr, 0);
            case 'p': {
                const int64_t lo = g.in_off[v], hi = g.in_off[v + 1];
                if (hi == lo) return -1;
                const int64_t j = lo + (int64_t)rng.below((uint64_t)(hi - lo));
                const int c = grow(node.kids[0], g.in_head[j]);
                if (c < 0) return -1;
                return q.add(NGDB_OP_PROJ, g.in_rel[j], &c, 1);
            }
            case 'n': {
                const int c = grow(node.kids[0], random_tail());
                if (c < 0) return -1;
                return q.add(NGDB_OP_NEG, 0, &c, 1);
            }
            case 'i': {
                std::vector<int> kids;
                std::vector<std::pair<size_t, size_t>> span;
                for (int kt : node.kids) {
                    int c = -1;
                    for (int attempt = 0; attempt < 8; ++attempt) {
                        const size_t start = q.op.size();
                        c = grow(kt, v);
                        if (c < 0) return -1;
                        bool dup = false;
                        for (const auto& sp : span) dup = dup || same_subtree(sp.first, sp.second, start, q.op.size());
                        if (!dup) {
                            span.emplace_back(start, q.op.size());
                            break;
                        }
                        q.truncate(start);
                        c = -1;
                    }
                    if (c < 0) return -1;
                    kids.push_back(c);
                }
                return q.add(NGDB_OP_INTER, 0, kids.data(), (int)kids.size());
            }
            case 'u': {
                std::vector<int> kids;
                for (size_t k = 0; k < node.kids.size(); ++k) {
                    const int c = grow(node.kids[k], k == 0 ? v : random_tail());
                    if (c < 0) return -1;
                    kids.push_back(c);
                }
                return q.add(NGDB_OP_UNION, 0, kids.data(), (int)kids.size());
            }
        }
        return -1;
    }
};

}  // namespace

struct BatchArrays {   // what ngdb_sampler_next hands out
    std::vector<int32_t> node_off, arg, in_off, in_idx, pos, neg;
    std::vector<uint8_t> op, tmpl;
};

struct ngdb_sampler_s {
    Graph g;
    std::vector<Template> templates;
    std::vector<double> cdf;
    uint64_t seed = 0, batch_no = 0;
    int n_threads = 1;
    std::unique_ptr<Workers> workers;   // n_threads - 1 helpers; the caller's thread works too
    std::vector<Query> queries;         // per query scratch, reused
    BatchArrays out[3];                 // three sets taking turns: a batch stays valid over the next call
                                        // while the one after it is already being drawn
    std::string err;
    // Read-ahead: after a call has returned batch t, a coordinator thread draws batch t+1 (same
    // sizes) with the helpers, so that the next call usually finds its batch ready.  The batches
    // are functions of (seed, batch number, query number): reading ahead changes nothing in them.
    std::thread coordinator;
    std::mutex pm;
    std::condition_variable pcv;
    bool pf_requested = false, pf_done = false, pf_stop = false;   // guarded by pm
    uint64_t pf_no = 0;
    int pf_B = 0, pf_K = 0, pf_rc = NGDB_OK;

    ~ngdb_sampler_s() {
        if (coordinator.joinable()) {
            {
                std::lock_guard<std::mutex> lk(pm);
                pf_stop = true;
            }
            pcv.notify_all();
            coordinator.join();
        }
    }
};

namespace {
int fill_batch(ngdb_sampler_s* s, uint64_t batch_no, int32_t B, int32_t K, BatchArrays& o);

void coordinator_loop(ngdb_sampler_s* s) {
    for (;;) {
        uint64_t no;
        int B, K;
        {
            std::unique_lock<std::mutex> lk(s->pm);
            s->pcv.wait(lk, [&] { return s->pf_stop || (s->pf_requested && !s->pf_done); });
            if (s->pf_stop) return;
            no = s->pf_no; B = s->pf_B; K = s->pf_K;
        }
        const int rc = fill_batch(s, no, B, K, s->out[no % 3]);
        {
            std::lock_guard<std::mutex> lk(s->pm);
            s->pf_rc = rc;
            s->pf_done = true;
        }
        s->pcv.notify_all();
    }
}
}  // namespace

extern "C" {

int ngdb_sampler_create(int32_t N, int32_t R, int64_t T, const int32_t* head, const int32_t* rel,
                        const int32_t* tail, const char* template_names, const float* weights, uint64_t seed,
                        int32_t n_threads, ngdb_sampler_t** out) {
    if (!out) return NGDB_ERR_ARG;
    *out = nullptr;
    if (N <= 0 || R <= 0 || T <= 0 || !head || !rel || !tail || !template_names || n_threads < 1 || n_threads > 256)
        return NGDB_ERR_ARG;
    for (int64_t i = 0; i < T; ++i)
        if (head[i] < 0 || head[i] >= N || tail[i] < 0 || tail[i] >= N || rel[i] < 0 || rel[i] >= R)
            return NGDB_ERR_RANGE;
    ngdb_sampler_t* s = new (std::nothrow) ngdb_sampler_s();
    if (!s) return NGDB_ERR_OOM;
    try {
        // templates: comma separated names
        std::string names(template_names), cur;
        names.push_back(',');
        for (char ch : names) {
            if (ch != ',') { cur.push_back(ch); continue; }
            if (cur.empty()) continue;
            const char* shape = shape_of(cur);
            if (!shape) { delete s; return NGDB_ERR_ARG; }
            Template tp;
            tp.name = cur;
            parse(shape, tp.nodes);
            s->templates.push_back(std::move(tp));
            cur.clear();
        }
        if (s->templates.empty()) { delete s; return NGDB_ERR_ARG; }
        double tot = 0.0;
        for (size_t i = 0; i < s->templates.size(); ++i) {
            const double w = weights ? (double)weights[i] : 1.0;
            if (!(w >= 0.0)) { delete s; return NGDB_ERR_ARG; }
            tot += w;
            s->cdf.push_back(tot);
        }
        if (!(tot > 0.0)) { delete s; return NGDB_ERR_ARG; }
        for (double& c : s->cdf) c /= tot;
        // adjacency by tail (in-edges) and by head (out-edges, sorted by relation and tail)
        Graph& g = s->g;
        g.N = N; g.R = R; g.T = T;
        g.tails.assign(tail, tail + T);
        g.in_off.assign((size_t)N + 1, 0);
        g.out_off.assign((size_t)N + 1, 0);
        for (int64_t i = 0; i < T; ++i) { ++g.in_off[tail[i] + 1]; ++g.out_off[head[i] + 1]; }
        for (int32_t v = 0; v < N; ++v) { g.in_off[v + 1] += g.in_off[v]; g.out_off[v + 1] += g.out_off[v]; }
        g.in_head.resize(T); g.in_rel.resize(T); g.out_rel.resize(T); g.out_tail.resize(T);
        std::vector<int64_t> in_fill(g.in_off.begin(), g.in_off.end() - 1), out_fill(g.out_off.begin(), g.out_off.end() - 1);
        for (int64_t i = 0; i < T; ++i) {
            const int64_t a = in_fill[tail[i]]++, b = out_fill[head[i]]++;
            g.in_head[a] = head[i]; g.in_rel[a] = rel[i];
            g.out_rel[b] = rel[i]; g.out_tail[b] = tail[i];
        }
        std::vector<std::pair<int32_t, int32_t>> tmp;
        for (int32_t v = 0; v < N; ++v) {
            const int64_t lo = g.out_off[v], hi = g.out_off[v + 1];
            tmp.resize((size_t)(hi - lo));
            for (int64_t j = lo; j < hi; ++j) tmp[(size_t)(j - lo)] = {g.out_rel[j], g.out_tail[j]};
            std::sort(tmp.begin(), tmp.end());
            for (int64_t j = lo; j < hi; ++j) { g.out_rel[j] = tmp[(size_t)(j - lo)].first; g.out_tail[j] = tmp[(size_t)(j - lo)].second; }
        }
    } catch (const std::bad_alloc&) {
        delete s;
        return NGDB_ERR_OOM;
    }
    s->seed = seed;
    s->n_threads = n_threads;
    try {
        if (n_threads > 1) s->workers.reset(new Workers(n_threads - 1));
        s->coordinator = std::thread(coordinator_loop, s);
    } catch (...) {
        delete s;
        return NGDB_ERR_OOM;
    }
    *out = s;
    return NGDB_OK;
}

void ngdb_sampler_destroy(ngdb_sampler_t* s) { delete s; }

extern "C++" {
namespace {
// draws batch number batch_no into o (the calling thread works beside the helpers)
int fill_batch(ngdb_sampler_s* s, uint64_t batch_no, int32_t B, int32_t K, BatchArrays& o) {
    std::vector<int> failed;
    try {
        if ((int)s->queries.size() < B) s->queries.resize((size_t)B);
        failed.assign((size_t)B, 0);
        o.pos.assign((size_t)B, 0);
        o.tmpl.assign((size_t)B, 0);
        o.neg.resize((size_t)B * K);
    } catch (const std::bad_alloc&) {
        return NGDB_ERR_OOM;
    }
    std::vector<Query>& queries = s->queries;
    auto work = [&](int lo, int hi) {
        for (int i = lo; i < hi; ++i) {
            Rng rng(s->seed, batch_no, (uint64_t)i);
            const double u = rng.unit();
            size_t t = 0;
            while (t + 1 < s->cdf.size() && u >= s->cdf[t]) ++t;
            o.tmpl[i] = (uint8_t)t;
            const Template& tp = s->templates[t];
            Query& q = queries[i];
            bool ok = false;
            for (int attempt = 0; attempt < 1000 && !ok; ++attempt) {
                q.clear();
                const int32_t v = s->g.tails[rng.below((uint64_t)s->g.T)];
                Builder b{s->g, tp, rng, q};
                if (b.grow((int)tp.nodes.size() - 1, v) < 0) continue;
                b.budget = 20000;
                if (b.contains((int)q.op.size() - 1, v) != 1) continue;   // e.g. the end point lies in a negated branch
                o.pos[i] = v;
                ok = true;
            }
            failed[i] = !ok;
            int32_t* nrow = o.neg.data() + (size_t)i * K;
            int k = 0;
            for (; k + 2 <= K; k += 2) rng.below32x2((uint32_t)s->g.N, nrow + k);
            if (k < K) nrow[k] = (int32_t)rng.below((uint64_t)s->g.N);
        }
    };
    const int parts = s->workers ? std::max(1, std::min(s->workers->size() + 1, B / 32 + 1)) : 1;
    if (parts == 1) {
        work(0, B);
    } else {
        const std::function<void(int)> fn = [&](int w) {      // helper w takes part w + 1
            if (w + 1 < parts) work((int)((int64_t)B * (w + 1) / parts), (int)((int64_t)B * (w + 2) / parts));
        };
        // the helpers run their parts while this thread does part 0
        s->workers->start(fn);
        bool oom = false;
        try {
            work(0, (int)((int64_t)B / parts));
        } catch (const std::bad_alloc&) {
            oom = true;
        }
        s->workers->wait();
        if (oom) return NGDB_ERR_OOM;
    }
    for (int i = 0; i < B; ++i)
        if (failed[i]) {
            s->err = "query instantiation kept failing for template " + s->templates[o.tmpl[i]].name;
            return NGDB_ERR_UNSUPPORTED;
        }
    // concatenate
    try {
        o.node_off.assign(1, 0);
        o.op.clear(); o.arg.clear(); o.in_idx.clear();
        o.in_off.assign(1, 0);
        for (int i = 0; i < B; ++i) {
            const Query& q = queries[i];
            o.op.insert(o.op.end(), q.op.begin(), q.op.end());
            o.arg.insert(o.arg.end(), q.arg.begin(), q.arg.end());
            const int32_t base = (int32_t)o.in_idx.size();
            o.in_idx.insert(o.in_idx.end(), q.in_idx.begin(), q.in_idx.end());
            for (size_t n = 1; n < q.in_off.size(); ++n) o.in_off.push_back(base + q.in_off[n]);
            o.node_off.push_back((int32_t)o.op.size());
        }
    } catch (const std::bad_alloc&) {
        return NGDB_ERR_OOM;
    }
    return NGDB_OK;
}
}  // namespace
}  // extern "C++"

int ngdb_sampler_next(ngdb_sampler_t* s, int32_t B, int32_t K, ngdb_query_batch* batch, const int32_t** neg,
                      const uint8_t** template_id) {
    if (!s || !batch || B < 0 || K < 0 || (K > 0 && !neg)) return NGDB_ERR_ARG;
    const uint64_t batch_no = s->batch_no++;
    BatchArrays& o = s->out[batch_no % 3];
    int rc;
    bool ready = false;
    {   // a batch read ahead by the coordinator?
        std::unique_lock<std::mutex> lk(s->pm);
        if (s->pf_requested) {
            s->pcv.wait(lk, [&] { return s->pf_done; });
            ready = s->pf_no == batch_no && s->pf_B == B && s->pf_K == K;
            rc = s->pf_rc;
            s->pf_requested = s->pf_done = false;
        }
    }
    if (!ready) rc = fill_batch(s, batch_no, B, K, o);     // first call, or other sizes than read ahead
    if (rc != NGDB_OK) return rc;
    if (s->coordinator.joinable()) {   // read ahead: the next batch with the same sizes
        {
            std::lock_guard<std::mutex> lk(s->pm);
            s->pf_no = batch_no + 1; s->pf_B = B; s->pf_K = K;
            s->pf_requested = true; s->pf_done = false;
        }
        s->pcv.notify_all();
    }
    batch->n_queries = B;
    batch->node_off = o.node_off.data();
    batch->op = o.op.data();
    batch->arg = o.arg.data();
    batch->in_off = o.in_off.data();
    batch->in_idx = o.in_idx.data();
    batch->pos = o.pos.data();
    if (neg) *neg = o.neg.data();
    if (template_id) *template_id = o.tmpl.data();
    return NGDB_OK;
}

const char* ngdb_sampler_last_error(const ngdb_sampler_t* s) { return s ? s->err.c_str() : ""; }

}  // extern "C"
