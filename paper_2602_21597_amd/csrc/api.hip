// C boundary and step orchestration: enqueues, per depth of the batch's operator
// DAG, one grouped launch sequence per operator type (Sec. 4.1 "Batched
// Execution"; Sec. 4.3 cardinality classes), then scoring, the reversed
// frontiers (Alg. 1: gradient nodes are scheduled like forward ones), the
// segmented table updates and Adam (Alg. 1, OptimizerStep).
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "common.h"
#include "planner.h"

using namespace ngdb;

static __device__ __align__(256) unsigned char scratch[(size_t)NGDB_NOALLOC_SCRATCH_MIB << 20];

namespace {

struct DevBuf {
    void* p = nullptr;
    size_t cap = 0;
};

struct Segment {   // the groups of one (level, type): contiguous MLP rows and references
    int type = 0;
    int rows = 0;          // MLP rows (members for PROJ/NEG, members*inputs for INTER)
    int mlp_base = 0;
    int ref_off = 0;
    int rel_off = -1;
    int out_base = 0;      // PROJ/NEG: first output slot
    int g_lo = 0, g_hi = 0;  // group range (INTER: one combine launch per group)
};

constexpr int T_PROJ = 0, T_INTER = 1, T_NEG = 2;
inline int type_index(int op) { return op == NGDB_OP_PROJ ? T_PROJ : (op == NGDB_OP_INTER ? T_INTER : T_NEG); }

}  // namespace

// Device copy of a plan's arrays plus its pinned staging buffer; recycled through
// the context so that planning allocates nothing in steady state.
struct PlanBlob {
    int32_t* dev = nullptr;
    int32_t* pinned = nullptr;
    size_t cap = 0;               // in int32 elements
    hipEvent_t last_use = nullptr;  // recorded after every step that read the blob
};

struct ngdb_plan_s {
    HostPlan hp;
    ngdb_ctx_t* owner = nullptr;
    PlanBlob blob;
    int32_t* d_blob = nullptr;
    // device views into the blob
    const int32_t *d_in_ref = nullptr, *d_in_gslot = nullptr, *d_rel = nullptr, *d_root_off = nullptr,
                  *d_root_slot = nullptr, *d_pos = nullptr, *d_ekeys_head = nullptr, *d_r_uniq = nullptr,
                  *d_r_seg_off = nullptr, *d_r_src = nullptr, *d_r_rec = nullptr, *d_n_r_uniq = nullptr;
    // forward-only passes with reclaimed outputs: references, output rows and root rows in storage rows
    const int32_t *d_f_in_ref = nullptr, *d_f_row = nullptr, *d_f_root = nullptr;
    std::vector<std::vector<Segment>> levels;   // levels[l] for l = 1..n_levels (index 0 unused)
    int32_t n_entities = 0;
};

struct ngdb_ctx_s {
    ngdb_config cfg{};
    ngdb_params prm{};
    bool bound = false;
    bool presized = false;          // workspace allocated once from declared maxima: steps must not grow it
    int64_t n_alloc = 0;            // device / pinned allocations made so far
    int64_t step = 0;
    std::string err;
    hipStream_t side[1]{};          // library stream (num_streams > 1)
    hipEvent_t ev_fork = nullptr;
    hipEvent_t ev_join = nullptr;
    int n_side = 0;
    // workspace
    DevBuf act, dact, Z[3], H[3], dH[3], Att, dAtt, Dx;
    DevBuf score, coef, win, mask, loss_terms, rec_coef, rec_row;
    DevBuf keys_a, keys_b, vals_a, vals_b, hist, scan_tmp, uniq, seg_off, n_uniq;
    DevBuf rank_dist;   // distances of one entity chunk in the all-entity ranking
    DevBuf rank_thr, rank_count;   // filtered ranks: distance of every listed answer, entities closer than it
    DevBuf colsum_part; // 6 scratch areas of the bias-gradient column sums
    DevBuf gW;          // gradients of the 12 MLP tensors, packed
    // The six weight matrices of the vector family's MLPs as ready-made B operands of the contraction
    // kernel (bf16 pieces in MFMA lane order), in both orientations: rebuilt at the start of every
    // forward pass, so they are never older than the weights the pass reads.
    DevBuf w_pieces;
    const uint16_t* wp[3][4]{};     // per type: Wa forward, Wb forward, Wb backward (dH = dY Wb), Wa backward (dZ = dH Wa)
    bool have_pieces = false;
    // The hidden activations of one depth (forward) or their gradients (backward) once more as bf16
    // pieces in tile order: written by the first launch of a layer pair, read as A operand by the
    // second, then free again.  Only steps whose launches use the small tile get that far.
    DevBuf h_pieces;
    DevBuf gE, gR;      // compact table gradients (ngdb_forward_backward only)
    // text-feature fusion: bf16 copy of Wp, fused rows of the touched entities, position of every
    // contribution's entity in that list, operator references redirected to it, bf16 row gradients,
    // split-wise partial sums and the gradient of Wp, fused rows of one ranking chunk
    DevBuf Wb, Ef, inv, refs_sem, g_bf16, wp_partial, gWp, rank_ef;
    // box family: offsets and their gradients by slot (act / dact hold the centres), per-input
    // outputs of the offset MLP with their gradients, direct gradient of the inputs' offsets,
    // compact gradient of Ro.  The offset MLP (V1 c1 V2 c2) uses the Z/H/dH buffers of index T_NEG.
    DevBuf off, doff, Gate, dGate, DxO, gRo;
    DevBuf Eb;          // bf16 copy of E for the scoring and ranking passes (score_bf16)
    size_t gw_off[13]{};
    hipStream_t upload = nullptr;        // plan uploads, independent of the compute streams
    std::vector<PlanBlob> blob_pool;
    std::vector<ngdb_plan_t*> live_plans;   // plans that hold a device buffer of this context
    std::mutex mu;                       // guards blob_pool, live_plans and err: planning may run on a second host thread
    // kernel timing
    uint32_t timing_mask = 0;
    struct Bracket { int cls; hipEvent_t a, b; int route; double flop; };
    std::vector<Bracket> brackets;
    std::vector<hipEvent_t> spare_events;
    ngdb_timing timing{};
    // results of the last step
    bool have_grads = false;
    ngdb_grad_view gv{};
};

namespace {

thread_local std::string g_create_err;

// Scratch of ngdb_score_noalloc: device memory that exists from the moment the library's code
// object is loaded on a GPU until the process ends, one copy per GPU.  In host code the array's
// name only stands for the symbol; its device address on a GPU is asked for once per device
// (noalloc_scratch) and only that address is ever passed to kernels.
constexpr size_t NOALLOC_BYTES = (size_t)NGDB_NOALLOC_SCRATCH_MIB << 20;
constexpr int NOALLOC_MAX_DEVICES = 64;
std::mutex g_scratch_mu;
unsigned char* g_scratch_ptr[NOALLOC_MAX_DEVICES] = {};

int fail(ngdb_ctx_t* c, int code, const std::string& msg) {
    if (c) {
        std::lock_guard<std::mutex> lk(c->mu);
        c->err = msg;
    }
    return code;
}

#define HIPCHK(c, expr)                                                                        \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess)                                                                  \
            return fail((c), e_ == hipErrorOutOfMemory ? NGDB_ERR_OOM : NGDB_ERR_HIP,          \
                        std::string(#expr) + ": " + hipGetErrorString(e_));                    \
    } while (0)

hipEvent_t take_event(ngdb_ctx_t* c) {
    if (!c->spare_events.empty()) {
        hipEvent_t e = c->spare_events.back();
        c->spare_events.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    return hipEventCreate(&e) == hipSuccess ? e : nullptr;
}

// Brackets one launch (sequence) with an event pair when its class is being timed.
struct Timed {
    ngdb_ctx_t* c;
    hipStream_t s;
    hipEvent_t b = nullptr;
    Timed(ngdb_ctx_t* ctx, int cls, hipStream_t stream) : c(ctx), s(stream) {
        if (!(c->timing_mask >> cls & 1u)) return;
        hipEvent_t a = take_event(c);
        b = take_event(c);
        if (!a || !b) { b = nullptr; return; }
        (void)hipEventRecord(a, s);
        c->brackets.push_back({cls, a, b, -1, 0.0});
    }
    // a contraction launch: the instructions it ran on and its algorithmic work
    void work(int route, double flop) {
        if (!b) return;
        c->brackets.back().route = route == GEMM_SPLIT ? 1 : 0;
        c->brackets.back().flop = flop;
    }
    ~Timed() { if (b) (void)hipEventRecord(b, s); }
};

// One grouped contraction launch, bracketed as class `cls`.
int gemm_timed(ngdb_ctx_t* c, int cls, const GemmArgs* g, int n, hipStream_t s, bool* emitted = nullptr);

// evaluation: a buffer only the ranking calls or ngdb_forward_backward use (allocated on first use
// also under declared maxima)
int ensure(ngdb_ctx_t* c, DevBuf& b, size_t bytes, bool evaluation = false) {
    if (bytes <= b.cap) return NGDB_OK;
    if (c->presized && !evaluation)
        return fail(c, NGDB_ERR_ARG, "the batch needs more workspace than the maxima declared at ngdb_create allow "
                                     "(b_max_queries, k_max, max_nodes_per_query)");
    // growing: nothing may still be using the old allocation
    HIPCHK(c, hipDeviceSynchronize());
    if (b.p) HIPCHK(c, hipFree(b.p));
    b.p = nullptr;
    b.cap = 0;
    const size_t want = bytes + bytes / 4 + 256;
    HIPCHK(c, hipMalloc(&b.p, want));
    ++c->n_alloc;
    b.cap = want;
    return NGDB_OK;
}

void release(DevBuf& b) {
    if (b.p) (void)hipFree(b.p);
    b.p = nullptr;
    b.cap = 0;
}

template <class T>
T* ptr(const DevBuf& b) { return static_cast<T*>(b.p); }

int gemm_timed(ngdb_ctx_t* c, int cls, const GemmArgs* g, int n, hipStream_t s, bool* emitted) {
    Timed tm(c, cls, s);
    int route = GEMM_FP32;
    HIPCHK(c, launch_gemm_group(g, n, s, &route, emitted));
    double flop = 0.0;
    for (int i = 0; i < n; ++i)
        if (g[i].M > 0 && g[i].N > 0) flop += 2.0 * g[i].M * g[i].N * g[i].K;
    tm.work(route, flop);
    return NGDB_OK;
}

struct MlpRefs {
    const float *Wa, *ba, *Wb, *bb;
};
MlpRefs mlp_of(const ngdb_params& p, int t) {
    if (t == T_PROJ) return {p.W1.p, p.b1.p, p.W2.p, p.b2.p};
    if (t == T_NEG) return {p.V1.p, p.c1.p, p.V2.p, p.c2.p};
    return {p.U1.p, p.u1.p, p.U2.p, p.u2.p};
}
// order of ngdb_grad_view::g_mlp: W1 b1 W2 b2 | V1 c1 V2 c2 | U1 u1 U2 u2
int gslot_of(int t) { return t == T_PROJ ? 0 : (t == T_NEG ? 4 : 8); }

struct FwdBytes;
FwdBytes forward_bytes(const ngdb_ctx_t* c, const ngdb_plan_t* pl, bool reclaim);
int size_forward_only(ngdb_ctx_t* c, const ngdb_plan_t* pl, int64_t n_tail);


// bytes of the split weights: per type two operands of ceil(h/32) x ceil(d/16) tiles and two of ceil(d/32) x ceil(h/16)
size_t weight_pieces_bytes(const ngdb_ctx_t* c) {
    if (c->cfg.family != NGDB_FAMILY_VEC) return 0;
    return 3 * 2 * (pieces_elems(c->cfg.h, c->cfg.d) + pieces_elems(c->cfg.d, c->cfg.h)) * sizeof(uint16_t);
}
// Room for the hidden rows of one depth as pieces: blocks of 32 rows per segment, k-tiles in pairs.
constexpr size_t H_PIECES_MAX_ROWS = 2048;      // launches over more rows do not write pieces
int h_pieces_kt(const ngdb_ctx_t* c) { return 2 * ((c->cfg.h + 31) / 32); }
size_t h_pieces_bytes(const ngdb_ctx_t* c, const HostPlan& hp) {
    if (c->cfg.family != NGDB_FAMILY_VEC) return 0;
    const size_t rows = std::min<size_t>((size_t)hp.n_proj + hp.n_int_rows + hp.n_neg, H_PIECES_MAX_ROWS);
    return (rows / 32 + 3) * h_pieces_kt(c) * 1536 * sizeof(uint16_t);
}
// Hands the segments of one depth their places in h_pieces (as output of `first`, as A operand of
// `second` once the launch of `first` reports that it wrote them).
struct HiddenPieces {
    uint16_t* at[3] = {};
    int kt = 0;
};
HiddenPieces place_hidden_pieces(ngdb_ctx_t* c, GemmArgs* first, int n) {
    HiddenPieces hpc;
    if (!c->have_pieces || !c->h_pieces.p) return hpc;
    hpc.kt = h_pieces_kt(c);
    const size_t tile_row = (size_t)hpc.kt * 1536;
    size_t blocks = 0;
    for (int i = 0; i < n; ++i) blocks += (size_t)(first[i].M + 31) / 32;
    if (blocks * tile_row * sizeof(uint16_t) > c->h_pieces.cap) return hpc;
    uint16_t* at = ptr<uint16_t>(c->h_pieces);
    for (int i = 0; i < n; ++i) {
        hpc.at[i] = first[i].c_pieces = at;
        first[i].c_kt = hpc.kt;
        at += (size_t)((first[i].M + 31) / 32) * tile_row;
    }
    return hpc;
}
void take_hidden_pieces(const HiddenPieces& hpc, GemmArgs* second, int n) {
    for (int i = 0; i < n; ++i) { second[i].a_pieces = hpc.at[i]; second[i].a_kt = hpc.kt; }
}

// Splits the weights of the three MLPs for this pass (one launch).  Without the buffer (a context
// that never sized a workspace) the contractions split their B operands themselves.
int make_weight_pieces(ngdb_ctx_t* c, hipStream_t s) {
    c->have_pieces = false;
    if (c->cfg.family != NGDB_FAMILY_VEC || c->w_pieces.cap < weight_pieces_bytes(c) || !c->w_pieces.p) return NGDB_OK;
    const int d = c->cfg.d, h = c->cfg.h;
    if ((d & 3) || (h & 3)) return NGDB_OK;   // the split reads rows as float4
    uint16_t* at = ptr<uint16_t>(c->w_pieces);
    PieceJobs J{};
    for (int t = 0; t < 3; ++t) {
        const MlpRefs W = mlp_of(c->prm, t);
        // Wa [h][d]: rows as n = forward operand of H = X Wa^T; columns as n = backward operand of dZ = dH Wa
        PieceJob& ja = J.job[J.count++];
        ja.W = W.Wa; ja.R = h; ja.C = d;
        c->wp[t][0] = ja.out_rk = at; at += pieces_elems(h, d);
        c->wp[t][3] = ja.out_ck = at; at += pieces_elems(d, h);
        // Wb [d][h]: rows as n = forward operand of Y = H Wb^T; columns as n = backward operand of dH = dY Wb
        PieceJob& jw = J.job[J.count++];
        jw.W = W.Wb; jw.R = d; jw.C = h;
        c->wp[t][1] = jw.out_rk = at; at += pieces_elems(d, h);
        c->wp[t][2] = jw.out_ck = at; at += pieces_elems(h, d);
    }
    HIPCHK(c, launch_weight_pieces(J, s));
    c->have_pieces = true;
    return NGDB_OK;
}

int size_workspace(ngdb_ctx_t* c, const ngdb_plan_t* pl, int K, bool want_table_grads) {
    const HostPlan& hp = pl->hp;
    const size_t d = c->cfg.d, h = c->cfg.h, f = sizeof(float);
    const size_t rows[3] = {(size_t)hp.n_proj, (size_t)hp.n_int_rows, (size_t)hp.n_neg};
    int rc;
#define ENS(buf, bytes) if ((rc = ensure(c, buf, std::max<size_t>((bytes), 256))) != NGDB_OK) return rc
    ENS(c->w_pieces, weight_pieces_bytes(c));
    ENS(c->h_pieces, h_pieces_bytes(c, hp));
    ENS(c->act, (size_t)hp.n_slots * d * f);
    ENS(c->dact, ((size_t)hp.n_slots + hp.n_anchor) * d * f);
    for (int t = 0; t < 3; ++t) {
        ENS(c->Z[t], rows[t] * d * f);
        ENS(c->H[t], rows[t] * h * f);
        ENS(c->dH[t], rows[t] * h * f);
    }
    const bool box = c->cfg.family == NGDB_FAMILY_BOX;
    if (box) {
        ENS(c->off, (size_t)hp.n_slots * d * f);
        ENS(c->doff, ((size_t)hp.n_slots + hp.n_anchor) * d * f);
        ENS(c->Z[T_NEG], rows[T_INTER] * d * f);
        ENS(c->H[T_NEG], rows[T_INTER] * h * f);
        ENS(c->dH[T_NEG], rows[T_INTER] * h * f);
        ENS(c->Gate, rows[T_INTER] * d * f);
        ENS(c->dGate, rows[T_INTER] * d * f);
        ENS(c->DxO, rows[T_INTER] * d * f);
    }
    ENS(c->Att, rows[T_INTER] * d * f);
    ENS(c->dAtt, rows[T_INTER] * d * f);
    ENS(c->Dx, rows[T_INTER] * d * f);
    const size_t pairs = (size_t)hp.n_queries * ((size_t)K + 1);
    ENS(c->score, pairs * f);
    ENS(c->coef, pairs * f);
    if (c->cfg.d_sem > 0) {
        ENS(c->mask, pairs * 64 * (d <= 256 ? 1 : (d <= 512 ? 2 : 4)));   // sign codes, per pair and lane
    } else {
        ENS(c->win, pairs * sizeof(int32_t));
    }
    ENS(c->loss_terms, (size_t)hp.n_queries * f);
    ENS(c->rec_coef, ((size_t)hp.n_anchor + pairs) * f);
    ENS(c->rec_row, ((size_t)hp.n_anchor + pairs) * sizeof(int32_t));
    const int64_t nk = (int64_t)hp.n_anchor + hp.n_queries + (int64_t)hp.n_queries * K;
    ENS(c->keys_a, (size_t)nk * 4);
    ENS(c->keys_b, (size_t)nk * 4);
    ENS(c->vals_a, (size_t)nk * 4);
    ENS(c->vals_b, (size_t)nk * 4);
    ENS(c->uniq, (size_t)nk * 4);
    ENS(c->seg_off, ((size_t)nk + 1) * 4);
    ENS(c->hist, index_hist_elems(nk) * 4);
    ENS(c->scan_tmp, index_scan_tmp_elems(nk) * 4);
    ENS(c->n_uniq, 256);
    ENS(c->colsum_part, 6 * (size_t)COLSUM_MAX_CHUNKS * std::max(d, h) * f);
    if (!c->gW.p) {
        size_t off = 0;
        for (int t = 0; t < 3; ++t) {
            const size_t sz[4] = {h * d, h, d * h, d};
            for (int k = 0; k < 4; ++k) {
                c->gw_off[t * 4 + k] = off;
                off += (sz[k] + 3) & ~size_t(3);
            }
        }
        c->gw_off[12] = off;
        ENS(c->gW, off * f);
    }
    if (c->cfg.d_sem > 0) {
        const size_t ds = c->cfg.d_sem;
        const size_t urows = (size_t)std::min<int64_t>(nk, c->cfg.n_entities);
        ENS(c->Wb, d * ds * sizeof(uint16_t));
        ENS(c->Ef, urows * d * f);
        ENS(c->inv, (size_t)nk * 4);
        ENS(c->refs_sem, hp.in_ref.size() * 4);
        ENS(c->g_bf16, urows * d * sizeof(uint16_t));
        ENS(c->wp_partial, (size_t)sem_wgrad_splits((int64_t)urows, (int)d, (int)ds) * d * ds * f);
        ENS(c->gWp, d * ds * f);
    }
    if (want_table_grads) {
        const size_t urows = (size_t)std::min<int64_t>(nk, c->cfg.n_entities);
        if ((rc = ensure(c, c->gE, urows * d * f, true)) != NGDB_OK) return rc;
        if ((rc = ensure(c, c->gR, (size_t)std::max<size_t>(hp.r_uniq.size(), 1) * d * f, true)) != NGDB_OK) return rc;
        if (box && (rc = ensure(c, c->gRo, (size_t)std::max<size_t>(hp.r_uniq.size(), 1) * d * f, true)) != NGDB_OK) return rc;
    }
#undef ENS
    return NGDB_OK;
}

// Where the entity rows of one call come from: the table itself, or (text-feature fusion) the
// fused rows of the touched entities, addressed by position in that list.
struct EntRows {
    const float* rows;
    const int32_t* refs;   // operator input references (anchors as -1-row)
    const int32_t* pos;    // [B] row of every query's positive
    const int32_t* cand;   // [B, C] rows of the candidates
};

// Builds the index over [anchors | positives | tail] and, with text features, the fused rows
// of its distinct entities and the references into them.  The index is left in the context's
// buffers; *e_src receives the sorted contribution numbers.
int prepare_entities(ngdb_ctx_t* c, const ngdb_plan_t* pl, const int32_t* d_tail, int64_t n_tail, hipStream_t s_idx,
                     hipStream_t stream, int32_t** e_src, EntRows* er, bool reclaim = false) {
    const HostPlan& hp = pl->hp;
    const int B = hp.n_queries, d = c->cfg.d, ds = c->cfg.d_sem;
    IndexBuffers ib{ptr<int32_t>(c->keys_a), ptr<int32_t>(c->keys_b), ptr<int32_t>(c->vals_a),
                    ptr<int32_t>(c->vals_b), ptr<int32_t>(c->hist),   ptr<int32_t>(c->scan_tmp),
                    ptr<int32_t>(c->uniq),   ptr<int32_t>(c->seg_off), ptr<int32_t>(c->n_uniq)};
    {
        Timed tm(c, NGDB_TK_INDEX, s_idx);
        HIPCHK(c, build_segment_index(pl->d_ekeys_head, hp.n_anchor + B, d_tail, n_tail, c->cfg.n_entities, ib, e_src,
                                      s_idx));
    }
    if (ds == 0) {
        *er = EntRows{c->prm.E.p, reclaim ? pl->d_f_in_ref : pl->d_in_ref, pl->d_pos, d_tail};
        return NGDB_OK;
    }
    // s_idx == stream in this mode: everything below needs the index
    const int64_t n_contrib = (int64_t)hp.n_anchor + B + n_tail;
    Timed tm(c, NGDB_TK_SEM, stream);
    HIPCHK(c, launch_cast_bf16(c->prm.Wp.p, ptr<uint16_t>(c->Wb), (int64_t)d * ds, stream));
    HIPCHK(c, launch_inverse_index(*e_src, ptr<int32_t>(c->seg_off), ptr<int32_t>(c->n_uniq), n_contrib,
                                   ptr<int32_t>(c->inv), stream));
    SemFuseArgs fa{};
    fa.H = c->prm.H_sem; fa.Wb = ptr<uint16_t>(c->Wb); fa.E = c->prm.E.p; fa.ids = ptr<int32_t>(c->uniq);
    fa.n_rows_dev = ptr<int32_t>(c->n_uniq); fa.n_rows = (int)std::min<int64_t>(n_contrib, c->cfg.n_entities);
    fa.d = d; fa.ds = ds; fa.out = ptr<float>(c->Ef);
    HIPCHK(c, launch_sem_fuse(fa, stream));
    HIPCHK(c, launch_translate_refs(reclaim ? pl->d_f_in_ref : pl->d_in_ref, pl->d_in_gslot, (int)hp.in_ref.size(), hp.n_slots,
                                    ptr<int32_t>(c->inv), ptr<int32_t>(c->refs_sem), stream));
    *er = EntRows{ptr<float>(c->Ef), ptr<int32_t>(c->refs_sem), ptr<int32_t>(c->inv) + hp.n_anchor,
                  ptr<int32_t>(c->inv) + hp.n_anchor + B};
    return NGDB_OK;
}

// The intersections of one segment as jobs of the pooling kernels: centres (box == false:
// X = Z[T_INTER], logits Att) or offsets of the box family (X = Z[T_NEG], MLP outputs Gate).
// With `pool` the jobs are appended to it and the offset jobs flagged (both kinds in one launch).
int inter_jobs(ngdb_ctx_t* c, const ngdb_plan_t* pl, const Segment& sg, bool offsets, bool backward, InterJobs* ij,
               BoxPoolJobs* pool = nullptr) {
    const HostPlan& hp = pl->hp;
    const int d = c->cfg.d;
    if (pool) ij = &pool->jobs;
    else *ij = InterJobs{};
    ij->d = d;
    for (int g = sg.g_lo; g < sg.g_hi; ++g) {
        const size_t mb = (size_t)hp.g_mlp_base[g] * d, ob = (size_t)hp.g_out_base[g] * d;
        if (ij->count == INTER_MAX_JOBS) return fail(c, NGDB_ERR_UNSUPPORTED, "too many intersection classes in one level");
        InterJob& jb = ij->job[ij->count++];
        jb.X = ptr<float>(c->Z[offsets ? T_NEG : T_INTER]) + mb;
        jb.Att = ptr<float>(offsets ? c->Gate : c->Att) + mb;
        jb.n = hp.g_n[g]; jb.k = hp.g_nin[g];
        if (pool && offsets) pool->gate_mask |= 1u << (ij->count - 1);
        if (!backward) {
            jb.out = ptr<float>(offsets ? c->off : c->act) + ob;
        } else {
            jb.dY = ptr<float>(offsets ? c->doff : c->dact) + ob;
            jb.dAtt = ptr<float>(offsets ? c->dGate : c->dAtt) + mb;
            jb.Dx = ptr<float>(offsets ? c->DxO : c->Dx) + mb;
        }
    }
    return NGDB_OK;
}

BoxProjArgs box_proj_args(ngdb_ctx_t* c, const ngdb_plan_t* pl, const Segment& sg) {
    BoxProjArgs a{};
    a.ref = pl->d_in_ref + sg.ref_off; a.gslot = pl->d_in_gslot + sg.ref_off; a.rel = pl->d_rel + sg.rel_off;
    a.E = c->prm.E.p; a.Rc = c->prm.R.p; a.Ro = c->prm.Ro.p;
    a.act_c = ptr<float>(c->act); a.act_o = ptr<float>(c->off);
    a.dact_c = ptr<float>(c->dact); a.dact_o = ptr<float>(c->doff);
    a.n = sg.rows; a.d = c->cfg.d; a.out_base = sg.out_base;
    return a;
}

// The projection group of a level that can ride in the level's pooling launch (they are
// independent of each other): the first one, if an intersection segment with few enough
// cardinality classes for the joint launch exists.
const Segment* riding_projection(const std::vector<Segment>& segs) {
    const Segment* proj = nullptr;
    bool joint = false;
    for (const Segment& sg : segs) {
        if (sg.type == T_PROJ && !proj) proj = &sg;
        if (sg.type == T_INTER && 2 * (sg.g_hi - sg.g_lo) <= INTER_MAX_JOBS) joint = true;
    }
    return joint ? proj : nullptr;
}

// Box family, forward: projections are one elementwise launch per group; an intersection runs two
// MLPs over its inputs (attention logits from the centres, gate inputs from the offsets), grouped
// into one launch per layer, then the two pooling kernels.
int enqueue_forward_box(ngdb_ctx_t* c, const ngdb_plan_t* pl, hipStream_t s) {
    const int d = c->cfg.d, h = c->cfg.h;
    for (int l = 1; l <= pl->hp.n_levels; ++l) {
        const std::vector<Segment>& segs = pl->levels[l];
        GemmArgs g1[GEMM_MAX_GROUP], g2[GEMM_MAX_GROUP];
        int n = 0;
        const Segment* ride = riding_projection(segs);
        for (const Segment& sg : segs) {
            if (sg.type == T_PROJ) {
                if (&sg == ride) continue;
                Timed tm(c, NGDB_TK_INTER, s);
                HIPCHK(c, launch_box_proj(box_proj_args(c, pl, sg), false, s));
                continue;
            }
            if (sg.type != T_INTER || n + 2 > GEMM_MAX_GROUP) return fail(c, NGDB_ERR_UNSUPPORTED, "operator not available in the box family");
            for (int part = 0; part < 2; ++part) {
                const int t = part ? T_NEG : T_INTER;
                const MlpRefs W = mlp_of(c->prm, t);
                float* Hh = ptr<float>(c->H[t]) + (size_t)sg.mlp_base * h;
                GemmArgs& a = g1[n];
                a.a_ref = pl->d_in_ref + sg.ref_off; a.a_base0 = ptr<float>(part ? c->off : c->act);
                a.a_base1 = c->prm.E.p;       // never taken: the plan holds no anchor below an intersection
                a.a_copy = ptr<float>(c->Z[t]) + (size_t)sg.mlp_base * d; a.lda = d; a.B = W.Wa; a.ldb = d;
                a.C = Hh; a.ldc = h; a.M = sg.rows; a.N = h; a.K = d; a.bias = W.ba; a.relu = true;
                GemmArgs& b = g2[n];
                b.A = Hh; b.lda = h; b.B = W.Wb; b.ldb = h; b.M = sg.rows; b.N = d; b.K = h; b.bias = W.bb; b.ldc = d;
                b.C = ptr<float>(part ? c->Gate : c->Att) + (size_t)sg.mlp_base * d;
                ++n;
            }
        }
        if (n == 0) continue;
        int rc_g;
        if ((rc_g = gemm_timed(c, NGDB_TK_GEMM_FWD, g1, n, s)) != NGDB_OK) return rc_g;
        if ((rc_g = gemm_timed(c, NGDB_TK_GEMM_FWD, g2, n, s)) != NGDB_OK) return rc_g;
        for (const Segment& sg : segs) {
            if (sg.type != T_INTER) continue;
            Timed tm(c, NGDB_TK_INTER, s);
            InterJobs ij;
            int rc;
            if (2 * (sg.g_hi - sg.g_lo) <= INTER_MAX_JOBS) {     // centre and offset jobs fit one launch
                BoxPoolJobs pool{};
                if ((rc = inter_jobs(c, pl, sg, false, false, nullptr, &pool)) != NGDB_OK) return rc;
                if ((rc = inter_jobs(c, pl, sg, true, false, nullptr, &pool)) != NGDB_OK) return rc;
                if (ride) { pool.has_proj = 1; pool.proj = box_proj_args(c, pl, *ride); ride = nullptr; }
                HIPCHK(c, launch_box_pool(pool, false, s));
                continue;
            }
            if ((rc = inter_jobs(c, pl, sg, false, false, &ij)) != NGDB_OK) return rc;
            HIPCHK(c, launch_inter(ij, false, s));
            if ((rc = inter_jobs(c, pl, sg, true, false, &ij)) != NGDB_OK) return rc;
            HIPCHK(c, launch_box_offset(ij, false, s));
        }
    }
    return NGDB_OK;
}

// Device memory the forward pass of the vector family writes: operator outputs by slot, and per
// type the gathered first-layer inputs, the hidden rows and (intersections) the logits.
// reclaim (forward-only passes, Sec. 4.3 eager reference counting): an output is kept only until
// its consumer has run -- act holds n_f_rows storage rows addressed through the plan's f_row map,
// and Z / H / Att hold the rows of one step at a time (sizes: forward_bytes).
struct FwdSpace {
    float* act;
    float* Z[3];
    float* H[3];
    float* Att;
    bool reclaim;
};
FwdSpace ctx_space(const ngdb_ctx_t* c, bool reclaim = false) {
    return FwdSpace{ptr<float>(c->act), {ptr<float>(c->Z[0]), ptr<float>(c->Z[1]), ptr<float>(c->Z[2])},
                    {ptr<float>(c->H[0]), ptr<float>(c->H[1]), ptr<float>(c->H[2])}, ptr<float>(c->Att), reclaim};
}
// Bytes of the buffers of a forward-only pass, in the order act, Att, then Z and H per type.
struct FwdBytes { size_t act, att, z[3], h[3]; };
FwdBytes forward_bytes(const ngdb_ctx_t* c, const ngdb_plan_t* pl, bool reclaim) {
    const HostPlan& hp = pl->hp;
    const size_t d = c->cfg.d, h = c->cfg.h, f = sizeof(float);
    const size_t all[3] = {(size_t)hp.n_proj, (size_t)hp.n_int_rows, (size_t)hp.n_neg};
    FwdBytes b{};
    b.act = (size_t)(reclaim ? hp.n_f_rows : hp.n_slots) * d * f;
    for (int t = 0; t < 3; ++t) {
        const size_t rows = reclaim ? (size_t)hp.f_step_rows[t] : all[t];
        b.z[t] = rows * d * f;
        b.h[t] = rows * h * f;
        if (t == T_INTER) b.att = rows * d * f;
    }
    return b;
}

// Workspace of a forward-only pass of the vector family: the activation buffers at their
// reclaimed sizes; with text features also the index over [anchors | tail] and the fused rows.
int size_forward_only(ngdb_ctx_t* c, const ngdb_plan_t* pl, int64_t n_tail) {
    const HostPlan& hp = pl->hp;
    const FwdBytes fb = forward_bytes(c, pl, true);
    int rc;
#define ENS(buf, bytes) if ((rc = ensure(c, buf, std::max<size_t>((bytes), 256))) != NGDB_OK) return rc
    ENS(c->w_pieces, weight_pieces_bytes(c));
    ENS(c->h_pieces, h_pieces_bytes(c, hp));
    ENS(c->act, fb.act);
    ENS(c->Att, fb.att);
    for (int t = 0; t < 3; ++t) {
        ENS(c->Z[t], fb.z[t]);
        ENS(c->H[t], fb.h[t]);
    }
    if (c->cfg.d_sem > 0) {
        const size_t d = c->cfg.d, ds = c->cfg.d_sem;
        const int64_t nk = (int64_t)hp.n_anchor + hp.n_queries + n_tail;
        const size_t urows = (size_t)std::min<int64_t>(nk, c->cfg.n_entities);
        ENS(c->keys_a, (size_t)nk * 4);
        ENS(c->keys_b, (size_t)nk * 4);
        ENS(c->vals_a, (size_t)nk * 4);
        ENS(c->vals_b, (size_t)nk * 4);
        ENS(c->uniq, (size_t)nk * 4);
        ENS(c->seg_off, ((size_t)nk + 1) * 4);
        ENS(c->hist, index_hist_elems(nk) * 4);
        ENS(c->scan_tmp, index_scan_tmp_elems(nk) * 4);
        ENS(c->n_uniq, 256);
        ENS(c->Wb, d * ds * sizeof(uint16_t));
        ENS(c->Ef, urows * d * sizeof(float));
        ENS(c->inv, (size_t)nk * 4);
        ENS(c->refs_sem, hp.in_ref.size() * 4);
    }
#undef ENS
    return NGDB_OK;
}

// forward over the plan's frontiers; results in w.act.  The type segments of one
// depth are independent: they share one grouped launch per MLP layer.
int enqueue_forward(ngdb_ctx_t* c, const ngdb_plan_t* pl, const EntRows& er, hipStream_t s, const FwdSpace& w) {
    if (c->cfg.family == NGDB_FAMILY_BOX) return enqueue_forward_box(c, pl, s);   // (always on the context's buffers)
    const int d = c->cfg.d, h = c->cfg.h;
    {
        Timed tm(c, NGDB_TK_GEMM_FWD, s);
        int rc_p = make_weight_pieces(c, s);
        if (rc_p != NGDB_OK) return rc_p;
    }
    for (int l = 1; l <= pl->hp.n_levels; ++l) {
        const std::vector<Segment>& segs = pl->levels[l];
        GemmArgs g1[3], g2[3];
        int n = 0;
        for (const Segment& sg : segs) {
            const MlpRefs W = mlp_of(c->prm, sg.type);
            // (with reclaimed outputs the per-type buffers hold this step's rows only)
            const size_t row0 = w.reclaim ? 0 : (size_t)sg.mlp_base;
            float* Z = w.Z[sg.type] + row0 * d;
            float* Hh = w.H[sg.type] + row0 * h;
            GemmArgs& a = g1[n];
            // first layer reads its rows through the plan's references and leaves a copy in Z
            a.a_ref = er.refs + sg.ref_off; a.a_base0 = w.act; a.a_base1 = er.rows;
            if (sg.rel_off >= 0) { a.a_add_idx = pl->d_rel + sg.rel_off; a.a_add = c->prm.R.p; }
            a.a_copy = Z; a.lda = d; a.B = W.Wa; a.ldb = d; a.C = Hh; a.ldc = h;
            a.M = sg.rows; a.N = h; a.K = d; a.bias = W.ba; a.relu = true;
            GemmArgs& b = g2[n];
            b.A = Hh; b.lda = h; b.B = W.Wb; b.ldb = h; b.M = sg.rows; b.N = d; b.K = h; b.bias = W.bb; b.ldc = d;
            if (c->have_pieces) {
                a.b_pieces = c->wp[sg.type][0]; a.b_kt = (d + 15) / 16;
                b.b_pieces = c->wp[sg.type][1]; b.b_kt = (h + 15) / 16;
            }
            if (sg.type == T_INTER) {
                b.C = w.Att + row0 * d;
            } else if (w.reclaim) {         // outputs go to their storage rows
                b.C = w.act;
                b.dst_row = pl->d_f_row + sg.out_base;
            } else {
                b.C = w.act + (size_t)sg.out_base * d;
            }
            ++n;
        }
        int rc_g;
        const HiddenPieces hpc = place_hidden_pieces(c, g1, n);
        bool emitted = false;
        if ((rc_g = gemm_timed(c, NGDB_TK_GEMM_FWD, g1, n, s, &emitted)) != NGDB_OK) return rc_g;
        if (emitted) take_hidden_pieces(hpc, g2, n);
        if ((rc_g = gemm_timed(c, NGDB_TK_GEMM_FWD, g2, n, s)) != NGDB_OK) return rc_g;
        for (const Segment& sg : segs) {
            if (sg.type != T_INTER) continue;
            Timed tm(c, NGDB_TK_INTER, s);
            InterJobs ij{};
            ij.d = d;
            for (int g = sg.g_lo; g < sg.g_hi; ++g) {
                const size_t mb = (size_t)(pl->hp.g_mlp_base[g] - (w.reclaim ? sg.mlp_base : 0)) * d;
                if (ij.count == INTER_MAX_JOBS) return fail(c, NGDB_ERR_UNSUPPORTED, "too many intersection classes in one level");
                InterJob& jb = ij.job[ij.count++];
                jb.X = w.Z[T_INTER] + mb; jb.Att = w.Att + mb;
                if (w.reclaim) {
                    jb.out = w.act;
                    jb.out_row = pl->d_f_row + pl->hp.g_out_base[g];
                } else {
                    jb.out = w.act + (size_t)pl->hp.g_out_base[g] * d;
                }
                jb.n = pl->hp.g_n[g]; jb.k = pl->hp.g_nin[g];
            }
            HIPCHK(c, launch_inter(ij, false, s));
        }
    }
    return NGDB_OK;
}

struct WgradJob {   // what enqueue_weight_grads needs after a backward chain
    int nt = 0;
    int types[3]{};
    size_t rows[3]{};
    const float* dY[3]{};
};

// Gradients of the MLP tensors of the given types (their Z / H / dH buffers, dY = gradient of
// the second layer's output): both weight matrices of every type in one grouped launch, the
// biases as column sums.
// With `open` the bias gradients are left as partial column sums (described in *open) for the
// dense Adam launch to add up: one launch less on the step's tail.
int enqueue_weight_grads(ngdb_ctx_t* c, const WgradJob& wj, hipStream_t s, ColsumJobs* open = nullptr) {
    const int d = c->cfg.d, h = c->cfg.h, nt = wj.nt;
    const int* types = wj.types;
    const size_t* rows = wj.rows;
    const float* const* dY = wj.dY;
    float* gW = ptr<float>(c->gW);
    Timed tm(c, NGDB_TK_WGRAD, s);
    GemmArgs w[6];
    ColsumJobs cs{};
    for (int i = 0; i < nt; ++i) {
        const int t = types[i], gs = gslot_of(t), r = (int)rows[i];
        GemmArgs& wa = w[2 * i];       // dWa[h,d] = dH^T Z
        wa.A = ptr<float>(c->dH[t]); wa.lda = h; wa.a_kcontig = false;
        wa.B = ptr<float>(c->Z[t]); wa.ldb = d; wa.b_kcontig = false;
        wa.C = gW + c->gw_off[gs + 0]; wa.ldc = d; wa.M = h; wa.N = d; wa.K = r;
        GemmArgs& wb = w[2 * i + 1];   // dWb[d,h] = dY^T H
        wb.A = dY[i]; wb.lda = d; wb.a_kcontig = false;
        wb.B = ptr<float>(c->H[t]); wb.ldb = h; wb.b_kcontig = false;
        wb.C = gW + c->gw_off[gs + 2]; wb.ldc = h; wb.M = d; wb.N = h; wb.K = r;
        float* part = ptr<float>(c->colsum_part) + (size_t)(2 * i) * COLSUM_MAX_CHUNKS * std::max(d, h);
        cs.job[cs.count++] = ColsumJob{ptr<float>(c->dH[t]), gW + c->gw_off[gs + 1], part, r, h, h, 0, 0};
        cs.job[cs.count++] = ColsumJob{dY[i], gW + c->gw_off[gs + 3], part + (size_t)COLSUM_MAX_CHUNKS * std::max(d, h),
                                       r, d, d, 0, 0};
    }
    {
        int route = GEMM_FP32;
        HIPCHK(c, launch_gemm_group(w, 2 * nt, s, &route));
        double flop = 0.0;
        for (int i = 0; i < 2 * nt; ++i) flop += 2.0 * w[i].M * w[i].N * w[i].K;
        tm.work(route, flop);
    }
    HIPCHK(c, launch_colsums(cs, s, open == nullptr));
    if (open) *open = cs;
    return NGDB_OK;
}

// reversed frontiers; *wj receives the inputs of the weight gradients (one grouped launch, later)
int enqueue_backward_box(ngdb_ctx_t* c, const ngdb_plan_t* pl, hipStream_t s, WgradJob* wj);
int enqueue_backward(ngdb_ctx_t* c, const ngdb_plan_t* pl, hipStream_t s, WgradJob* wj) {
    if (c->cfg.family == NGDB_FAMILY_BOX) return enqueue_backward_box(c, pl, s, wj);
    const int d = c->cfg.d, h = c->cfg.h;
    const HostPlan& hp = pl->hp;
    float* dact = ptr<float>(c->dact);
    for (int l = hp.n_levels; l >= 1; --l) {
        const std::vector<Segment>& segs = pl->levels[l];
        GemmArgs b2[3], b1[3];
        int n = 0;
        for (const Segment& sg : segs) {
            const MlpRefs W = mlp_of(c->prm, sg.type);
            const float* dOut;
            const float* addend = nullptr;
            if (sg.type == T_INTER) {
                Timed tm(c, NGDB_TK_INTER, s);
                InterJobs ij{};
                ij.d = d;
                for (int g = sg.g_lo; g < sg.g_hi; ++g) {
                    const size_t mb = (size_t)hp.g_mlp_base[g] * d;
                    if (ij.count == INTER_MAX_JOBS) return fail(c, NGDB_ERR_UNSUPPORTED, "too many intersection classes in one level");
                    InterJob& jb = ij.job[ij.count++];
                    jb.X = ptr<float>(c->Z[T_INTER]) + mb; jb.Att = ptr<float>(c->Att) + mb;
                    jb.dY = dact + (size_t)hp.g_out_base[g] * d;
                    jb.dAtt = ptr<float>(c->dAtt) + mb; jb.Dx = ptr<float>(c->Dx) + mb;
                    jb.n = hp.g_n[g]; jb.k = hp.g_nin[g];
                }
                HIPCHK(c, launch_inter(ij, true, s));
                dOut = ptr<float>(c->dAtt) + (size_t)sg.mlp_base * d;
                addend = ptr<float>(c->Dx) + (size_t)sg.mlp_base * d;
            } else {
                dOut = dact + (size_t)sg.out_base * d;
            }
            const float* Hh = ptr<float>(c->H[sg.type]) + (size_t)sg.mlp_base * h;
            float* dHh = ptr<float>(c->dH[sg.type]) + (size_t)sg.mlp_base * h;
            GemmArgs& x = b2[n];   // dH = (dOut * Wb) masked by relu
            x.A = dOut; x.lda = d; x.B = W.Wb; x.ldb = h; x.b_kcontig = false;
            x.C = dHh; x.ldc = h; x.M = sg.rows; x.N = h; x.K = d; x.mask = Hh; x.ldmask = h;
            GemmArgs& y = b1[n];   // dZ = dH * Wa, scattered to the gradient rows of the inputs
            y.A = dHh; y.lda = h; y.B = W.Wa; y.ldb = d; y.b_kcontig = false;
            y.C = dact; y.ldc = d; y.M = sg.rows; y.N = d; y.K = h;
            y.addend = addend; y.ldadd = d; y.dst_row = pl->d_in_gslot + sg.ref_off;
            if (c->have_pieces) {
                x.b_pieces = c->wp[sg.type][2]; x.b_kt = (d + 15) / 16;
                y.b_pieces = c->wp[sg.type][3]; y.b_kt = (h + 15) / 16;
            }
            ++n;
        }
        int rc_g;
        const HiddenPieces hpc = place_hidden_pieces(c, b2, n);
        bool emitted = false;
        if ((rc_g = gemm_timed(c, NGDB_TK_GEMM_BWD, b2, n, s, &emitted)) != NGDB_OK) return rc_g;
        if (emitted) take_hidden_pieces(hpc, b1, n);
        if ((rc_g = gemm_timed(c, NGDB_TK_GEMM_BWD, b1, n, s)) != NGDB_OK) return rc_g;
    }
    // weight gradients: one contraction per tensor over all rows of the type
    wj->nt = 3;
    const int types[3] = {T_PROJ, T_INTER, T_NEG};
    const size_t rows[3] = {(size_t)hp.n_proj, (size_t)hp.n_int_rows, (size_t)hp.n_neg};
    const float* dY[3] = {dact, ptr<float>(c->dAtt), dact + ((size_t)hp.n_proj + hp.n_inter) * d};
    for (int i = 0; i < 3; ++i) { wj->types[i] = types[i]; wj->rows[i] = rows[i]; wj->dY[i] = dY[i]; }
    return NGDB_OK;
}

// Box family, backward: the reverse of enqueue_forward_box; the gradient of a projection's
// input is the gradient of its output (copied to the input's rows, where the relation tables
// pick it up too).
int enqueue_backward_box(ngdb_ctx_t* c, const ngdb_plan_t* pl, hipStream_t s, WgradJob* wj) {
    const int d = c->cfg.d, h = c->cfg.h;
    const HostPlan& hp = pl->hp;
    for (int l = hp.n_levels; l >= 1; --l) {
        const std::vector<Segment>& segs = pl->levels[l];
        GemmArgs b2[GEMM_MAX_GROUP], b1[GEMM_MAX_GROUP];
        int n = 0;
        const Segment* ride = riding_projection(segs);
        for (const Segment& sg : segs) {
            if (sg.type == T_PROJ) {
                if (&sg == ride) continue;
                Timed tm(c, NGDB_TK_INTER, s);
                HIPCHK(c, launch_box_proj(box_proj_args(c, pl, sg), true, s));
                continue;
            }
            if (sg.type != T_INTER || n + 2 > GEMM_MAX_GROUP) return fail(c, NGDB_ERR_UNSUPPORTED, "operator not available in the box family");
            {
                Timed tm(c, NGDB_TK_INTER, s);
                InterJobs ij;
                int rc;
                if (2 * (sg.g_hi - sg.g_lo) <= INTER_MAX_JOBS) {
                    BoxPoolJobs pool{};
                    if ((rc = inter_jobs(c, pl, sg, false, true, nullptr, &pool)) != NGDB_OK) return rc;
                    if ((rc = inter_jobs(c, pl, sg, true, true, nullptr, &pool)) != NGDB_OK) return rc;
                    if (ride) { pool.has_proj = 1; pool.proj = box_proj_args(c, pl, *ride); ride = nullptr; }
                    HIPCHK(c, launch_box_pool(pool, true, s));
                } else {
                    if ((rc = inter_jobs(c, pl, sg, false, true, &ij)) != NGDB_OK) return rc;
                    HIPCHK(c, launch_inter(ij, true, s));
                    if ((rc = inter_jobs(c, pl, sg, true, true, &ij)) != NGDB_OK) return rc;
                    HIPCHK(c, launch_box_offset(ij, true, s));
                }
            }
            for (int part = 0; part < 2; ++part) {
                const int t = part ? T_NEG : T_INTER;
                const MlpRefs W = mlp_of(c->prm, t);
                const size_t mb = (size_t)sg.mlp_base;
                const float* Hh = ptr<float>(c->H[t]) + mb * h;
                float* dHh = ptr<float>(c->dH[t]) + mb * h;
                GemmArgs& x = b2[n];
                x.A = ptr<float>(part ? c->dGate : c->dAtt) + mb * d; x.lda = d; x.B = W.Wb; x.ldb = h; x.b_kcontig = false;
                x.C = dHh; x.ldc = h; x.M = sg.rows; x.N = h; x.K = d; x.mask = Hh; x.ldmask = h;
                GemmArgs& y = b1[n];
                y.A = dHh; y.lda = h; y.B = W.Wa; y.ldb = d; y.b_kcontig = false;
                y.C = ptr<float>(part ? c->doff : c->dact); y.ldc = d; y.M = sg.rows; y.N = d; y.K = h;
                y.addend = ptr<float>(part ? c->DxO : c->Dx) + mb * d; y.ldadd = d; y.dst_row = pl->d_in_gslot + sg.ref_off;
                ++n;
            }
        }
        if (n == 0) continue;
        int rc_g;
        if ((rc_g = gemm_timed(c, NGDB_TK_GEMM_BWD, b2, n, s)) != NGDB_OK) return rc_g;
        if ((rc_g = gemm_timed(c, NGDB_TK_GEMM_BWD, b1, n, s)) != NGDB_OK) return rc_g;
    }
    wj->nt = 2;
    wj->types[0] = T_INTER; wj->types[1] = T_NEG;
    wj->rows[0] = wj->rows[1] = (size_t)hp.n_int_rows;
    wj->dY[0] = ptr<float>(c->dAtt); wj->dY[1] = ptr<float>(c->dGate);
    return NGDB_OK;
}

int run_step(ngdb_ctx_t* c, const ngdb_plan_t* pl, const int32_t* d_neg, int K, hipStream_t stream, float* d_loss,
             bool apply) {
    if (!c || !pl) return NGDB_ERR_ARG;
    if (!c->bound) return fail(c, NGDB_ERR_STATE, "parameters not bound");
    if (K < 1 || (pl->hp.n_queries > 0 && !d_neg) || !d_loss)
        return fail(c, NGDB_ERR_ARG, "bad negatives (K >= 1 is required) / loss pointer");
    if (pl->n_entities != c->cfg.n_entities || !pl->d_blob)
        return fail(c, NGDB_ERR_ARG, "plan belongs to another configuration or was built without a device");
    const HostPlan& hp = pl->hp;
    const int d = c->cfg.d, B = hp.n_queries;
    if (c->presized && (K > c->cfg.k_max || B > c->cfg.b_max_queries))
        return fail(c, NGDB_ERR_ARG, "batch beyond the maxima declared at ngdb_create (b_max_queries, k_max)");
    c->have_grads = false;
    int rc = size_workspace(c, pl, K, !apply);
    if (rc != NGDB_OK) return rc;

    // 1. entity gradient index (depends only on the plan and the negatives)
    int32_t* e_src = nullptr;
    // With a library stream two independent pieces leave the caller's stream: the index build runs
    // beside the forward pass (without text features, where nothing before the tables needs it), and
    // the table updates run beside the weight gradients and the dense Adam step.
    const bool sem = c->cfg.d_sem > 0;
    const bool aside = c->n_side > 0;
    const bool idx_aside = aside && !sem;
    hipStream_t s_idx = idx_aside ? c->side[0] : stream;
    if (idx_aside) {
        HIPCHK(c, hipEventRecord(c->ev_fork, stream));
        HIPCHK(c, hipStreamWaitEvent(s_idx, c->ev_fork, 0));
    }
    EntRows er{};
    rc = prepare_entities(c, pl, d_neg, (int64_t)B * K, s_idx, stream, &e_src, &er);
    if (rc != NGDB_OK) return rc;

    // 2. forward frontiers
    rc = enqueue_forward(c, pl, er, stream, ctx_space(c));
    if (rc != NGDB_OK) return rc;

    // 3. scores, loss terms, dL/ds, gradients of the branch embeddings
    ScoreArgs sa{};
    sa.act = ptr<float>(c->act); sa.E = er.rows; sa.root_off = pl->d_root_off; sa.root_slot = pl->d_root_slot;
    sa.pos = er.pos; sa.cand = er.cand; sa.B = B; sa.C = K; sa.d = d; sa.max_branch = std::max(1, hp.max_branch);
    sa.gamma = c->cfg.gamma; sa.score = ptr<float>(c->score); sa.coef = ptr<float>(c->coef);
    sa.win = sem ? nullptr : ptr<int32_t>(c->win); sa.mask = sem ? c->mask.p : nullptr; sa.dact = ptr<float>(c->dact); sa.loss_terms = ptr<float>(c->loss_terms);
    const bool box = c->cfg.family == NGDB_FAMILY_BOX;
    if (box) { sa.off = ptr<float>(c->off); sa.doff = ptr<float>(c->doff); sa.alpha = c->cfg.box_alpha; }
    if (c->cfg.score_bf16) sa.E16 = ptr<uint16_t>(c->Eb);
    {
        Timed tm(c, NGDB_TK_SCORE, stream);
        hipError_t e = launch_score(sa, true, stream);
        if (e == hipErrorInvalidValue) return fail(c, NGDB_ERR_UNSUPPORTED, "embedding width / union branch count too large for the scoring kernel");
        HIPCHK(c, e);
    }

    // The records of the table pass (and the sum of the loss terms, in the same launch) depend on
    // the scoring pass only.  In a large step, where the table pass on the library stream ends the
    // step, they are resolved beside the backward pass; in a small step the extra fork costs more
    // than the launch it hides.
    hipStream_t s_tab = aside ? c->side[0] : stream;     // after the index on the same stream
    const int64_t n_contrib = (int64_t)hp.n_anchor + B + (int64_t)B * K;
    const bool small_step = std::min<int64_t>(n_contrib, c->cfg.n_entities) <= 65536;
    const bool resolve_early = aside && !small_step;
    auto resolve_records = [&]() -> int {
        HIPCHK(c, launch_resolve(e_src, n_contrib, hp.n_anchor, hp.n_slots, B, K, ptr<float>(c->coef),
                                 sem ? nullptr : ptr<int32_t>(c->win), ptr<float>(c->rec_coef), ptr<int32_t>(c->rec_row),
                                 ptr<float>(c->loss_terms), B > 0 ? 1.f / (2.f * B) : 0.f, d_loss, s_tab));
        return NGDB_OK;
    };
    if (resolve_early) {
        HIPCHK(c, hipEventRecord(c->ev_fork, stream));
        HIPCHK(c, hipStreamWaitEvent(s_tab, c->ev_fork, 0));
        if ((rc = resolve_records()) != NGDB_OK) return rc;
    }

    // 4. reversed frontiers
    WgradJob wj;
    rc = enqueue_backward(c, pl, stream, &wj);
    if (rc != NGDB_OK) return rc;

    // 5. table gradients (+ Adam), dense Adam
    const int64_t t = c->step + 1;
    AdamHyper ah{c->cfg.lr, c->cfg.beta1, c->cfg.beta2, c->cfg.eps,
                 (float)(1.0 - std::pow((double)c->cfg.beta1, (double)t)),
                 (float)(1.0 - std::pow((double)c->cfg.beta2, (double)t))};
    if (aside) {
        HIPCHK(c, hipEventRecord(c->ev_fork, stream));
        HIPCHK(c, hipStreamWaitEvent(s_tab, c->ev_fork, 0));
    }
    // (the sum of the loss terms is off the critical path there, in the launch that resolves the records)
    if (!resolve_early && (rc = resolve_records()) != NGDB_OK) return rc;
    TableArgs te{};
    te.P = c->prm.E.p; te.Mo = c->prm.E.m; te.Vo = c->prm.E.v;
    te.uniq = ptr<int32_t>(c->uniq); te.seg_off = ptr<int32_t>(c->seg_off);
    te.n_uniq_dev = ptr<int32_t>(c->n_uniq); te.d = d;
    te.rec_coef = ptr<float>(c->rec_coef); te.rec_row = ptr<int32_t>(c->rec_row);
    te.dact = ptr<float>(c->dact); te.act = ptr<float>(c->act); te.g_out = apply ? nullptr : ptr<float>(c->gE);
    if (sem) { te.mask = c->mask.p; te.g_bf16 = ptr<uint16_t>(c->g_bf16); }
    TableArgs tr = te;
    // parameters + two moments beyond what the 256 MB last-level cache could keep between steps
    te.streaming = (size_t)c->cfg.n_entities * d * 3 * sizeof(float) > ((size_t)512 << 20);
    if (c->cfg.score_bf16) te.shadow = ptr<uint16_t>(c->Eb);   // signs against the rounded rows; written only when updating
    if (box) { te.off = ptr<float>(c->off); te.alpha = c->cfg.box_alpha; }
    tr.g_bf16 = nullptr; tr.mask = nullptr;
    tr.P = c->prm.R.p; tr.Mo = c->prm.R.m; tr.Vo = c->prm.R.v;
    tr.uniq = pl->d_r_uniq; tr.seg_off = pl->d_r_seg_off; tr.n_uniq_dev = pl->d_n_r_uniq;
    tr.rec_coef = nullptr; tr.rec_row = pl->d_r_rec; tr.g_out = apply ? nullptr : ptr<float>(c->gR);
    // in a small step the relation tables ride in the entity table's launch (a launch of their own
    // each would add its latency to the tail of the step)
    TableArgs small[2] = {tr, tr};
    int n_small = 1;
    small[0].shadow = nullptr; small[0].off = nullptr;
    if (box) {   // relation offsets: the same segments over the offset gradients, gated by relu
        TableArgs& to = small[n_small++];
        to = small[0];
        to.P = c->prm.Ro.p; to.Mo = c->prm.Ro.m; to.Vo = c->prm.Ro.v;
        to.dact = ptr<float>(c->doff); to.relu_gate = true; to.g_out = apply ? nullptr : ptr<float>(c->gRo);
    }
    if (small_step) {   // one launch for all tables
        Timed tm(c, NGDB_TK_TABLE_E, s_tab);
        HIPCHK(c, launch_table_update(te, ah, s_tab, small, n_small, c->cfg.n_relations));
    } else {
        { Timed tm(c, NGDB_TK_TABLE_E, s_tab); HIPCHK(c, launch_table_update(te, ah, s_tab)); }
        for (int k = 0; k < n_small; ++k) {
            Timed tm(c, NGDB_TK_TABLE_R, s_tab);
            HIPCHK(c, launch_table_update(small[k], ah, s_tab));
        }
    }
    ColsumJobs open_sums{};
    rc = enqueue_weight_grads(c, wj, stream, apply ? &open_sums : nullptr);
    if (rc != NGDB_OK) return rc;
    if (apply) {
        DenseAdamJob job{};
        const ngdb_tensor* ts[12] = {&c->prm.W1, &c->prm.b1, &c->prm.W2, &c->prm.b2, &c->prm.V1, &c->prm.c1,
                                     &c->prm.V2, &c->prm.c2, &c->prm.U1, &c->prm.u1, &c->prm.U2, &c->prm.u2};
        const int64_t hd = (int64_t)c->cfg.h * d;
        const int64_t sz[4] = {hd, c->cfg.h, hd, d};
        for (int i = box ? 4 : 0; i < 12; ++i) {   // the box family has no projection MLP
            const int k = job.count++;
            job.p[k] = ts[i]->p; job.m[k] = ts[i]->m; job.v[k] = ts[i]->v;
            job.g[k] = ptr<float>(c->gW) + c->gw_off[i];
            job.n[k] = sz[i % 4];
            for (int q = 0; q < open_sums.count; ++q)     // a bias: its gradient is still in chunks
                if (open_sums.job[q].out == job.g[k]) {
                    job.gsum[k] = open_sums.job[q].out;
                    job.g[k] = open_sums.job[q].part;
                    job.chunks[k] = open_sums.job[q].chunks;
                }
        }
        Timed tm(c, NGDB_TK_ADAM, stream);
        HIPCHK(c, launch_dense_adam(job, ah, stream));
    }
    if (aside) {
        HIPCHK(c, hipEventRecord(c->ev_join, s_tab));
        HIPCHK(c, hipStreamWaitEvent(stream, c->ev_join, 0));
    }
    if (sem) {
        // gradient of the text projection over the touched rows, then its Adam step
        Timed tm(c, NGDB_TK_SEM, stream);
        const int ds = c->cfg.d_sem;
        SemWgradArgs wa{};
        wa.H = c->prm.H_sem; wa.ids = ptr<int32_t>(c->uniq); wa.G = ptr<uint16_t>(c->g_bf16);
        wa.n_rows_dev = ptr<int32_t>(c->n_uniq); wa.n_rows = (int)std::min<int64_t>(n_contrib, c->cfg.n_entities);
        wa.d = d; wa.ds = ds; wa.n_splits = sem_wgrad_splits(wa.n_rows, d, ds); wa.partial = ptr<float>(c->wp_partial);
        HIPCHK(c, launch_sem_wgrad(wa, ptr<float>(c->gWp), stream));
        if (apply) {
            DenseAdamJob job{};
            job.p[0] = c->prm.Wp.p; job.m[0] = c->prm.Wp.m; job.v[0] = c->prm.Wp.v;
            job.g[0] = ptr<float>(c->gWp); job.n[0] = (int64_t)d * ds; job.count = 1;
            HIPCHK(c, launch_dense_adam(job, ah, stream));
        }
    }

    HIPCHK(c, hipEventRecord(pl->blob.last_use, stream));
    if (apply) c->step = t;
    // describe the results
    ngdb_grad_view& gv = c->gv;
    std::memset(&gv, 0, sizeof(gv));
    gv.n_e_contrib = hp.n_anchor + B + B * K;
    gv.n_r_uniq = (int32_t)hp.r_uniq.size();
    gv.n_slots = hp.n_slots;
    gv.n_pairs = B * (K + 1);
    gv.e_uniq = ptr<int32_t>(c->uniq);
    gv.e_seg_off = ptr<int32_t>(c->seg_off);
    gv.e_src = e_src;
    gv.gE = apply ? nullptr : ptr<float>(c->gE);
    gv.gR = apply ? nullptr : ptr<float>(c->gR);
    for (int i = box ? 4 : 0; i < 12; ++i) gv.g_mlp[i] = ptr<float>(c->gW) + c->gw_off[i];
    if (box) {
        gv.gRo = apply ? nullptr : ptr<float>(c->gRo);
        gv.off = ptr<float>(c->off);
        gv.doff = ptr<float>(c->doff);
    }
    gv.e_shadow = c->cfg.score_bf16 ? ptr<uint16_t>(c->Eb) : nullptr;
    gv.g_Wp = sem ? ptr<float>(c->gWp) : nullptr;
    gv.act = ptr<float>(c->act);
    gv.dact = ptr<float>(c->dact);
    gv.n_grad_rows = hp.n_slots + hp.n_anchor;
    gv.pair_score = ptr<float>(c->score);
    gv.loss_terms = ptr<float>(c->loss_terms);
    c->have_grads = true;
    return NGDB_OK;
}

bool new_blob(ngdb_ctx_t* c, size_t cap, PlanBlob* pb) {
    pb->cap = cap;
    if (hipMalloc((void**)&pb->dev, cap * 4) != hipSuccess ||
        hipHostMalloc((void**)&pb->pinned, cap * 4, hipHostMallocDefault) != hipSuccess ||
        hipEventCreateWithFlags(&pb->last_use, hipEventDisableTiming) != hipSuccess) {
        if (pb->dev) (void)hipFree(pb->dev);
        if (pb->pinned) (void)hipHostFree(pb->pinned);
        *pb = PlanBlob{};
        return false;
    }
    c->n_alloc += 2;
    return true;
}

// The whole workspace and four plan buffers for the largest batch the configuration declares
// (b_max_queries queries of at most max_nodes_per_query nodes, k_max negatives): every count a plan
// can reach is bounded by the number of nodes.
int presize(ngdb_ctx_t* c) {
    const size_t B = (size_t)c->cfg.b_max_queries, cap = B * (size_t)c->cfg.max_nodes_per_query;
    if (cap > (size_t)INT32_MAX / 4 || B * ((size_t)c->cfg.k_max + 1) > (size_t)INT32_MAX)
        return fail(c, NGDB_ERR_ARG, "declared maxima too large");
    ngdb_plan_s most;
    HostPlan& hp = most.hp;
    hp.n_queries = (int32_t)B;
    hp.n_slots = hp.n_anchor = hp.n_proj = hp.n_int_rows = hp.n_neg = hp.n_roots = (int32_t)cap;
    hp.n_f_rows = (int32_t)cap;
    for (int t = 0; t < 3; ++t) hp.f_step_rows[t] = (int32_t)cap;
    hp.in_ref.resize(cap);
    int rc = size_workspace(c, &most, c->cfg.k_max, false);
    if (rc != NGDB_OK) return rc;
    const size_t blob_cap = 10 * cap + 4 * B + 2 * (size_t)std::min<size_t>(cap, c->cfg.n_relations) + 256;
    for (int i = 0; i < 4; ++i) {
        PlanBlob pb;
        if (!new_blob(c, blob_cap, &pb)) return fail(c, NGDB_ERR_OOM, "allocation of the plan buffers failed");
        c->blob_pool.push_back(pb);
    }
    c->presized = true;
    return NGDB_OK;
}

// Device address of the scratch array on the current GPU (looked up on first use per device).
hipError_t noalloc_scratch(unsigned char** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        unsigned char* p = nullptr;
        e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

// ------------------------------------------------------------------------ C ABI
extern "C" {

int ngdb_create(const ngdb_config* cfg, ngdb_ctx_t** out) {
    if (!cfg || !out) return NGDB_ERR_ARG;
    *out = nullptr;
    if (cfg->n_entities <= 0 || cfg->n_relations <= 0 || cfg->d <= 0 || cfg->h <= 0 || (cfg->d & 3) ||
        (cfg->h & 3) || cfg->d > 1024 || cfg->num_streams < 1 || cfg->num_streams > 4 || cfg->d_sem < 0)
        return NGDB_ERR_ARG;
    if (cfg->d_sem != 0 && ((cfg->d_sem & 63) || (cfg->d & 7))) return NGDB_ERR_ARG;
    if ((cfg->schedule != NGDB_SCHED_LEVEL && cfg->schedule != NGDB_SCHED_MAX_FILL) || cfg->b_max < 0) return NGDB_ERR_ARG;
    if (cfg->family != NGDB_FAMILY_VEC && cfg->family != NGDB_FAMILY_BOX) return NGDB_ERR_ARG;
    if (cfg->family == NGDB_FAMILY_BOX && (cfg->d_sem != 0 || !(cfg->box_alpha >= 0.f && cfg->box_alpha <= 1.f)))
        return NGDB_ERR_ARG;
    if ((cfg->score_bf16 != 0 && cfg->score_bf16 != 1) || (cfg->score_bf16 && (cfg->family != NGDB_FAMILY_VEC || cfg->d_sem != 0 || (cfg->d & 7))))
        return NGDB_ERR_ARG;
    if (cfg->b_max_queries < 0 || cfg->k_max < 0 || cfg->max_nodes_per_query < 0 ||
        (cfg->b_max_queries > 0 && cfg->k_max < 1) || (cfg->b_max_queries == 0 && (cfg->k_max || cfg->max_nodes_per_query)))
        return NGDB_ERR_ARG;
    ngdb_ctx_t* c = new (std::nothrow) ngdb_ctx_s();
    if (!c) return NGDB_ERR_OOM;
    c->cfg = *cfg;
    if (c->cfg.b_max_queries > 0 && c->cfg.max_nodes_per_query == 0) c->cfg.max_nodes_per_query = 12;
    c->n_side = cfg->num_streams > 1 ? 1 : 0;
    bool ok = true;
    if (c->n_side) ok = hipStreamCreateWithFlags(&c->side[0], hipStreamNonBlocking) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) == hipSuccess;
    ok = ok && hipStreamCreateWithFlags(&c->upload, hipStreamNonBlocking) == hipSuccess;
    unsigned char* sp = nullptr;
    ok = ok && noalloc_scratch(&sp) == hipSuccess;     // address of the static scratch on this GPU
    if (!ok) {
        ngdb_destroy(c);
        return NGDB_ERR_HIP;
    }
    if (c->cfg.b_max_queries > 0) {
        const int rc = presize(c);
        if (rc != NGDB_OK) {
            ngdb_destroy(c);
            return rc;
        }
    }
    *out = c;
    return NGDB_OK;
}

void ngdb_destroy(ngdb_ctx_t* c) {
    if (!c) return;
    (void)hipDeviceSynchronize();
    DevBuf* all[] = {&c->act, &c->dact, &c->Z[0], &c->Z[1], &c->Z[2], &c->H[0], &c->H[1], &c->H[2], &c->dH[0],
                     &c->dH[1], &c->dH[2], &c->Att, &c->dAtt, &c->Dx, &c->score, &c->coef, &c->win, &c->mask,
                     &c->loss_terms, &c->rec_coef, &c->rec_row, &c->keys_a, &c->keys_b, &c->vals_a, &c->vals_b, &c->hist, &c->scan_tmp,
                     &c->uniq, &c->seg_off, &c->n_uniq, &c->gW, &c->w_pieces, &c->h_pieces, &c->gE, &c->gR, &c->colsum_part, &c->rank_dist, &c->rank_thr, &c->rank_count,
                     &c->Wb, &c->Ef, &c->inv, &c->refs_sem, &c->g_bf16, &c->wp_partial, &c->gWp, &c->rank_ef,
                     &c->off, &c->doff, &c->Gate, &c->dGate, &c->DxO, &c->gRo, &c->Eb};
    for (DevBuf* b : all) release(*b);
    if (c->side[0]) (void)hipStreamDestroy(c->side[0]);
    if (c->ev_join) (void)hipEventDestroy(c->ev_join);
    if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
    if (c->upload) (void)hipStreamDestroy(c->upload);
    // plans that outlive the context keep their host arrays (export, free) and lose their device buffer
    for (ngdb_plan_t* pl : c->live_plans) {
        c->blob_pool.push_back(pl->blob);
        pl->blob = PlanBlob{};
        pl->d_blob = nullptr;
        pl->owner = nullptr;
    }
    c->live_plans.clear();
    for (PlanBlob& b : c->blob_pool) {
        if (b.dev) (void)hipFree(b.dev);
        if (b.pinned) (void)hipHostFree(b.pinned);
        if (b.last_use) (void)hipEventDestroy(b.last_use);
    }
    for (const ngdb_ctx_s::Bracket& b : c->brackets) {
        (void)hipEventDestroy(b.a);
        (void)hipEventDestroy(b.b);
    }
    for (hipEvent_t e : c->spare_events) (void)hipEventDestroy(e);
    delete c;
}

int ngdb_bind_params(ngdb_ctx_t* c, const ngdb_params* p) {
    if (!c || !p) return NGDB_ERR_ARG;
    const bool box = c->cfg.family == NGDB_FAMILY_BOX;
    const ngdb_tensor* ts[14] = {&p->E, &p->R, &p->V1, &p->c1, &p->V2, &p->c2, &p->U1, &p->u1, &p->U2, &p->u2,
                                 box ? &p->Ro : &p->W1, box ? &p->Ro : &p->b1, box ? &p->Ro : &p->W2,
                                 box ? &p->Ro : &p->b2};
    for (const ngdb_tensor* t : ts) {
        if (!t->p || !t->m || !t->v) return fail(c, NGDB_ERR_ARG, "null parameter or moment tensor");
        if (((uintptr_t)t->p | (uintptr_t)t->m | (uintptr_t)t->v) & 15)
            return fail(c, NGDB_ERR_ARG, "tensors must be 16-byte aligned");
    }
    if (c->cfg.d_sem > 0) {
        if (!p->Wp.p || !p->Wp.m || !p->Wp.v || !p->H_sem)
            return fail(c, NGDB_ERR_ARG, "text features configured: Wp (with moments) and H_sem are required");
        if (((uintptr_t)p->Wp.p | (uintptr_t)p->Wp.m | (uintptr_t)p->Wp.v | (uintptr_t)p->H_sem) & 15)
            return fail(c, NGDB_ERR_ARG, "tensors must be 16-byte aligned");
    }
    if (p->step < 0) return fail(c, NGDB_ERR_ARG, "negative step count");
    if (c->cfg.score_bf16) {   // the bf16 copy of the entity table
        const size_t n = (size_t)c->cfg.n_entities * c->cfg.d;
        int rc = ensure(c, c->Eb, n * sizeof(uint16_t), true);
        if (rc != NGDB_OK) return rc;
        HIPCHK(c, launch_cast_bf16(p->E.p, ptr<uint16_t>(c->Eb), (int64_t)n, nullptr));
        HIPCHK(c, hipDeviceSynchronize());
    }
    c->prm = *p;
    c->step = p->step;
    c->bound = true;
    c->have_grads = false;
    return NGDB_OK;
}

// host part of planning: frontiers, index arrays, level/type segments
static int plan_host(const ngdb_query_batch* qb, int32_t n_entities, int32_t n_relations, int32_t schedule,
                     int32_t b_max, ngdb_plan_t** out, std::string& err) {
    *out = nullptr;
    ngdb_plan_t* pl = new (std::nothrow) ngdb_plan_s();
    if (!pl) {
        err = "host allocation failed";
        return NGDB_ERR_OOM;
    }
    int rc = NGDB_OK;
    try {
        rc = build_plan(*qb, n_entities, n_relations, schedule, b_max, pl->hp, err);
    } catch (const std::bad_alloc&) {
        rc = NGDB_ERR_OOM;
        err = "host allocation failed";
    }
    if (rc != NGDB_OK) {
        delete pl;
        return rc;
    }
    HostPlan& hp = pl->hp;
    pl->n_entities = n_entities;
    pl->levels.assign(hp.n_levels + 1, {});
    for (int g = 0; g < hp.n_groups; ++g) {
        std::vector<Segment>& segs = pl->levels[hp.g_level[g]];
        const int t = type_index(hp.g_type[g]);
        const int rows = hp.g_n[g] * (t == T_INTER ? hp.g_nin[g] : 1);
        if (!segs.empty() && segs.back().type == t) {   // further intersection class of the same level
            segs.back().rows += rows;
            segs.back().g_hi = g + 1;
        } else {
            Segment sg;
            sg.type = t; sg.rows = rows; sg.mlp_base = hp.g_mlp_base[g]; sg.ref_off = hp.g_ref_off[g];
            sg.rel_off = hp.g_rel_off[g]; sg.out_base = hp.g_out_base[g]; sg.g_lo = g; sg.g_hi = g + 1;
            segs.push_back(sg);
        }
    }
    *out = pl;
    return NGDB_OK;
}

int ngdb_plan_host(int32_t n_entities, int32_t n_relations, const ngdb_query_batch* qb, ngdb_plan_t** out) {
    return ngdb_plan_host_sched(n_entities, n_relations, qb, NGDB_SCHED_LEVEL, 0, out);
}

int ngdb_plan_host_sched(int32_t n_entities, int32_t n_relations, const ngdb_query_batch* qb, int32_t schedule,
                         int32_t b_max, ngdb_plan_t** out) {
    if (!qb || !out || n_entities <= 0 || n_relations <= 0) return NGDB_ERR_ARG;
    std::string err;
    return plan_host(qb, n_entities, n_relations, schedule, b_max, out, err);
}

int ngdb_plan(ngdb_ctx_t* c, const ngdb_query_batch* qb, ngdb_plan_t** out) {
    if (!c || !qb || !out) return NGDB_ERR_ARG;
    std::string err;
    ngdb_plan_t* pl = nullptr;
    int rc = plan_host(qb, c->cfg.n_entities, c->cfg.n_relations, c->cfg.schedule, c->cfg.b_max, &pl, err);
    if (rc != NGDB_OK) return fail(c, rc, err);
    HostPlan& hp = pl->hp;
    if (c->presized && (hp.n_queries > c->cfg.b_max_queries ||
                        (size_t)hp.n_slots + hp.n_anchor > (size_t)c->cfg.b_max_queries * c->cfg.max_nodes_per_query)) {
        delete pl;
        return fail(c, NGDB_ERR_ARG, "batch beyond the maxima declared at ngdb_create (b_max_queries, max_nodes_per_query)");
    }
    if (c->cfg.family == NGDB_FAMILY_BOX) {
        bool ok = hp.n_neg == 0;
        for (int g = 0; g < hp.n_groups && ok; ++g) {
            if (hp.g_type[g] != NGDB_OP_INTER) continue;
            const int n_ref = hp.g_n[g] * hp.g_nin[g];
            for (int i = 0; i < n_ref && ok; ++i) ok = hp.in_ref[hp.g_ref_off[g] + i] >= 0;
        }
        if (!ok) {
            delete pl;
            return fail(c, NGDB_ERR_UNSUPPORTED, "box family: no negation, and an intersection input must be an operator output");
        }
    }

    // one upload: every device-side array, each padded to 16 bytes
    std::vector<int32_t> blob;
    auto put = [&](const std::vector<int32_t>& v) {
        const size_t off = blob.size();
        blob.insert(blob.end(), v.begin(), v.end());
        while (blob.size() & 3) blob.push_back(0);
        if (v.empty()) blob.resize(blob.size() + 4, 0);
        return off;
    };
    std::vector<int32_t> r_rec(hp.r_src.size());     // relation contributions are gradient rows
    for (size_t i = 0; i < r_rec.size(); ++i) r_rec[i] = -1 - hp.r_src[i];
    std::vector<int32_t> ekeys = hp.anchor_ent;
    ekeys.insert(ekeys.end(), hp.pos.begin(), hp.pos.end());
    const size_t o_ref = put(hp.in_ref), o_gs = put(hp.in_gslot), o_rel = put(hp.rel), o_ro = put(hp.root_off),
                 o_rs = put(hp.root_slot), o_pos = put(hp.pos), o_ek = put(ekeys), o_ru = put(hp.r_uniq),
                 o_rso = put(hp.r_seg_off), o_rsrc = put(hp.r_src), o_rrec = put(r_rec),
                 o_nru = put(std::vector<int32_t>{(int32_t)hp.r_uniq.size()});
    std::vector<int32_t> f_in_ref(hp.in_ref.size()), f_root(hp.root_slot.size());
    for (size_t i = 0; i < f_in_ref.size(); ++i) f_in_ref[i] = hp.in_ref[i] >= 0 ? hp.f_row[hp.in_ref[i]] : hp.in_ref[i];
    for (size_t i = 0; i < f_root.size(); ++i) f_root[i] = hp.f_row[hp.root_slot[i]];
    const size_t o_fref = put(f_in_ref), o_frow = put(hp.f_row), o_froot = put(f_root);
    // a recycled blob (its last reader has finished) or a new one
    PlanBlob pb;
    {
        std::lock_guard<std::mutex> lk(c->mu);
        for (size_t i = 0; i < c->blob_pool.size(); ++i)
            if (c->blob_pool[i].cap >= blob.size()) {
                pb = c->blob_pool[i];
                c->blob_pool.erase(c->blob_pool.begin() + i);
                break;
            }
    }
    if (!pb.dev) {
        bool ok;
        {
            std::lock_guard<std::mutex> lk(c->mu);     // (the allocation counter)
            ok = new_blob(c, blob.size() + blob.size() / 2 + 1024, &pb);
        }
        if (!ok) {
            delete pl;
            return fail(c, NGDB_ERR_OOM, "allocation for the plan failed");
        }
    } else if (hipEventSynchronize(pb.last_use) != hipSuccess) {
        delete pl;
        return fail(c, NGDB_ERR_HIP, "waiting for a recycled plan buffer failed");
    }
    std::memcpy(pb.pinned, blob.data(), blob.size() * 4);
    if (hipMemcpyAsync(pb.dev, pb.pinned, blob.size() * 4, hipMemcpyHostToDevice, c->upload) != hipSuccess ||
        hipStreamSynchronize(c->upload) != hipSuccess) {
        {
            std::lock_guard<std::mutex> lk(c->mu);
            c->blob_pool.push_back(pb);
        }
        delete pl;
        return fail(c, NGDB_ERR_HIP, "plan upload failed");
    }
    pl->owner = c;
    pl->blob = pb;
    {
        std::lock_guard<std::mutex> lk(c->mu);
        c->live_plans.push_back(pl);
    }
    pl->d_blob = pb.dev;
    pl->d_in_ref = pl->d_blob + o_ref; pl->d_in_gslot = pl->d_blob + o_gs; pl->d_rel = pl->d_blob + o_rel;
    pl->d_root_off = pl->d_blob + o_ro; pl->d_root_slot = pl->d_blob + o_rs; pl->d_pos = pl->d_blob + o_pos;
    pl->d_ekeys_head = pl->d_blob + o_ek; pl->d_r_uniq = pl->d_blob + o_ru; pl->d_r_seg_off = pl->d_blob + o_rso;
    pl->d_r_src = pl->d_blob + o_rsrc; pl->d_r_rec = pl->d_blob + o_rrec; pl->d_n_r_uniq = pl->d_blob + o_nru;
    pl->d_f_in_ref = pl->d_blob + o_fref; pl->d_f_row = pl->d_blob + o_frow; pl->d_f_root = pl->d_blob + o_froot;
    *out = pl;
    return NGDB_OK;
}

int ngdb_plan_export(const ngdb_plan_t* pl, ngdb_plan_view* v) {
    if (!pl || !v) return NGDB_ERR_ARG;
    const HostPlan& hp = pl->hp;
    v->n_queries = hp.n_queries; v->n_groups = hp.n_groups; v->n_levels = hp.n_levels; v->n_slots = hp.n_slots;
    v->n_anchor = hp.n_anchor; v->n_proj = hp.n_proj; v->n_inter = hp.n_inter; v->n_neg = hp.n_neg;
    v->n_int_rows = hp.n_int_rows; v->n_roots = hp.n_roots; v->n_refs = (int32_t)hp.in_ref.size();
    v->n_r_uniq = (int32_t)hp.r_uniq.size();
    v->peak_live = hp.peak_live;
    v->lvl_off = hp.lvl_off.data(); v->g_level = hp.g_level.data(); v->g_type = hp.g_type.data();
    v->g_nin = hp.g_nin.data(); v->g_n = hp.g_n.data(); v->g_out_base = hp.g_out_base.data();
    v->g_mlp_base = hp.g_mlp_base.data(); v->g_ref_off = hp.g_ref_off.data(); v->g_rel_off = hp.g_rel_off.data();
    v->in_ref = hp.in_ref.data(); v->in_gslot = hp.in_gslot.data(); v->rel = hp.rel.data();
    v->root_off = hp.root_off.data(); v->root_slot = hp.root_slot.data(); v->anchor_ent = hp.anchor_ent.data();
    v->pos = hp.pos.data(); v->r_uniq = hp.r_uniq.data(); v->r_seg_off = hp.r_seg_off.data();
    v->r_src = hp.r_src.data();
    v->n_f_rows = hp.n_f_rows;
    for (int k = 0; k < 3; ++k) v->f_step_rows[k] = hp.f_step_rows[k];
    v->f_row = hp.f_row.data();
    return NGDB_OK;
}

void ngdb_plan_free(ngdb_plan_t* pl) {
    if (!pl) return;
    if (pl->owner) {   // the device buffer goes back to its context (reused once last_use has passed)
        ngdb_ctx_t* c = pl->owner;
        std::lock_guard<std::mutex> lk(c->mu);
        c->live_plans.erase(std::remove(c->live_plans.begin(), c->live_plans.end(), pl), c->live_plans.end());
        if (pl->blob.dev) c->blob_pool.push_back(pl->blob);
    }
    delete pl;
}

int ngdb_train_step(ngdb_ctx_t* c, const ngdb_plan_t* pl, const int32_t* d_neg, int32_t K, void* stream,
                    float* d_loss) {
    return run_step(c, pl, d_neg, K, static_cast<hipStream_t>(stream), d_loss, true);
}

int ngdb_forward_backward(ngdb_ctx_t* c, const ngdb_plan_t* pl, const int32_t* d_neg, int32_t K, void* stream,
                          float* d_loss) {
    return run_step(c, pl, d_neg, K, static_cast<hipStream_t>(stream), d_loss, false);
}

int ngdb_get_grads(ngdb_ctx_t* c, ngdb_grad_view* out) {
    if (!c || !out) return NGDB_ERR_ARG;
    if (!c->have_grads) return fail(c, NGDB_ERR_STATE, "no step has been run on this context");
    HIPCHK(c, hipDeviceSynchronize());
    HIPCHK(c, hipMemcpy(&c->gv.n_e_uniq, c->n_uniq.p, sizeof(int32_t), hipMemcpyDeviceToHost));
    *out = c->gv;
    return NGDB_OK;
}

int ngdb_score(ngdb_ctx_t* c, const ngdb_plan_t* pl, const int32_t* d_cand, int32_t C, int32_t topk,
               float* d_scores, int32_t* d_topk_ids, float* d_topk_dist, void* stream) {
    if (!c || !pl) return NGDB_ERR_ARG;
    if (!c->bound) return fail(c, NGDB_ERR_STATE, "parameters not bound");
    if (pl->n_entities != c->cfg.n_entities || !pl->d_blob)
        return fail(c, NGDB_ERR_ARG, "plan belongs to another configuration or was built without a device");
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (d_cand) {
        if (C <= 0 || !d_scores) return fail(c, NGDB_ERR_ARG, "candidate mode needs C > 0 and d_scores");
    } else if (topk < 1 || topk > NGDB_MAX_TOPK || !d_topk_ids || !d_topk_dist) {
        return fail(c, NGDB_ERR_ARG, "all-entity mode needs 1 <= topk <= NGDB_MAX_TOPK and both output arrays");
    }
    c->have_grads = false;
    const bool sem = c->cfg.d_sem > 0;
    // forward only: an operator output is reclaimed as soon as its consumer has run (Sec. 4.3);
    // the box family keeps one row per output
    const bool reclaim = c->cfg.family == NGDB_FAMILY_VEC;
    const int64_t n_tail = d_cand ? (int64_t)pl->hp.n_queries * C : 0;
    if (c->presized && d_cand && C > c->cfg.k_max)
        return fail(c, NGDB_ERR_ARG, "more candidates per query than the k_max declared at ngdb_create");
    int rc = reclaim ? size_forward_only(c, pl, n_tail) : size_workspace(c, pl, d_cand ? C : 0, false);
    if (rc != NGDB_OK) return rc;
    const int32_t* roots = reclaim ? pl->d_f_root : pl->d_root_slot;
    EntRows er{c->prm.E.p, reclaim ? pl->d_f_in_ref : pl->d_in_ref, pl->d_pos, d_cand};
    if (sem) {   // fused rows of the anchors (and candidates) first
        int32_t* e_src = nullptr;
        rc = prepare_entities(c, pl, d_cand, n_tail, s, s, &e_src, &er, reclaim);
        if (rc != NGDB_OK) return rc;
    }
    rc = enqueue_forward(c, pl, er, s, ctx_space(c, reclaim));
    if (rc != NGDB_OK) return rc;
    if (d_cand) {
        ScoreArgs sa{};
        sa.act = ptr<float>(c->act); sa.E = er.rows; sa.root_off = pl->d_root_off; sa.root_slot = roots;
        sa.pos = nullptr; sa.cand = er.cand; sa.B = pl->hp.n_queries; sa.C = C; sa.d = c->cfg.d;
        sa.max_branch = std::max(1, pl->hp.max_branch); sa.gamma = c->cfg.gamma; sa.score = d_scores;
        if (c->cfg.family == NGDB_FAMILY_BOX) { sa.off = ptr<float>(c->off); sa.alpha = c->cfg.box_alpha; }
        if (c->cfg.score_bf16) sa.E16 = ptr<uint16_t>(c->Eb);
        hipError_t e;
        { Timed tm(c, NGDB_TK_SCORE, s); e = launch_score(sa, false, s); }
        if (e == hipErrorInvalidValue) return fail(c, NGDB_ERR_UNSUPPORTED, "embedding width / union branch count too large for the scoring kernel");
        HIPCHK(c, e);
    } else {
        // entity chunks: distances of every branch row to the chunk, then the running top-k
        const int N = c->cfg.n_entities, d = c->cfg.d, R = pl->hp.n_roots;
        const float* box_off = c->cfg.family == NGDB_FAMILY_BOX ? ptr<float>(c->off) : nullptr;
        const int chunk = std::min(N, 1 << 16);
        const int ld = (chunk + 3) & ~3;
        rc = ensure(c, c->rank_dist, std::max<size_t>((size_t)R * ld * sizeof(float), 256), true);
        if (rc != NGDB_OK) return rc;
        if (sem) {
            rc = ensure(c, c->rank_ef, (size_t)chunk * d * sizeof(float), true);
            if (rc != NGDB_OK) return rc;
        }
        Timed tm(c, NGDB_TK_SCORE, s);
        for (int e0 = 0; e0 < N; e0 += chunk) {
            const int cnt = std::min(chunk, N - e0);
            const float* rows = c->prm.E.p + (size_t)e0 * d;
            if (sem) {   // the chunk's fused rows
                SemFuseArgs fa{};
                fa.H = c->prm.H_sem; fa.Wb = ptr<uint16_t>(c->Wb); fa.E = c->prm.E.p; fa.id_base = e0;
                fa.n_rows = cnt; fa.d = d; fa.ds = c->cfg.d_sem; fa.out = ptr<float>(c->rank_ef);
                HIPCHK(c, launch_sem_fuse(fa, s));
                rows = ptr<float>(c->rank_ef);
            }
            HIPCHK(c, launch_l1_tile(ptr<float>(c->act), box_off, c->cfg.box_alpha, roots, R, rows, nullptr, cnt, d,
                                     ptr<float>(c->rank_dist), ld, s,
                                     c->cfg.score_bf16 ? ptr<uint16_t>(c->Eb) + (size_t)e0 * d : nullptr));
            HIPCHK(c, launch_topk_merge(ptr<float>(c->rank_dist), ld, pl->d_root_off, pl->hp.n_queries, e0, cnt, topk,
                                        e0 == 0, d_topk_dist, d_topk_ids, s));
        }
    }
    HIPCHK(c, hipEventRecord(pl->blob.last_use, s));
    return NGDB_OK;
}

size_t ngdb_score_noalloc_bytes(const ngdb_ctx_t* c, const ngdb_plan_t* pl) {
    if (!c || !pl) return 0;
    const FwdBytes fb = forward_bytes(c, pl, true);
    auto up = [](size_t b) { return (b + 255) & ~size_t(255); };
    size_t need = up(fb.act) + up(fb.att);
    for (int t = 0; t < 3; ++t) need += up(fb.z[t]) + up(fb.h[t]);
    return need;
}

int ngdb_score_noalloc(ngdb_ctx_t* c, const ngdb_plan_t* pl, const int32_t* d_cand, int32_t C, float* d_scores,
                       void* stream) {
    if (!c || !pl) return NGDB_ERR_ARG;
    if (!c->bound) return fail(c, NGDB_ERR_STATE, "parameters not bound");
    if (pl->n_entities != c->cfg.n_entities || !pl->d_blob)
        return fail(c, NGDB_ERR_ARG, "plan belongs to another configuration or was built without a device");
    if (c->cfg.family != NGDB_FAMILY_VEC || c->cfg.d_sem != 0)
        return fail(c, NGDB_ERR_UNSUPPORTED, "ngdb_score_noalloc: vector family without text features only");
    if (!d_cand || C <= 0 || !d_scores) return fail(c, NGDB_ERR_ARG, "ngdb_score_noalloc needs candidates, C > 0 and d_scores");
    const size_t need = ngdb_score_noalloc_bytes(c, pl);
    if (need > NOALLOC_BYTES)
        return fail(c, NGDB_ERR_ARG, "ngdb_score_noalloc: this batch needs " + std::to_string(need) +
                                         " bytes of forward workspace, the static scratch holds " +
                                         std::to_string(NOALLOC_BYTES) + " (NGDB_NOALLOC_SCRATCH_MIB)");
    unsigned char* base = nullptr;
    HIPCHK(c, noalloc_scratch(&base));
    // carve the forward buffers out of the scratch (outputs reclaimed once their consumer has run,
    // per-step buffers: as in ngdb_score); every row that is read was written earlier in this call
    // (operator outputs before their consumers, copies and hidden rows by the launch before the
    // one that reads them), so nothing has to be cleared
    const HostPlan& hp = pl->hp;
    const FwdBytes fb = forward_bytes(c, pl, true);
    size_t at = 0;
    auto take = [&](size_t bytes) {
        float* p = reinterpret_cast<float*>(base + at);
        at += (bytes + 255) & ~size_t(255);
        return p;
    };
    FwdSpace w{};
    w.reclaim = true;
    w.act = take(fb.act);
    w.Att = take(fb.att);
    for (int t = 0; t < 3; ++t) {
        w.Z[t] = take(fb.z[t]);
        w.H[t] = take(fb.h[t]);
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    c->have_grads = false;
    const uint32_t timing = c->timing_mask;     // event brackets would create events: off for this call
    c->timing_mask = 0;
    const EntRows er{c->prm.E.p, pl->d_f_in_ref, pl->d_pos, d_cand};
    int rc = enqueue_forward(c, pl, er, s, w);
    if (rc == NGDB_OK) {
        ScoreArgs sa{};
        sa.act = w.act; sa.E = er.rows; sa.root_off = pl->d_root_off; sa.root_slot = pl->d_f_root;
        sa.pos = nullptr; sa.cand = d_cand; sa.B = hp.n_queries; sa.C = C; sa.d = c->cfg.d;
        sa.max_branch = std::max(1, hp.max_branch); sa.gamma = c->cfg.gamma; sa.score = d_scores;
        if (c->cfg.score_bf16) sa.E16 = ptr<uint16_t>(c->Eb);
        const hipError_t e = launch_score(sa, false, s);
        if (e == hipErrorInvalidValue) rc = fail(c, NGDB_ERR_UNSUPPORTED, "embedding width / union branch count too large for the scoring kernel");
        else if (e != hipSuccess) rc = fail(c, NGDB_ERR_HIP, std::string("scoring launch: ") + hipGetErrorString(e));
    }
    c->timing_mask = timing;
    if (rc != NGDB_OK) return rc;
    HIPCHK(c, hipEventRecord(pl->blob.last_use, s));
    return NGDB_OK;
}

int ngdb_rank_answers(ngdb_ctx_t* c, const ngdb_plan_t* pl, const int32_t* d_ans_off, const int32_t* d_ans,
                      int32_t n_ans, int32_t* d_rank, float* d_ans_dist, void* stream) {
    if (!c || !pl) return NGDB_ERR_ARG;
    if (!c->bound) return fail(c, NGDB_ERR_STATE, "parameters not bound");
    if (pl->n_entities != c->cfg.n_entities || !pl->d_blob)
        return fail(c, NGDB_ERR_ARG, "plan belongs to another configuration or was built without a device");
    if (n_ans < 0 || !d_ans_off || (n_ans > 0 && (!d_ans || !d_rank)))
        return fail(c, NGDB_ERR_ARG, "answer lists / rank output missing");
    if (pl->hp.n_queries > 65535) return fail(c, NGDB_ERR_UNSUPPORTED, "more than 65535 queries in one ranking call");
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool sem = c->cfg.d_sem > 0;
    c->have_grads = false;
    const bool reclaim = c->cfg.family == NGDB_FAMILY_VEC;     // as in ngdb_score
    int rc = reclaim ? size_forward_only(c, pl, 0) : size_workspace(c, pl, 0, false);
    if (rc != NGDB_OK) return rc;
    const int32_t* roots = reclaim ? pl->d_f_root : pl->d_root_slot;
    EntRows er{c->prm.E.p, reclaim ? pl->d_f_in_ref : pl->d_in_ref, pl->d_pos, nullptr};
    if (sem) {
        int32_t* e_src = nullptr;
        rc = prepare_entities(c, pl, nullptr, 0, s, s, &e_src, &er, reclaim);
        if (rc != NGDB_OK) return rc;
    }
    rc = enqueue_forward(c, pl, er, s, ctx_space(c, reclaim));
    if (rc != NGDB_OK) return rc;
    if (n_ans > 0) {
        const int N = c->cfg.n_entities, d = c->cfg.d, R = pl->hp.n_roots, B = pl->hp.n_queries;
        const float* box_off = c->cfg.family == NGDB_FAMILY_BOX ? ptr<float>(c->off) : nullptr;
        const int chunk = std::min(std::max(N, n_ans), 1 << 16);
        const int ld = (chunk + 3) & ~3;
        if ((rc = ensure(c, c->rank_dist, std::max<size_t>((size_t)R * ld * sizeof(float), 256), true)) != NGDB_OK) return rc;
        if ((rc = ensure(c, c->rank_count, (size_t)n_ans * 4, true)) != NGDB_OK) return rc;
        if (!d_ans_dist && (rc = ensure(c, c->rank_thr, (size_t)n_ans * 4, true)) != NGDB_OK) return rc;
        if (sem && (rc = ensure(c, c->rank_ef, (size_t)chunk * d * sizeof(float), true)) != NGDB_OK) return rc;
        float* thr = d_ans_dist ? d_ans_dist : ptr<float>(c->rank_thr);
        Timed tm(c, NGDB_TK_SCORE, s);
        HIPCHK(c, launch_fill_zero_i32(ptr<int32_t>(c->rank_count), n_ans, s));
        SemFuseArgs fa{};
        fa.H = c->prm.H_sem; fa.Wb = ptr<uint16_t>(c->Wb); fa.E = c->prm.E.p; fa.d = d; fa.ds = c->cfg.d_sem;
        fa.out = ptr<float>(c->rank_ef);
        // distance of every listed answer to its query, by the kernels of the all-entity pass
        // (the same arithmetic, so an answer compares equal to itself there)
        for (int a0 = 0; a0 < n_ans; a0 += chunk) {
            const int cnt = std::min(chunk, n_ans - a0);
            const float* rows = c->prm.E.p;
            const int32_t* ids = d_ans + a0;
            if (sem) {
                fa.ids = d_ans + a0; fa.id_base = 0; fa.n_rows = cnt;
                HIPCHK(c, launch_sem_fuse(fa, s));
                rows = ptr<float>(c->rank_ef);
                ids = nullptr;
            }
            HIPCHK(c, launch_l1_tile(ptr<float>(c->act), box_off, c->cfg.box_alpha, roots, R, rows, ids, cnt, d,
                                     ptr<float>(c->rank_dist), ld, s, c->cfg.score_bf16 ? ptr<uint16_t>(c->Eb) : nullptr));
            HIPCHK(c, launch_answer_dist(ptr<float>(c->rank_dist), ld, pl->d_root_off, d_ans_off, B, a0, cnt, thr, s));
        }
        // entities strictly closer than each answer, chunk by chunk
        for (int e0 = 0; e0 < N; e0 += chunk) {
            const int cnt = std::min(chunk, N - e0);
            const float* rows = c->prm.E.p + (size_t)e0 * d;
            if (sem) {
                fa.ids = nullptr; fa.id_base = e0; fa.n_rows = cnt;
                HIPCHK(c, launch_sem_fuse(fa, s));
                rows = ptr<float>(c->rank_ef);
            }
            HIPCHK(c, launch_l1_tile(ptr<float>(c->act), box_off, c->cfg.box_alpha, roots, R, rows, nullptr, cnt, d,
                                     ptr<float>(c->rank_dist), ld, s,
                                     c->cfg.score_bf16 ? ptr<uint16_t>(c->Eb) + (size_t)e0 * d : nullptr));
            HIPCHK(c, launch_count_less(ptr<float>(c->rank_dist), ld, pl->d_root_off, d_ans_off, thr, B, cnt,
                                        ptr<int32_t>(c->rank_count), s));
        }
        HIPCHK(c, launch_finish_rank(ptr<int32_t>(c->rank_count), thr, d_ans_off, B, n_ans, d_rank, s));
    }
    HIPCHK(c, hipEventRecord(pl->blob.last_use, s));
    return NGDB_OK;
}

int ngdb_rank_metrics(const int32_t* d_rank, const int32_t* d_ans_off, const int32_t* d_n_take, int32_t n_queries,
                      float* d_out, void* stream) {
    if (!d_ans_off || !d_out || n_queries < 0 || (n_queries > 0 && !d_rank)) return NGDB_ERR_ARG;
    const hipError_t e = launch_rank_metrics(d_rank, d_ans_off, d_n_take, n_queries, d_out,
                                             static_cast<hipStream_t>(stream));
    return e == hipSuccess ? NGDB_OK : NGDB_ERR_HIP;
}

int ngdb_debug_gemm(const float* A, const float* B, float* C, int32_t M, int32_t N, int32_t K, int32_t lda,
                    int32_t ldb, int32_t ldc, int32_t a_kcontig, int32_t b_kcontig, const float* bias, int32_t relu,
                    const float* mask, int32_t ldmask, const float* addend, int32_t ldadd, const int32_t* dst_row,
                    int32_t arith, void* stream) {
    if (!A || !B || !C || M < 0 || N < 0 || K < 0 || arith < 0 || arith > 2) return NGDB_ERR_ARG;
    GemmArgs g;
    g.A = A; g.B = B; g.C = C; g.M = M; g.N = N; g.K = K; g.lda = lda; g.ldb = ldb; g.ldc = ldc;
    g.a_kcontig = a_kcontig != 0; g.b_kcontig = b_kcontig != 0; g.bias = bias; g.relu = relu != 0;
    g.mask = mask; g.ldmask = ldmask; g.addend = addend; g.ldadd = ldadd; g.dst_row = dst_row;
    g.arith = arith;
    const hipError_t e = launch_gemm(g, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? NGDB_OK : (e == hipErrorInvalidValue ? NGDB_ERR_ARG : NGDB_ERR_HIP);
}

int ngdb_debug_mlp(const float* X, const float* W1, const float* b1, const float* W2, const float* b2, const float* mask,
                   float* H, float* Y, int32_t M, int32_t d, int32_t h, int32_t backward, int32_t* used, void* stream) {
    if (!X || !W1 || !W2 || !H || !Y || M < 1 || d < 4 || h < 4 || (d & 3) || (h & 3) || (backward && !mask)) return NGDB_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int kt = 2 * ((h + 31) / 32);
    const size_t w_elems = 2 * (pieces_elems(h, d) + pieces_elems(d, h));
    const size_t h_elems = (size_t)((M + 31) / 32) * kt * 1536;
    uint16_t* buf = nullptr;
    if (hipMalloc(&buf, (w_elems + h_elems) * sizeof(uint16_t)) != hipSuccess) return NGDB_ERR_OOM;
    PieceJobs J{};
    J.count = 2;
    J.job[0].W = W1; J.job[0].R = h; J.job[0].C = d;
    J.job[0].out_rk = buf; J.job[0].out_ck = buf + pieces_elems(h, d);
    J.job[1].W = W2; J.job[1].R = d; J.job[1].C = h;
    J.job[1].out_rk = J.job[0].out_ck + pieces_elems(d, h); J.job[1].out_ck = J.job[1].out_rk + pieces_elems(d, h);
    uint16_t* hp = buf + w_elems;
    GemmArgs first, second;
    first.A = X; first.lda = d; first.M = M; first.N = h; first.K = d; first.C = H; first.ldc = h;
    second.A = H; second.lda = h; second.M = M; second.N = d; second.K = h; second.C = Y; second.ldc = d;
    first.arith = second.arith = GEMM_SPLIT;
    first.c_pieces = hp; first.c_kt = kt;
    if (!backward) {
        first.B = W1; first.ldb = d; first.bias = b1; first.relu = true; first.b_pieces = J.job[0].out_rk; first.b_kt = (d + 15) / 16;
        second.B = W2; second.ldb = h; second.bias = b2; second.b_pieces = J.job[1].out_rk; second.b_kt = (h + 15) / 16;
    } else {
        first.B = W2; first.ldb = h; first.b_kcontig = false; first.mask = mask; first.ldmask = h;
        first.b_pieces = J.job[1].out_ck; first.b_kt = (d + 15) / 16;
        second.B = W1; second.ldb = d; second.b_kcontig = false; second.b_pieces = J.job[0].out_ck; second.b_kt = (h + 15) / 16;
    }
    bool emitted = false;
    hipError_t e = launch_weight_pieces(J, s);
    if (e == hipSuccess) e = launch_gemm_group(&first, 1, s, nullptr, &emitted);
    if (e == hipSuccess && emitted) { second.a_pieces = hp; second.a_kt = kt; }
    if (e == hipSuccess) e = launch_gemm_group(&second, 1, s, nullptr, nullptr);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    (void)hipFree(buf);
    if (used) *used = 1 | (emitted ? 2 : 0);
    return e == hipSuccess ? NGDB_OK : (e == hipErrorInvalidValue ? NGDB_ERR_ARG : NGDB_ERR_HIP);
}

int ngdb_debug_copy(void* d_dst, const void* d_src, size_t bytes, void* stream) {
    if (!d_dst || !d_src) return NGDB_ERR_ARG;
    const hipError_t e = launch_copy(d_dst, d_src, bytes, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? NGDB_OK : (e == hipErrorInvalidValue ? NGDB_ERR_ARG : NGDB_ERR_HIP);
}

int ngdb_debug_stream(int32_t mode, void* d_dst, const void* d_src, size_t bytes, const int32_t* d_rows, int64_t n_rows,
                      int32_t row_floats, void* stream) {
    if (!d_dst || (mode != NGDB_STREAM_WRITE && mode != NGDB_STREAM_UPDATE && mode != NGDB_STREAM_UPDATE_NT && !d_src)) return NGDB_ERR_ARG;
    const hipError_t e = launch_stream_pattern(mode, d_dst, d_src, bytes, d_rows, n_rows, row_floats,
                                               static_cast<hipStream_t>(stream));
    return e == hipSuccess ? NGDB_OK : (e == hipErrorInvalidValue ? NGDB_ERR_ARG : NGDB_ERR_HIP);
}

int ngdb_set_timing(ngdb_ctx_t* c, uint32_t class_mask) {
    if (!c) return NGDB_ERR_ARG;
    c->timing_mask = class_mask & ((1u << NGDB_TK_COUNT) - 1u);
    return NGDB_OK;
}

int ngdb_get_timing(ngdb_ctx_t* c, ngdb_timing* out, int reset) {
    if (!c || !out) return NGDB_ERR_ARG;
    HIPCHK(c, hipDeviceSynchronize());
    for (const ngdb_ctx_s::Bracket& b : c->brackets) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, b.a, b.b) == hipSuccess) {
            c->timing.ms[b.cls] += ms;
            c->timing.brackets[b.cls] += 1;
            if (b.route >= 0) {
                c->timing.route_ms[b.cls][b.route] += ms;
                c->timing.route_launches[b.cls][b.route] += 1;
                c->timing.route_flop[b.cls][b.route] += b.flop;
            }
        }
        c->spare_events.push_back(b.a);
        c->spare_events.push_back(b.b);
    }
    c->brackets.clear();
    *out = c->timing;
    if (reset) c->timing = ngdb_timing{};
    return NGDB_OK;
}

int ngdb_copy_to_host(void* h_dst, const void* d_src, size_t bytes) {
    if (bytes == 0) return NGDB_OK;
    if (!h_dst || !d_src) return NGDB_ERR_ARG;
    if (hipDeviceSynchronize() != hipSuccess) return NGDB_ERR_HIP;
    return hipMemcpy(h_dst, d_src, bytes, hipMemcpyDeviceToHost) == hipSuccess ? NGDB_OK : NGDB_ERR_HIP;
}

int64_t ngdb_debug_alloc_count(const ngdb_ctx_t* c) { return c ? c->n_alloc : -1; }

int64_t ngdb_step_count(const ngdb_ctx_t* c) { return c ? c->step : -1; }

const char* ngdb_strerror(int code) {
    switch (code) {
        case NGDB_OK: return "ok";
        case NGDB_ERR_ARG: return "invalid argument";
        case NGDB_ERR_UNSUPPORTED: return "unsupported query or configuration";
        case NGDB_ERR_RANGE: return "entity or relation id out of range";
        case NGDB_ERR_OOM: return "out of memory";
        case NGDB_ERR_HIP: return "HIP runtime error";
        case NGDB_ERR_STATE: return "call order error";
        default: return "unknown error";
    }
}

const char* ngdb_last_error(const ngdb_ctx_t* c) { return c ? c->err.c_str() : ""; }

}  // extern "C"
