/*
 * libngdb -- one operator-level training step of a neural graph database on one
 * MI355X (gfx950).  C boundary: plain pointers and sizes, no C++ or torch types.
 *
 * The step follows the paper's operator-level training loop (Alg. 1): a batch
 * of first-order-logic queries of mixed shapes is decomposed into a DAG of
 * atomic operators (Sec. 4.1 "Graph Decomposition"), operators of one type that
 * are ready at the same depth are executed as one batch with that type's
 * shared parameters (Sec. 4.1 "Batched Execution"), intersections are split by
 * input count (Sec. 4.3, equivalence classes C_k), the objective is evaluated
 * for all positive and negative candidates at once with gather/scatter
 * offsets computed ahead of time (Sec. 4.2), gradients flow back through the
 * same groups in reverse, and one Adam step ends it (Alg. 1, last line).
 *
 * Model (the paper names the operators but prints no formulas; these are the
 * definitions of the workloads this library is measured on):
 *   projection    y = W2 relu(W1 (x + R[r]) + b1) + b2        W1 [h,d], W2 [d,h]
 *   negation      y = V2 relu(V1 x + c1) + c2
 *   intersection  a_k = U2 relu(U1 x_k + u1) + u2; w = softmax over the k inputs
 *                 (per coordinate); y = sum_k w_k * x_k
 *   union         disjunctive normal form; score = max over branches
 *   score         s(q,e) = gamma - min_b ||y_b - E[e]||_1
 *   loss          1/(2B) sum_i [ -log sig(s(q_i,pos_i)) - 1/K sum_j log sig(-s(q_i,neg_ij)) ]
 *   entity row    with text features (d_sem > 0) every entity row that is read --
 *                 anchors, positives, negatives, ranking -- is
 *                 Ef[e] = E[e] + bf16(Wp) H_sem[e]  (Sec. 4.4: cached encoder
 *                 outputs, gathered per batch, linear projection to width d);
 *                 bf16 products accumulated in fp32; H_sem is frozen, Wp is kept
 *                 in fp32, rounded to bf16 for every step and trained with Adam
 *   optimiser     Adam; dense on the MLP tensors, row-sparse (lazy) on E and R:
 *                 a table row is updated only in steps in which it received a
 *                 gradient contribution; the bias correction uses the global step.
 *
 * Second operator family (cfg.family = NGDB_FAMILY_BOX): box embeddings, one of the
 * backbones the paper trains on the framework (Sec. 5.1 "Backbone models", Q2B); the
 * decomposition, scheduling, objective and optimiser are the ones above, the operators are
 *   state         a box (c, o), centre and non-negative offset, both of width d
 *   anchor        (E[e], 0)
 *   projection    (c + R[r], o + relu(Ro[r]))                  no MLP
 *   intersection  centre: as above (U1 u1 U2 u2 on the centres);
 *                 offset: o = min_k o_k * sigmoid(mean_k (V2 relu(V1 o_k + c1) + c2))
 *   negation      not available: ngdb_plan returns NGDB_ERR_UNSUPPORTED
 *   score         s(q,e) = gamma - min_b [ ||relu(|E[e]-c_b| - o_b)||_1
 *                                          + box_alpha * ||min(|E[e]-c_b|, o_b)||_1 ]
 *                 (a coordinate with |e-c| == o counts as inside)
 *   tensors       E, R, Ro [n_relations, d] (row-sparse Adam), V1 c1 V2 c2, U1 u1 U2 u2;
 *                 W1 b1 W2 b2, Wp and H_sem are not read.  An intersection input must be
 *                 an operator output (true of every pattern of Sec. 3.1).
 *   not available in this family: text features (d_sem must be 0).
 *
 * Conventions
 *   - Every call returns 0 (NGDB_OK) or a negative error code; nothing throws
 *     or aborts across the boundary.  ngdb_last_error() gives the text.
 *   - "device" pointers are HIP device memory owned by the caller (row-major,
 *     contiguous, 16-byte aligned); the library borrows them.  "host" pointers
 *     are ordinary memory, borrowed only for the duration of the call.
 *   - The library keeps a private device workspace that grows on demand, or is allocated once
 *     by ngdb_create from declared maxima (ngdb_config.b_max_queries).
 *   - A stream argument is a hipStream_t passed as void*; NULL = the null
 *     stream.  Calls that take a stream are asynchronous with respect to the
 *     host unless stated otherwise.  One context must not be used from two
 *     host threads or two streams at the same time, with one exception:
 *     ngdb_plan and ngdb_plan_free may run on a second host thread while the
 *     first enqueues steps (the producer/consumer arrangement of Sec. 4.3:
 *     batch t+1 is planned while step t runs).
 *   - All index arrays are int32.  d and h must be multiples of 4.
 */
#ifndef NGDB_H
#define NGDB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NGDB_OK               0
#define NGDB_ERR_ARG         -1   /* null pointer, bad size, malformed query        */
#define NGDB_ERR_UNSUPPORTED -2   /* union below an intersection/negation, query
                                     without an operator, more than NGDB_MAX_CARD
                                     inputs, deeper than NGDB_MAX_LEVELS            */
#define NGDB_ERR_RANGE       -3   /* entity / relation id out of range              */
#define NGDB_ERR_OOM         -4   /* host or device allocation failed               */
#define NGDB_ERR_HIP         -5   /* a HIP runtime call failed                      */
#define NGDB_ERR_STATE       -6   /* call order: parameters not bound, no gradients */

#define NGDB_OP_ANCHOR 0   /* arg = entity id, no inputs            */
#define NGDB_OP_PROJ   1   /* arg = relation id, one input          */
#define NGDB_OP_INTER  2   /* 2..NGDB_MAX_CARD inputs               */
#define NGDB_OP_NEG    3   /* one input                             */
#define NGDB_OP_UNION  4   /* >= 1 inputs; removed by the planner   */

#define NGDB_MAX_CARD    8    /* inputs of one intersection             */
#define NGDB_MAX_LEVELS 64    /* operator depth of one query            */
#define NGDB_MAX_BRANCH 64    /* conjunctive branches of one query      */
#define NGDB_MAX_TOPK   16    /* entities returned per query by the all-entity ranking */

/* Order in which the operators of a batch are executed (Sec. 4.1 "Dynamic Scheduling").
 * LEVEL: all operators of one depth are one step; their classes (type, input count)
 *   run as the groups of one launch sequence.
 * MAX_FILL: the paper's ready-set loop (Alg. 1), resolved on the host: ready operators
 *   wait in one pool per class, ordered PROJ < INTER by input count < NEG; each step
 *   files the newly ready operators into their pools in node order, takes the pool
 *   with the most entries (fillness = entries / b_max, one b_max for all classes; ties
 *   to the first class) and runs its first min(entries, b_max) operators (b_max = 0:
 *   all of them); the loop ends when every pool is empty.  Values do not depend on
 *   the schedule; only the fp32 summation order of the weight gradients does.        */
#define NGDB_SCHED_LEVEL    0
#define NGDB_SCHED_MAX_FILL 1

/* Operator family: VEC = the vector model above, BOX = box embeddings. */
#define NGDB_FAMILY_VEC 0
#define NGDB_FAMILY_BOX 1

typedef struct ngdb_ctx_s ngdb_ctx_t;     /* opaque: configuration, workspace, streams */
typedef struct ngdb_plan_s ngdb_plan_t;   /* opaque: one planned batch                 */

typedef struct ngdb_config {
    int32_t n_entities;
    int32_t n_relations;
    int32_t d;             /* embedding width (multiple of 4)                        */
    int32_t h;             /* hidden width of the three MLPs (multiple of 4)         */
    int32_t d_sem;         /* width of the frozen text features, 0 = none; otherwise
                              a multiple of 64, and d a multiple of 8                */
    int32_t num_streams;   /* 1 = everything on the caller's stream; 2..4 = one
                              library-owned stream takes the work that does not depend
                              on the operator chain: the gradient index is built beside
                              the forward pass and the embedding tables are updated
                              beside the weight gradients (Sec. 4.3 "Multi-stream
                              Operator Execution"; the operator groups of one depth
                              already share one launch).  Results are identical, and
                              everything is joined to the caller's stream before the
                              call returns                                           */
    float gamma;
    float lr, beta1, beta2, eps;
    int32_t schedule;      /* NGDB_SCHED_* used by ngdb_plan                          */
    int32_t b_max;         /* largest batch of one Max-Fillness step, 0 = unbounded   */
    int32_t family;        /* NGDB_FAMILY_*                                           */
    float box_alpha;       /* weight of the inside distance (box family), 0..1        */
    int32_t score_bf16;    /* 1: the scoring and ranking passes read candidate rows from a
                              bf16 copy of E that the library keeps (half the gather
                              bytes): s(q,e) = gamma - min_b ||y_b - bf16(E[e])||_1,
                              rounded to nearest even; anchors and the optimiser use the
                              fp32 rows, the gradient of a rounded row goes to its fp32
                              row unchanged.  The copy is made by ngdb_bind_params and
                              kept current by ngdb_train_step: bind again after writing
                              to E from outside.  Vector family without text features
                              only; d a multiple of 8                                  */
    /* Declared maxima (all 0: the workspace grows on demand, and a step with a larger batch than
     * any before waits for the device, frees and allocates).  With b_max_queries > 0 ngdb_create
     * allocates the whole workspace and four plan buffers for batches of at most b_max_queries
     * queries with at most k_max negatives / candidates per query and at most
     * max_nodes_per_query nodes per query after the removal of unions (0 = 12, enough for the
     * patterns of Sec. 3.1); from then on ngdb_plan (with at most four plans alive),
     * ngdb_train_step and ngdb_score in candidate mode make no device allocation, no free and
     * never wait for the device, and a batch beyond the maxima is refused with NGDB_ERR_ARG.
     * The all-entity ranking calls and ngdb_forward_backward still allocate what only they need
     * on first use.                                                                           */
    int32_t b_max_queries;
    int32_t k_max;
    int32_t max_nodes_per_query;
} ngdb_config;

/* A trainable tensor with its Adam moments (all device, fp32, same shape). */
typedef struct ngdb_tensor {
    float* p;
    float* m;
    float* v;
} ngdb_tensor;

typedef struct ngdb_params {
    ngdb_tensor E;                  /* [n_entities, d]                               */
    ngdb_tensor R;                  /* [n_relations, d]                              */
    ngdb_tensor W1, b1, W2, b2;     /* projection   [h,d] [h] [d,h] [d]              */
    ngdb_tensor V1, c1, V2, c2;     /* negation                                      */
    ngdb_tensor U1, u1, U2, u2;     /* intersection attention                        */
    ngdb_tensor Wp;                 /* [d, d_sem] text projection, unused if d_sem=0 */
    const uint16_t* H_sem;          /* device [n_entities, d_sem] bf16 bit patterns,
                                       frozen (Sec. 4.4, GPU-resident semantic cache) */
    int64_t step;                   /* optimiser steps already applied to this state */
    ngdb_tensor Ro;                 /* [n_relations, d] relation offsets (box family only) */
} ngdb_params;

/* A batch of queries, host memory.  Query i owns nodes node_off[i]..node_off[i+1]-1;
 * inputs of node n are in_idx[in_off[n]..in_off[n+1]-1], positions local to the
 * query that must be smaller than n's own position; the root is the query's last
 * node (Sec. 3.1 query patterns; Sec. 4.1 DAG of atomic operators).              */
typedef struct ngdb_query_batch {
    int32_t n_queries;
    const int32_t* node_off;   /* [n_queries+1] */
    const uint8_t* op;         /* [n_nodes]  NGDB_OP_*                              */
    const int32_t* arg;        /* [n_nodes]                                         */
    const int32_t* in_off;     /* [n_nodes+1]                                       */
    const int32_t* in_idx;     /* [in_off[n_nodes]]                                 */
    const int32_t* pos;        /* [n_queries] positive answer entity                */
} ngdb_query_batch;

/* Read-only host view of a plan; valid until ngdb_plan_free().  Canonical form:
 *  - unions removed by DNF (branches in input order; projections above a union
 *    repeated per branch); nodes numbered in (query, branch, depth-first
 *    post-order) order; level(anchor)=0, level(op)=1+max level of its inputs
 *    (NGDB_SCHED_LEVEL) or the Max-Fillness step in which the operator runs
 *    (NGDB_SCHED_MAX_FILL; a step then holds exactly one group);
 *  - group = operator nodes with equal (level, type, input count), ordered by
 *    level, type (PROJ<INTER<NEG), input count; members in node order;
 *  - output slots type-major (projections, intersections, negations), in group
 *    order inside a type; gradient row of anchor a is n_slots + a;
 *  - in_ref[g_ref_off[g] + j*n + i] = input j of member i: slot (>=0) or
 *    -1-entity; in_gslot = the same as a gradient row;
 *  - MLP rows: PROJ/NEG rank inside the type; INTER group: g_mlp_base + j*n + i;
 *  - relation gradient index: stable grouping by relation id of the projections
 *    in slot order, r_src = gradient row of the projection's input;
 *  - f_row: see below.                                                          */
typedef struct ngdb_plan_view {
    int32_t n_queries, n_groups, n_levels, n_slots, n_anchor;
    int32_t n_proj, n_inter, n_neg, n_int_rows, n_roots, n_refs, n_r_uniq;
    int32_t peak_live;           /* most operator outputs alive at once if an output were freed as
                                    soon as its consumer has run (Sec. 4.3, eager reference
                                    counting; outputs of roots live until scoring)               */
    const int32_t* lvl_off;      /* [n_levels+2] groups of level l: lvl_off[l]..lvl_off[l+1]-1 */
    const int32_t* g_level;      /* [n_groups] ... */
    const int32_t* g_type;
    const int32_t* g_nin;
    const int32_t* g_n;
    const int32_t* g_out_base;
    const int32_t* g_mlp_base;
    const int32_t* g_ref_off;
    const int32_t* g_rel_off;    /* offset into rel, -1 if not a projection group */
    const int32_t* in_ref;       /* [n_refs] */
    const int32_t* in_gslot;     /* [n_refs] */
    const int32_t* rel;          /* [n_proj] */
    const int32_t* root_off;     /* [n_queries+1] */
    const int32_t* root_slot;    /* [n_roots] */
    const int32_t* anchor_ent;   /* [n_anchor] */
    const int32_t* pos;          /* [n_queries] */
    const int32_t* r_uniq;       /* [n_r_uniq] */
    const int32_t* r_seg_off;    /* [n_r_uniq+1] */
    const int32_t* r_src;        /* [n_proj] */
    /* Forward-only passes (ngdb_score, ngdb_rank_answers) reclaim an operator output as soon as its
     * consumer has run (Sec. 4.3, eager reference counting): f_row[s] is the storage row of output
     * slot s when, step by step, every output takes the lowest free row (in group and member order)
     * and the rows of the outputs a step consumed are free again after it; roots keep theirs.
     * n_f_rows = rows used = peak_live; f_step_rows = the most MLP rows one step needs per type
     * (projection, intersection inputs, negation): what the per-step buffers of such a pass hold. */
    int32_t n_f_rows;
    int32_t f_step_rows[3];
    const int32_t* f_row;        /* [n_slots] */
} ngdb_plan_view;

/* Device-side results of the last ngdb_forward_backward / ngdb_train_step on a
 * context (pointers into the private workspace, valid until the next call on
 * the context).  Gradients of table rows are compact: row i of gE belongs to
 * entity e_uniq[i].  The entity index is the stable grouping by entity id of
 * the contributions [anchors | positives | negatives row-major] (Sec. 4.2
 * "Efficient Tensor Indexing").                                                  */
typedef struct ngdb_grad_view {
    int32_t n_e_uniq, n_e_contrib, n_r_uniq, n_slots, n_pairs;
    const int32_t* e_uniq;      /* [n_e_uniq]                                    */
    const int32_t* e_seg_off;   /* [n_e_uniq+1]                                  */
    const int32_t* e_src;       /* [n_e_contrib] contribution numbers            */
    const float* gE;            /* [n_e_uniq, d]   (forward_backward only)       */
    const float* gR;            /* [n_r_uniq, d]   (forward_backward only)       */
    const float* g_mlp[12];     /* W1 b1 W2 b2 V1 c1 V2 c2 U1 u1 U2 u2           */
    const float* g_Wp;          /* [d, d_sem] or NULL                            */
    const float* act;           /* [n_slots, d] operator outputs by slot         */
    const float* dact;          /* [n_slots + n_anchor, d] dL/d(output) by slot, then dL/d(anchor row) */
    int32_t n_grad_rows;        /* n_slots + n_anchor                            */
    const float* pair_score;    /* [n_pairs] s(q_i, cand), pair = i*(K+1)+c, c=0 positive */
    const float* loss_terms;    /* [n_queries] per-query loss before the 1/(2B)  */
    /* box family only (NULL otherwise): */
    const float* gRo;           /* [n_r_uniq, d]   (forward_backward only)       */
    const float* off;           /* [n_slots, d] box offsets by slot (act holds the centres) */
    const float* doff;          /* [n_slots + n_anchor, d] dL/d(offset) by slot  */
    const uint16_t* e_shadow;   /* [n_entities, d] the bf16 copy of E (score_bf16), else NULL */
} ngdb_grad_view;

/* Create a context (allocates streams and a small workspace).  cfg: host. */
int ngdb_create(const ngdb_config* cfg, ngdb_ctx_t** out);
void ngdb_destroy(ngdb_ctx_t* ctx);

/* Record the caller's parameter / moment tensors (device) and the step count.
 * The struct is copied; the tensors stay the caller's and are updated in place
 * by ngdb_train_step.  Wp and H_sem are required iff d_sem > 0.                  */
int ngdb_bind_params(ngdb_ctx_t* ctx, const ngdb_params* params);

/* Queries -> operator-level frontiers and index arrays (Alg. 1, graph construction and
 * the pools of Sec. 4.1, resolved ahead of time level by level).  Host work
 * plus one upload; deterministic.  Ids are range-checked here (NGDB_ERR_RANGE).
 * The plan may be used for any number of steps on this context.                  */
int ngdb_plan(ngdb_ctx_t* ctx, const ngdb_query_batch* batch, ngdb_plan_t** out);
/* The host half of ngdb_plan alone (no context, no device, nothing uploaded):
 * the result can be exported and freed, not executed.                            */
int ngdb_plan_host(int32_t n_entities, int32_t n_relations, const ngdb_query_batch* batch,
                   ngdb_plan_t** out);
/* The same with an explicit schedule (ngdb_plan_host uses NGDB_SCHED_LEVEL). */
int ngdb_plan_host_sched(int32_t n_entities, int32_t n_relations, const ngdb_query_batch* batch,
                         int32_t schedule, int32_t b_max, ngdb_plan_t** out);
int ngdb_plan_export(const ngdb_plan_t* plan, ngdb_plan_view* out);
/* May be called right after the last step that uses the plan has been enqueued:
 * the plan's device buffer goes back to its context and is reused only after
 * that step has finished.  A plan that outlives its context loses its device
 * buffer there: it can still be exported and must still be freed, not executed. */
void ngdb_plan_free(ngdb_plan_t* plan);

/* One training step (Alg. 1, the scheduling loop and the optimiser step): forward over the plan's frontiers,
 * L1 scores of every query against its positive and its K negatives, loss,
 * backward, segmented scatter-add of the table gradients, Adam on every bound
 * tensor, step count + 1.  d_neg: device [n_queries, K] entity ids, K >= 1 (range is
 * the caller's responsibility: ids index E directly).  d_loss: device, 1 float,
 * written on the stream.  No host synchronisation except when the workspace
 * has to grow (first call with a larger batch).                                  */
int ngdb_train_step(ngdb_ctx_t* ctx, const ngdb_plan_t* plan, const int32_t* d_neg,
                    int32_t K, void* stream, float* d_loss);

/* The same without the optimiser: gradients are left in the workspace for
 * ngdb_get_grads().  Used by parity tests.                                       */
int ngdb_forward_backward(ngdb_ctx_t* ctx, const ngdb_plan_t* plan, const int32_t* d_neg,
                          int32_t K, void* stream, float* d_loss);
int ngdb_get_grads(ngdb_ctx_t* ctx, ngdb_grad_view* out);

/* Forward only (Sec. 3.2: rank entities by f(q,e)).
 *  candidate mode (d_cand != NULL): d_cand device [n_queries, C] entity ids, every one in
 *    [0, n_entities): they index E on the device and are not checked (as d_neg);
 *    d_scores device [n_queries, C] receives s(q_i, cand).
 *  all-entity mode (d_cand == NULL): for every query the topk entities of
 *    smallest L1 distance, ascending, ties to the lower id, into
 *    d_topk_ids [n_queries, topk] and d_topk_dist [n_queries, topk].             */
int ngdb_score(ngdb_ctx_t* ctx, const ngdb_plan_t* plan, const int32_t* d_cand, int32_t C,
               int32_t topk, float* d_scores, int32_t* d_topk_ids, float* d_topk_dist,
               void* stream);

/* ngdb_score in candidate mode for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and the same
 * results as ngdb_score(ctx, plan, d_cand, C, 0, d_scores, NULL, NULL, stream), but the forward
 * workspace (operator outputs, gathered inputs, hidden rows, attention logits) is a static array
 * of NGDB_NOALLOC_SCRATCH_MIB MiB that lives in the library's device image, one copy per GPU,
 * held until the process ends: the call makes no hipMalloc / hipFree, creates no events and
 * never waits for the device.  A batch whose workspace (ngdb_score_noalloc_bytes) exceeds the
 * array is refused with NGDB_ERR_ARG and a message in ngdb_last_error; vector family without
 * text features only (else NGDB_ERR_UNSUPPORTED).  All contexts and calls on one GPU share the
 * array: calls that overlap on one GPU (two streams, two threads, two contexts) race; the array
 * keeps the last call's contents, and nothing in it has to start at zero (every row is written
 * before it is read within a call).  The plan comes from ngdb_plan (which may allocate), the
 * parameters from ngdb_bind_params; d_cand and d_scores as for ngdb_score.                    */
#define NGDB_NOALLOC_SCRATCH_MIB 32
int ngdb_score_noalloc(ngdb_ctx_t* ctx, const ngdb_plan_t* plan, const int32_t* d_cand, int32_t C,
                       float* d_scores, void* stream);
/* Bytes of that workspace the plan needs (0 for NULL arguments). */
size_t ngdb_score_noalloc_bytes(const ngdb_ctx_t* ctx, const ngdb_plan_t* plan);

/* Evaluation (the filtered MRR / Hit@k the paper reports, Sec. 5.3): forward, then for
 * every listed answer of every query its filtered rank
 *     1 + #{entities that are not listed answers of the query and lie strictly closer}.
 * d_ans_off: device [n_queries+1], answers of query q are d_ans[d_ans_off[q]..d_ans_off[q+1]-1]
 * (device, n_ans ids in total; ranges are the caller's responsibility).  d_rank: device
 * [n_ans].  d_ans_dist: device [n_ans] or NULL, receives the L1 distance of every answer.
 * Distances are fp32: entities within rounding of an answer's distance may fall on
 * either side.  At most 65535 queries per call.                                        */
int ngdb_rank_answers(ngdb_ctx_t* ctx, const ngdb_plan_t* plan, const int32_t* d_ans_off,
                      const int32_t* d_ans, int32_t n_ans, int32_t* d_rank, float* d_ans_dist,
                      void* stream);
/* d_out[0] = mean reciprocal rank, d_out[1..3] = Hit@1, Hit@3, Hit@10 (device, 4 floats):
 * per query the mean over its first d_n_take[q] listed answers (NULL: all of them -- list
 * the answers to be scored first, the ones only to be filtered after them), then the mean
 * over the queries that have at least one.                                              */
int ngdb_rank_metrics(const int32_t* d_rank, const int32_t* d_ans_off, const int32_t* d_n_take,
                      int32_t n_queries, float* d_out, void* stream);

/* Online query sampler (App. "Stochastic Online Query Sampling"): host only, no device.
 * Batches are synthesised from the graph on the fly: a template (names out of 1p 2p 3p 2i 3i
 * ip pi 2u up 2in 3in inp pin pni, comma separated in template_names; weights: one per name
 * or NULL for uniform) is instantiated by a random walk backwards from the answer, with
 * rejection of walks that dead-end, of intersections with identical children and of queries
 * whose end point is not an answer (negation); the accepted end point is the positive.
 * head/rel/tail: host arrays of n_triples directed triples (copied).  Every query draws from
 * its own random stream (seed, batch number, query number): batches do not depend on
 * n_threads.  ngdb_sampler_next fills `batch` (and *neg: host [n_queries, K] uniform entity
 * ids; *template_id: host [n_queries] index into the names) with arrays owned by the sampler,
 * valid until the call after the next one on it; the batch can go straight to ngdb_plan.
 * After a call has returned batch t the sampler's own threads draw batch t+1 with the same
 * sizes in the background (three sets of buffers take turns), so a caller that asks for equal
 * sizes call after call waits only for what is not drawn yet; a call with other sizes drops
 * the batch read ahead and draws its own (the stream of batches is the same either way).
 * One sampler must not be used from two threads at once (it may run beside a context's
 * calls).                                                                                */
typedef struct ngdb_sampler_s ngdb_sampler_t;
int ngdb_sampler_create(int32_t n_entities, int32_t n_relations, int64_t n_triples,
                        const int32_t* head, const int32_t* rel, const int32_t* tail,
                        const char* template_names, const float* weights, uint64_t seed,
                        int32_t n_threads, ngdb_sampler_t** out);
int ngdb_sampler_next(ngdb_sampler_t* sampler, int32_t n_queries, int32_t K, ngdb_query_batch* batch,
                      const int32_t** neg, const uint8_t** template_id);
void ngdb_sampler_destroy(ngdb_sampler_t* sampler);
const char* ngdb_sampler_last_error(const ngdb_sampler_t* sampler);

/* The contraction kernel of the grouped MLPs on its own (used by tests):
 * C[M,N] = A[M,K] * B[K,N], all device fp32.  Element (m,k) of A is at
 * A[m*lda+k] if a_kcontig else A[k*lda+m]; element (k,n) of B at B[n*ldb+k] if
 * b_kcontig else B[k*ldb+n].  Then, in this order and each only if its pointer
 * is not NULL (relu: flag): + bias[n]; relu; zero where mask[m*ldmask+n] <= 0;
 * + addend[m*ldadd+n]; row m is stored at C row dst_row[m].  Leading dimensions
 * and the contiguous extents must be multiples of 4.  arith: 0 = as the training
 * step chooses, 1 = fp32 matrix instructions, 2 = every fp32 operand as the exact
 * sum of three bf16 values and the six largest of the nine partial products on
 * the bf16 matrix instructions with fp32 accumulation (the rest is below 2^-23 of
 * a product; always in the kernel's small tiles).                                 */
int ngdb_debug_gemm(const float* A, const float* B, float* C, int32_t M, int32_t N, int32_t K,
                    int32_t lda, int32_t ldb, int32_t ldc, int32_t a_kcontig, int32_t b_kcontig,
                    const float* bias, int32_t relu, const float* mask, int32_t ldmask,
                    const float* addend, int32_t ldadd, const int32_t* dst_row, int32_t arith,
                    void* stream);

/* The two launches of one operator MLP as the training step chains them when every operand
 * it prepares once is read as bf16 pieces (used by tests; Sec. 4.1 batched kernels).  All
 * pointers device fp32, row-major: W1 [h,d], W2 [d,h], H [M,h] and Y [M,d] outputs.
 *   backward = 0: H = relu(X W1^T + b1), Y = H W2^T + b2              (X [M,d])
 *   backward = 1: H = X W2 where mask > 0, else 0; Y = H W1           (X [M,d], mask [M,h])
 * Both weight matrices are split once into three bf16 pieces per value in both operand
 * forms; the first launch leaves H also as pieces where the step would (launches of at most
 * 256 tiles of 32 x 32 outputs), and the second then reads them as its A operand.  *used
 * (host, may be NULL): bit 0 weights read as pieces, bit 1 H read as pieces.  d and h
 * multiples of 4.  Allocates and frees its own scratch and waits for the stream.          */
int ngdb_debug_mlp(const float* X, const float* W1, const float* b1, const float* W2, const float* b2,
                   const float* mask, float* H, float* Y, int32_t M, int32_t d, int32_t h,
                   int32_t backward, int32_t* used, void* stream);

/* A plain device-to-device copy kernel (16 bytes per thread and step) of `bytes`
 * bytes, a multiple of 16: the reference point for scaling hardware traffic
 * counters and for the copy bandwidth of the machine.                           */
int ngdb_debug_copy(void* d_dst, const void* d_src, size_t bytes, void* stream);

/* Plain access patterns of the step's memory-bound kernels without their arithmetic, to measure
 * what the machine delivers for each (all pointers device; every call moves what it says once):
 *   NGDB_STREAM_COPY    d_dst[0..bytes) = d_src[0..bytes)                       (ngdb_debug_copy)
 *   NGDB_STREAM_READ    reads d_src[0..bytes); d_dst: 4 bytes, left untouched
 *   NGDB_STREAM_WRITE   writes d_dst[0..bytes)
 *   NGDB_STREAM_GATHER  reads row d_rows[i], i < n_rows, of the fp32 table d_src [*, row_floats], one
 *                       wavefront per row with the next row requested ahead (the scoring kernel's
 *                       candidate gather); d_dst: 4 bytes, left untouched; bytes ignored
 *   NGDB_STREAM_UPDATE  d_dst holds three fp32 tables [bytes/12/row_floats, row_floats] one after the
 *                       other; row d_rows[i] of each is read and written back (+1), one wavefront
 *                       per row (the table kernel's parameter / moment traffic)
 *   NGDB_STREAM_COPY_NT / NGDB_STREAM_UPDATE_NT   the same two with non-temporal loads and stores
 * bytes a multiple of 16; row_floats a multiple of 4, at most 1024; row ids are the caller's
 * responsibility.                                                                          */
#define NGDB_STREAM_COPY   0
#define NGDB_STREAM_READ   1
#define NGDB_STREAM_WRITE  2
#define NGDB_STREAM_GATHER 3
#define NGDB_STREAM_UPDATE 4
#define NGDB_STREAM_COPY_NT   5
#define NGDB_STREAM_UPDATE_NT 6
int ngdb_debug_stream(int32_t mode, void* d_dst, const void* d_src, size_t bytes, const int32_t* d_rows,
                      int64_t n_rows, int32_t row_floats, void* stream);

/* Kernel timing with HIP events recorded on the stream each kernel is launched
 * on.  Classes whose bit is set in class_mask are bracketed by an event pair at
 * every launch (NGDB_TK_INDEX brackets the whole index build); everything else
 * runs untouched.  ngdb_get_timing waits for the device, adds the elapsed times
 * of all brackets recorded since the last call, and optionally clears the sums. */
#define NGDB_TK_INDEX     0   /* gradient index: radix sort + segment heads        */
#define NGDB_TK_SEM       1   /* text features: fused rows and projection gradient */
#define NGDB_TK_GEMM_FWD  2   /* forward MLP contractions                          */
#define NGDB_TK_INTER     3   /* intersection pooling (box family: also projections
                                 and offsets), forward and backward                */
#define NGDB_TK_SCORE     4   /* fused L1 score + loss + dL/ds                     */
#define NGDB_TK_GEMM_BWD  5   /* data-gradient contractions                        */
#define NGDB_TK_WGRAD     6   /* weight-gradient contractions and bias sums        */
#define NGDB_TK_TABLE_E   7   /* entity table: segmented scatter-add + Adam        */
#define NGDB_TK_TABLE_R   8   /* relation table: the same                          */
#define NGDB_TK_ADAM      9   /* dense Adam on the MLP tensors                     */
#define NGDB_TK_COUNT    10
typedef struct ngdb_timing {
    double ms[NGDB_TK_COUNT];         /* summed elapsed time per class             */
    int64_t brackets[NGDB_TK_COUNT];  /* number of event pairs per class           */
    /* The contraction launches of a class (GEMM_FWD, GEMM_BWD, WGRAD), by the matrix instructions
     * they ran on: [.][0] fp32 instructions; [.][1] bf16 instructions on operands split into three
     * pieces, which execute six bf16 products per fp32 product.  route_flop counts algorithmic work,
     * 2*M*N*K per contraction.                                                              */
    double route_ms[NGDB_TK_COUNT][2];
    int64_t route_launches[NGDB_TK_COUNT][2];
    double route_flop[NGDB_TK_COUNT][2];
} ngdb_timing;
int ngdb_set_timing(ngdb_ctx_t* ctx, uint32_t class_mask);
int ngdb_get_timing(ngdb_ctx_t* ctx, ngdb_timing* out, int reset);

/* Synchronous device-to-host copy of `bytes` bytes (waits for the device). */
int ngdb_copy_to_host(void* h_dst, const void* d_src, size_t bytes);

/* Device allocations (hipMalloc / hipHostMalloc) this context has made so far, for tests of the
 * declared maxima of ngdb_config.                                                              */
int64_t ngdb_debug_alloc_count(const ngdb_ctx_t* ctx);

int64_t ngdb_step_count(const ngdb_ctx_t* ctx);
const char* ngdb_strerror(int code);
const char* ngdb_last_error(const ngdb_ctx_t* ctx);   /* text of the last failure on ctx */

#ifdef __cplusplus
}
#endif
#endif /* NGDB_H */
