// Shared declarations of the library's translation units (host side) and the
// small device helpers every kernel file uses.
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <string>
#include <utility>

#include "ngdb.h"

namespace ngdb {

constexpr int WAVE = 64;

// ---------------------------------------------------------------- device helpers
#if defined(__HIPCC__)
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, WAVE);
    return v;
}
__device__ __forceinline__ int lane_id() { return threadIdx.x & (WAVE - 1); }
__device__ __forceinline__ float sgn(float x) { return (float)((x > 0.f) - (x < 0.f)); }
// bf16 bit patterns <-> fp32 (round to nearest, ties to even)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) {
    const uint32_t b = __float_as_uint(x);
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ float bf16_round_f32(float x) { return __uint_as_float(f32_to_bf16_bits(x) << 16); }
// 4 consecutive bf16 values (8 bytes) -> float4
__device__ __forceinline__ float4 bf16x4_to_f32(uint2 v) {
    return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xFFFF0000u), __uint_as_float(v.y << 16),
                       __uint_as_float(v.y & 0xFFFF0000u));
}
// Sum over the 64 lanes of a wavefront on the vector ALU alone (data-parallel primitives: adds inside
// quads, inside rows of 16 lanes, then across the four rows through row broadcasts), returned in
// every lane.  No LDS round trips: a chain of six ds_bpermute exchanges costs several hundred
// cycles of latency per sum.  Fixed summation order.
__device__ __forceinline__ float wave_sum_dpp(float v) {
#define NGDB_DPP_ADD(ctrl, rows)                                                                        \
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), ctrl, rows, 0xf, false))
    NGDB_DPP_ADD(0xB1, 0xf);    // quad_perm [1,0,3,2]: lane ^ 1
    NGDB_DPP_ADD(0x4E, 0xf);    // quad_perm [2,3,0,1]: lane ^ 2
    NGDB_DPP_ADD(0x141, 0xf);   // row_half_mirror: the other quad of the half row
    NGDB_DPP_ADD(0x140, 0xf);   // row_mirror: the other half row -> every lane holds its row's sum
    NGDB_DPP_ADD(0x142, 0xa);   // row_bcast15 into rows 1 and 3: sums of rows 0+1 and 2+3
    NGDB_DPP_ADD(0x143, 0xc);   // row_bcast31 into rows 2 and 3: row 3 holds the total
#undef NGDB_DPP_ADD
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
// The value lane `l` holds, for an l that is the same in all lanes: a register read, where a
// shuffle with a per-lane index would go through LDS hardware.
__device__ __forceinline__ int32_t lane_value(int32_t v, int l) {
    return __builtin_amdgcn_readlane(v, __builtin_amdgcn_readfirstlane(l));
}
__device__ __forceinline__ float lane_value(float v, int l) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), __builtin_amdgcn_readfirstlane(l)));
}
// Hardware transcendental approximations (about 1 ulp each; the results they feed are held to 1e-4).
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ __forceinline__ float fast_sqrt(float x) { return __builtin_amdgcn_sqrtf(x); }
// exp(-a) for a >= 0
__device__ __forceinline__ float fast_exp_neg(float a) { return __builtin_amdgcn_exp2f(a * -1.44269504088896341f); }
// log(1 + e) for 0 <= e <= 1: the series where 1 + e would lose e's bits, else the hardware logarithm
__device__ __forceinline__ float fast_log1p_unit(float e) {
    const float series = e * (1.f - e * (0.5f - e * (1.f / 3.f)));
    const float direct = __builtin_amdgcn_logf(1.f + e) * 0.693147180559945309f;
    return e < 0.01f ? series : direct;
}
// sign(x) as -1, 0 or +1 in two instructions and without the condition register: x scaled by 2^252
// is 0 for 0, at least 2^103 in size for every other finite x (denormals included), or infinite;
// clamped to [-1, 1].  c * sign(x) then fuses into the accumulating multiply-add.
__device__ __forceinline__ float sign_unit(float x) {
    return __builtin_amdgcn_fmed3f(__builtin_ldexpf(x, 252), -1.f, 1.f);
}
__device__ __forceinline__ float signed_by(float c, float x) { return c * sign_unit(x); }
// log(1+exp(x)) and 1/(1+exp(-x)) without overflow
__device__ __forceinline__ float softplus_f(float x) { return fmaxf(x, 0.f) + log1pf(expf(-fabsf(x))); }
__device__ __forceinline__ float sigmoid_f(float x) {
    const float e = expf(-fabsf(x));
    return x >= 0.f ? 1.f / (1.f + e) : e / (1.f + e);
}
#endif

// ---------------------------------------------------------------- GEMM (gemm.hip)
// C[M,N] = A[M,K] * B[K,N] with fp32 MFMA.  Element (m,k) of A is at
// A[m*lda+k] if a_kcontig else A[k*lda+m]; element (k,n) of B is at B[n*ldb+k]
// if b_kcontig else B[k*ldb+n].  Epilogue, in this order: + bias[n]; relu;
// * (mask[m*ldmask+n] > 0); + addend[m*ldadd+n]; row m goes to C row
// dst_row[m] if dst_row else m.
// Fused gather (k-contiguous A only): if a_ref is set, row m of A is
// a_base0 + a_ref[m]*lda for a_ref[m] >= 0, else a_base1 + (-1-a_ref[m])*lda, plus
// row a_add_idx[m] of a_add if a_add_idx is set; the assembled rows are also
// written to a_copy (same leading dimension) if it is set.
struct GemmArgs {
    const int32_t* a_ref = nullptr;
    const float* a_base0 = nullptr;
    const float* a_base1 = nullptr;
    const int32_t* a_add_idx = nullptr;
    const float* a_add = nullptr;
    float* a_copy = nullptr;
    const float* A = nullptr;
    const float* B = nullptr;
    float* C = nullptr;
    int M = 0, N = 0, K = 0;
    int lda = 0, ldb = 0, ldc = 0;
    bool a_kcontig = true, b_kcontig = true;
    const float* bias = nullptr;
    bool relu = false;
    const float* mask = nullptr;
    int ldmask = 0;
    const float* addend = nullptr;
    int ldadd = 0;
    const int32_t* dst_row = nullptr;
    int arith = 0;                 // GEMM_AUTO / GEMM_FP32 / GEMM_SPLIT: how the products are formed
    const uint16_t* b_pieces = nullptr;
    int b_kt = 0;
    // The same for A (rows of A in blocks of 32: tile (m / 32, k / 16), a_kt tiles per block row), and
    // for the output, written once more in that form where c_pieces is given (c_kt tiles per block
    // row, at least 2 * ceil(N / 32); no dst_row) for the launch that reads it as its A operand.
    const uint16_t* a_pieces = nullptr;
    int a_kt = 0;
    uint16_t* c_pieces = nullptr;
    int c_kt = 0;
};
// GEMM_FP32: fp32 MFMA.  GEMM_SPLIT: every fp32 operand value as the exact sum of three bf16
// values, the six largest of the nine partial products on the bf16 MFMA with fp32 accumulation
// (what is left out is below 2^-23 of a product, about 2^-27 on average).  GEMM_AUTO: GEMM_SPLIT
// where it is faster, else GEMM_FP32.
constexpr int GEMM_AUTO = 0, GEMM_FP32 = 1, GEMM_SPLIT = 2;
hipError_t launch_gemm(const GemmArgs& a, hipStream_t s);
// Up to GEMM_MAX_GROUP independent contractions with the same operand layout in one
// launch (the operator groups of one depth, or the weight gradients of all types).
constexpr int GEMM_MAX_GROUP = 6;
struct GemmGroup {
    int count;
    int tile_start[GEMM_MAX_GROUP + 1];   // first workgroup of every problem
    GemmArgs p[GEMM_MAX_GROUP];
};
// *route (if given) receives the arithmetic the launch used: GEMM_FP32 or GEMM_SPLIT; *emitted (if
// given) whether the launch wrote c_pieces (only the kernels that read their B operand as pieces do,
// in launches of at most 256 small tiles, and only if every problem of the group asks for it).
hipError_t launch_gemm_group(const GemmArgs* problems, int count, hipStream_t s, int* route = nullptr, bool* emitted = nullptr);

// A row-major matrix W [R][C] as B operand of the bf16 MFMA block in both forms, each value split
// into three bf16 pieces, stored tile by tile (32 n x 16 k) in lane order and zero beyond the
// matrix: out_rk holds B[n = row][k = column] (ceil(R/32) x ceil(C/16) tiles), out_ck holds
// B[n = column][k = row] (ceil(C/32) x ceil(R/16) tiles).  C a multiple of 4.
constexpr int PIECE_MAX_JOBS = 6;
struct PieceJob {
    const float* W;
    uint16_t *out_rk, *out_ck;
    int R, C;
};
struct PieceJobs {
    int count;
    PieceJob job[PIECE_MAX_JOBS];
    int block0[PIECE_MAX_JOBS + 1];
};
inline size_t pieces_elems(int N, int K) { return (size_t)((N + 31) / 32) * ((K + 15) / 16) * 1536; }
hipError_t launch_weight_pieces(PieceJobs& jobs, hipStream_t s);

// ---------------------------------------------------------------- elementwise ops (ops.hip)
// Intersections of one level, one job per cardinality class: n members with k inputs each,
// rows j*n+i of X (inputs) and Att (logits).  Forward: out[i] = sum_j w_j x_j, w = softmax over
// the inputs per coordinate.  Backward: dAtt[j*n+i] = w_j*(dy*x_j - sum_l w_l dy x_l),
// Dx[j*n+i] = w_j*dy.
constexpr int INTER_MAX_JOBS = 8;
struct InterJob {
    const float *X, *Att, *dY;
    float *out, *dAtt, *Dx;
    int n, k;
    const int32_t* out_row;   // forward: member i is written to row out_row[i] of out (null: row i)
};
struct InterJobs {
    int count;
    int d;
    InterJob job[INTER_MAX_JOBS];
};
hipError_t launch_inter(const InterJobs& jobs, bool backward, hipStream_t s);
// Box family, offset part of the intersections (same job layout: X = the inputs' offsets, Att =
// the per-input outputs of the offset MLP).  Forward: out[i] = min_j x_j * sigmoid(mean_j att_j).
// Backward: dAtt[j*n+i] = dy * min * g(1-g) / k;  Dx[j*n+i] = dy * g for the first j attaining
// the minimum, 0 for the others.
hipError_t launch_box_offset(const InterJobs& jobs, bool backward, hipStream_t s);

// Box family, projections of one group: member i reads its input box through ref[i] (slot, or
// -1-entity: centre E[e], offset 0) and writes (c + Rc[rel[i]], o + relu(Ro[rel[i]])) to slot
// out_base + i.  Backward copies the gradient rows of slot out_base + i (centre and offset) to
// the input's gradient rows gslot[i].
struct BoxProjArgs {
    const int32_t *ref, *gslot, *rel;
    const float *E, *Rc, *Ro;
    float *act_c, *act_o, *dact_c, *dact_o;
    int n, d, out_base;
};
hipError_t launch_box_proj(const BoxProjArgs& a, bool backward, hipStream_t s);
// Both poolings of the box family's intersections in one launch: jobs flagged in gate_mask are
// offset jobs (launch_box_offset), the others centre jobs (launch_inter).  With has_proj the
// projections of a group of the same level (independent of the intersections) ride along as
// one more job.
struct BoxPoolJobs {
    InterJobs jobs;
    uint32_t gate_mask;
    int has_proj;
    BoxProjArgs proj;
};
hipError_t launch_box_pool(const BoxPoolJobs& jobs, bool backward, hipStream_t s);
// out[c] = sum_m X[m*ld + c], c < cols, for several matrices in one launch pair (fixed
// summation order); `part` is scratch of COLSUM_MAX_CHUNKS * cols floats per matrix
constexpr int COLSUM_MAX_CHUNKS = 128;
constexpr int COLSUM_MAX_JOBS = 6;
struct ColsumJob {
    const float* X;
    float* out;
    float* part;
    int rows, cols, ld;
    int chunk_rows, chunks;   // filled by launch_colsums
};
struct ColsumJobs {
    int count;
    ColsumJob job[COLSUM_MAX_JOBS];
};
// finish == false: only the partial sums (part[chunk * cols + c], chunks filled in); whoever
// consumes them adds the chunks up in colsum_final_kernel's order.
hipError_t launch_colsums(ColsumJobs& jobs, hipStream_t s, bool finish = true);
hipError_t launch_fill_zero(float* p, size_t n, hipStream_t s);
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s);
// calibration access patterns (ngdb_debug_stream)
hipError_t launch_stream_pattern(int mode, void* dst, const void* src, size_t bytes, const int32_t* rows, int64_t n_rows,
                                 int row_floats, hipStream_t s);

struct AdamHyper {
    float lr, beta1, beta2, eps;
    float bc1, bc2;   // 1 - beta^t for the step being applied
};
struct DenseAdamJob {
    float* p[13];
    float* m[13];
    float* v[13];
    const float* g[13];
    int64_t n[13];
    // chunks[t] > 0: g[t] holds that many partial column sums of n[t] columns each (launch_colsums
    // without its last step); they are added up here, the sum also stored in gsum[t]
    int chunks[13];
    float* gsum[13];
    int count;
};
hipError_t launch_dense_adam(const DenseAdamJob& job, const AdamHyper& hp, hipStream_t s);
// loss[0] = scale * sum_i terms[i]
hipError_t launch_loss_reduce(const float* terms, int n, float scale, float* loss, hipStream_t s);

// ---------------------------------------------------------------- scoring (score.hip)
struct ScoreArgs {
    const float* act;          // [n_slots, d]
    const float* E;            // [N, d]
    const int32_t* root_off;   // [B+1]
    const int32_t* root_slot;  // [n_roots]
    const int32_t* pos;        // [B] or null (then candidates only)
    const int32_t* cand;       // [B, C]
    int B, C, d, max_branch;
    float gamma;
    // outputs
    float* score;              // [B, C + (pos?1:0)]
    float* coef;               // same shape, dL/ds (training only)
    int32_t* win;              // same shape, root slot of the winning branch (training, if set)
    void* mask;                // if set (training with text features): [pairs, 64] sign codes of (winning branch - entity row), 2 bits per
                               // coordinate; lane l of a wavefront owns coordinates 4l..4l+3 of every
                               // 256-coordinate chunk: 1, 2 or 4 bytes per lane for d <= 256, 512, 1024
                               // (one of win / mask is set in training)
    float* dact;               // gradient arena (training only)
    float* loss_terms;         // [B] (training only)
    // box family (off set): act holds the centres, off the offsets [n_slots, d]; the distance is
    // sum relu(|e-c| - o) + alpha * sum min(|e-c|, o); doff receives dL/d(offset) of the roots
    const float* off = nullptr;
    float* doff = nullptr;
    float alpha = 0.f;
    // candidate rows from a bf16 copy of the table [N, d] (bit patterns) instead of E
    const uint16_t* E16 = nullptr;
};
hipError_t launch_score(const ScoreArgs& a, bool train, hipStream_t s);

// ---------------------------------------------------------------- ranking (rank.hip)
// dist[r*ld + e] = ||act[row_ids[r]] - Emat[id(e)]||_1 for r < n_rows, e < n_ent; id(e) = ent_ids[e] or e.
// With off (box family, 0 <= alpha <= 1): the box distance of (act row, off row) to the entity row.
// With Emat16 (bf16 bit patterns, same shape and indexing as Emat) the entity rows are read from it.
hipError_t launch_l1_tile(const float* act, const float* off, float alpha, const int32_t* row_ids, int n_rows,
                          const float* Emat, const int32_t* ent_ids, int n_ent, int d, float* dist, int ld, hipStream_t s,
                          const uint16_t* Emat16 = nullptr);
// filtered ranks of listed answers (answers of query q: ans_off[q]..ans_off[q+1]-1):
// thr[a] = distance of answer a (column a - a0 of dist) to its query, min over the query's rows
hipError_t launch_answer_dist(const float* dist, int ld, const int32_t* root_off, const int32_t* ans_off, int n_queries,
                              int a0, int cnt, float* thr, hipStream_t s);
// count[a] += #{entities e < n_ent of this chunk: min over rows dist[row, e] < thr[a]}
hipError_t launch_count_less(const float* dist, int ld, const int32_t* root_off, const int32_t* ans_off,
                             const float* thr, int n_queries, int n_ent, int32_t* count, hipStream_t s);
// rank[a] = 1 + count[a] - #{listed answers b of a's query: thr[b] < thr[a]}
hipError_t launch_finish_rank(const int32_t* count, const float* thr, const int32_t* ans_off, int n_queries, int n_ans,
                              int32_t* rank, hipStream_t s);
// out[0..3] = MRR, Hit@1, Hit@3, Hit@10 over the first n_take[q] (null: all) answers of every query
hipError_t launch_rank_metrics(const int32_t* rank, const int32_t* ans_off, const int32_t* n_take, int n_queries,
                               float* out, hipStream_t s);
hipError_t launch_fill_zero_i32(int32_t* p, int n, hipStream_t s);
// per query q: entity value = min over rows root_off[q]..root_off[q+1]-1 of dist; merges the
// k best (value, ent_base + e) of this chunk into out_dist/out_ids [n_queries, k]
hipError_t launch_topk_merge(const float* dist, int ld, const int32_t* root_off, int n_queries, int ent_base, int n_ent,
                             int k, bool first_chunk, float* out_dist, int32_t* out_ids, hipStream_t s);

// ---------------------------------------------------------------- index (index.hip)
struct IndexBuffers {   // device scratch owned by the context, sized for n_keys
    int32_t *keys_a, *keys_b, *vals_a, *vals_b;   // [n_keys]
    int32_t* hist;                                // [256 * n_tiles] + scan scratch
    int32_t* scan_tmp;                            // block sums
    int32_t *uniq, *seg_off;                      // [n_keys], [n_keys+1]
    int32_t* n_uniq;                              // device scalar
};
size_t index_hist_elems(int64_t n_keys);
size_t index_scan_tmp_elems(int64_t n_keys);
// keys = [head[0..n_head) | tail[0..n_tail)], values < key_bound.  On return
// (stream order) uniq/seg_off/n_uniq are filled and the contribution order is in
// *src_out (one of vals_a / vals_b).
hipError_t build_segment_index(const int32_t* head, int n_head, const int32_t* tail, int64_t n_tail,
                               int32_t key_bound, const IndexBuffers& buf, int32_t** src_out,
                               hipStream_t s);

// ---------------------------------------------------------------- tables (table.hip)
struct TableArgs {
    float *P, *Mo, *Vo;            // table and moments [rows, d]
    const int32_t* uniq;           // [n_uniq] row ids
    const int32_t* seg_off;        // [n_uniq+1]
    const int32_t* n_uniq_dev;     // device scalar
    int d;
    // contribution records in segment order, gradient rows before pairs inside a segment:
    // rec_row[t] < 0 is row -1-rec_row[t] of dact, added as it is; rec_row[t] >= 0 is a
    // (query, candidate) pair and the contribution is rec_coef[t] * sign: without mask,
    // rec_row[t] is a row of act and sign = sign(act row - table row); with mask (text
    // features) it is the pair number and the signs are the pair's entry of mask (layout:
    // ScoreArgs::mask).  rec_coef may be null if all records are gradient rows.
    const float* rec_coef;
    const int32_t* rec_row;
    const float* dact;
    const float* act;
    const void* mask;              // set together with g_bf16
    float* g_out;                  // if set: write gradients [n_uniq, d] instead of updating
    // text-feature fusion: the row gradient is also left in g_bf16 [n_uniq, d] (bf16 bit
    // patterns) for the gradient of the projection
    uint16_t* g_bf16 = nullptr;
    // box family: pair records carry rows of act (centres) and off (offsets); the contribution is
    // rec_coef * w * sign(centre - table row), w = 1 where |centre - row| > offset, else alpha
    const float* off = nullptr;
    float alpha = 0.f;
    // the row's gradient is multiplied by [table row > 0] (a table that is used through relu)
    bool relu_gate = false;
    // bf16 copy of the table [rows, d] that the scoring pass reads: pair signs are taken against
    // the rounded row, and the updated row is rounded into the copy
    uint16_t* shadow = nullptr;
    // the table and its moments are far larger than the caches: their rows move with non-temporal
    // loads and stores (single-table launches only)
    bool streaming = false;
};
// sorted contribution numbers -> records: c < n_rowsrc is gradient row row_base + c,
// otherwise a (query, candidate) pair in the order [B positives | B*K negatives]
// (win: winning rows per pair -> records carry act rows; null -> records carry pair numbers).
// With loss_terms [B] the same launch also writes loss[0] = loss_scale * sum of the terms.
hipError_t launch_resolve(const int32_t* src, int64_t n, int n_rowsrc, int row_base, int B, int K, const float* coef,
                          const int32_t* win, float* rec_coef, int32_t* rec_row, const float* loss_terms,
                          float loss_scale, float* loss, hipStream_t s);
// Up to two small plain tables of the same width (no text features, box weights or bf16 copy: the
// relation tables), updated by extra workgroups of the main table's launch (meant for small steps).
struct TableTail {
    int main_blocks;
    int blocks[2];
    TableArgs job[2];
};
// small[0..n_small): such tables, each of at most small_rows touched rows.
hipError_t launch_table_update(const TableArgs& a, const AdamHyper& hp, hipStream_t s, const TableArgs* small = nullptr,
                               int n_small = 0, int small_rows = 0);

// ---------------------------------------------------------------- text-feature fusion (sem.hip)
hipError_t launch_cast_bf16(const float* x, uint16_t* y, int64_t n, hipStream_t s);
// inv[src[t]] = u for seg_off[u] <= t < seg_off[u+1]
hipError_t launch_inverse_index(const int32_t* src, const int32_t* seg_off, const int32_t* n_uniq_dev, int64_t n,
                                int32_t* inv, hipStream_t s);
// out[i] = in_ref[i] if it is a slot, else -1 - inv[in_gslot[i] - n_slots] (anchor -> its touched-row position)
hipError_t launch_translate_refs(const int32_t* in_ref, const int32_t* in_gslot, int n, int n_slots,
                                 const int32_t* inv, int32_t* out, hipStream_t s);
// out[u, :] = E[id(u), :] + Wb * H[id(u), :] for u < n_rows; id(u) = ids[u] or id_base + u
struct SemFuseArgs {
    const uint16_t* H;          // [N, ds] bf16
    const uint16_t* Wb;         // [d, ds] bf16
    const float* E;             // [N, d]
    const int32_t* ids;         // [n_rows] or null
    int64_t id_base;
    const int32_t* n_rows_dev;  // device scalar (then n_rows is an upper bound) or null
    int n_rows;
    int d, ds;                  // ds a multiple of 64
    float* out;                 // [n_rows, d]
};
hipError_t launch_sem_fuse(const SemFuseArgs& a, hipStream_t s);
// out[m, n] = sum_u G[u, m] * H[ids[u], n] over u < *n_rows_dev
struct SemWgradArgs {
    const uint16_t* H;
    const int32_t* ids;
    const uint16_t* G;          // [n_rows, d] bf16, d a multiple of 8
    const int32_t* n_rows_dev;
    int n_rows;                 // upper bound
    int d, ds;
    int n_splits;               // from sem_wgrad_splits
    float* partial;             // [n_splits, d, ds]
};
int sem_wgrad_splits(int64_t n_rows_bound, int d, int ds);
hipError_t launch_sem_wgrad(const SemWgradArgs& a, float* out, hipStream_t s);

}  // namespace ngdb
