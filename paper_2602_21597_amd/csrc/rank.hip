// All-entity ranking (Sec. 3.2: answer a query by ranking every entity by
// f(q,e) = gamma - min_b ||y_b - E[e]||_1): L1 distances of every branch
// embedding to a chunk of entity rows, then a running top-k per query.
//
// The distance pass is bound by plain vector arithmetic (two VALU operations per
// coordinate: subtract, add-absolute; an L1 distance is not a contraction, so the
// matrix cores cannot help): a workgroup owns a 128 x 128 tile of (branch rows x
// entities), stages both operands k-major in LDS 16 coordinates at a time, and
// every lane accumulates an 8 x 8 block of distances in registers, so that one
// 16-byte LDS read feeds 32 accumulations.
//
// The selection pass keeps, per lane, the best KMAX (distance, id) pairs of the
// entities it scanned (a union query takes the minimum over its branch rows
// first), then merges the 256 sorted lists of the workgroup and the running
// result of earlier chunks by repeated workgroup-wide minimum.  Order is
// (distance, entity id), so equal distances rank the lower id first.
#include <climits>

#include "common.h"

namespace ngdb {
namespace {

constexpr int TQ = 128, TE = 128, DC = 16, LDT = 128 + 4;

// entity e of the tile is row ent_ids[e] of Emat if ent_ids is given, else row e.  The
// distance of a (row, entity) pair is summed by one lane over the coordinates in ascending
// order, so its value does not depend on where in a tile, or in which launch, the pair falls.
// BOX (box family): the row side is a box, centre from act and offset from off, and a coordinate
// contributes relu(a - o) + alpha * min(a, o) = max(alpha * a, a - (1 - alpha) * o), a = |e - c|;
// the offsets are staged already multiplied by (1 - alpha): five VALU operations per coordinate.
// Emat16 (if set): the entity rows are read from this bf16 copy of Emat.
template <bool BOX>
__global__ __launch_bounds__(256) void l1_tile_kernel(const float* __restrict__ act, const float* __restrict__ off,
                                                      float alpha, const int32_t* __restrict__ row_ids,
                                                      int n_rows, const float* __restrict__ Emat,
                                                      const uint16_t* __restrict__ Emat16,
                                                      const int32_t* __restrict__ ent_ids, int n_ent, int d,
                                                      float* __restrict__ dist, int ld) {
    __shared__ __attribute__((aligned(16))) float Ys[2][DC][LDT];
    __shared__ __attribute__((aligned(16))) float Es[2][DC][LDT];
    __shared__ __attribute__((aligned(16))) float Os[BOX ? 2 : 1][BOX ? DC : 1][LDT];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int e0 = blockIdx.x * TE, r0 = blockIdx.y * TQ;

    // loader: 128 rows x 16 coordinates = 512 float4, two per thread and operand
    const float* yrow[2];
    const float* orow[2];
    const float* erow[2];
    const uint16_t* erow16[2];
    int lrow[2], lkq[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int idx = tid + i * 256;
        lrow[i] = idx >> 2;
        lkq[i] = idx & 3;
        const int r = min(r0 + lrow[i], n_rows - 1);          // clamped rows are computed and never stored
        yrow[i] = act + (size_t)row_ids[r] * d;
        orow[i] = BOX ? off + (size_t)row_ids[r] * d : nullptr;
        const int ec = min(e0 + lrow[i], n_ent - 1);
        erow[i] = Emat + (size_t)(ent_ids ? ent_ids[ec] : ec) * d;
        erow16[i] = Emat16 ? Emat16 + (size_t)(ent_ids ? ent_ids[ec] : ec) * d : nullptr;
    }
    float4 ry[2], re[2], ro[2];
    const float shrink = 1.f - alpha;
    auto issue = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int kc = min(k0 + lkq[i] * 4, d - 4);
            ry[i] = *reinterpret_cast<const float4*>(yrow[i] + kc);
            re[i] = Emat16 ? bf16x4_to_f32(*reinterpret_cast<const uint2*>(erow16[i] + kc))
                           : *reinterpret_cast<const float4*>(erow[i] + kc);
            if (BOX) ro[i] = *reinterpret_cast<const float4*>(orow[i] + kc);
        }
    };
    auto stage = [&](int buf, int k0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            // coordinates past d contribute |0 - 0|
            const bool ok = k0 + lkq[i] * 4 < d;
            const float4 y = ok ? ry[i] : make_float4(0.f, 0.f, 0.f, 0.f);
            const float4 e = ok ? re[i] : make_float4(0.f, 0.f, 0.f, 0.f);
            Ys[buf][lkq[i] * 4 + 0][lrow[i]] = y.x; Ys[buf][lkq[i] * 4 + 1][lrow[i]] = y.y;
            Ys[buf][lkq[i] * 4 + 2][lrow[i]] = y.z; Ys[buf][lkq[i] * 4 + 3][lrow[i]] = y.w;
            Es[buf][lkq[i] * 4 + 0][lrow[i]] = e.x; Es[buf][lkq[i] * 4 + 1][lrow[i]] = e.y;
            Es[buf][lkq[i] * 4 + 2][lrow[i]] = e.z; Es[buf][lkq[i] * 4 + 3][lrow[i]] = e.w;
            if (BOX) {
                const float4 o = ok ? ro[i] : make_float4(0.f, 0.f, 0.f, 0.f);
                Os[buf][lkq[i] * 4 + 0][lrow[i]] = shrink * o.x; Os[buf][lkq[i] * 4 + 1][lrow[i]] = shrink * o.y;
                Os[buf][lkq[i] * 4 + 2][lrow[i]] = shrink * o.z; Os[buf][lkq[i] * 4 + 3][lrow[i]] = shrink * o.w;
            }
        }
    };

    float acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;

    const int nk = (d + DC - 1) / DC;
    issue(0);
    stage(0, 0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) issue((kt + 1) * DC);
#pragma unroll
        for (int k = 0; k < DC; ++k) {
            const float4 y0 = *reinterpret_cast<const float4*>(&Ys[buf][k][ty * 8]);
            const float4 y1 = *reinterpret_cast<const float4*>(&Ys[buf][k][ty * 8 + 4]);
            const float4 x0 = *reinterpret_cast<const float4*>(&Es[buf][k][tx * 8]);
            const float4 x1 = *reinterpret_cast<const float4*>(&Es[buf][k][tx * 8 + 4]);
            const float yv[8] = {y0.x, y0.y, y0.z, y0.w, y1.x, y1.y, y1.z, y1.w};
            const float ev[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
            if (BOX) {
                const float4 o0 = *reinterpret_cast<const float4*>(&Os[buf][k][ty * 8]);
                const float4 o1 = *reinterpret_cast<const float4*>(&Os[buf][k][ty * 8 + 4]);
                const float ov[8] = {o0.x, o0.y, o0.z, o0.w, o1.x, o1.y, o1.z, o1.w};
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float a = fabsf(yv[i] - ev[j]);
                        acc[i][j] += fmaxf(alpha * a, a - ov[i]);
                    }
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[i][j] += fabsf(yv[i] - ev[j]);
            }
        }
        if (kt + 1 < nk) stage(buf ^ 1, (kt + 1) * DC);
        __syncthreads();
    }

#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = r0 + ty * 8 + i;
        if (r >= n_rows) continue;
        float* out = dist + (size_t)r * ld + e0 + tx * 8;
        if (e0 + tx * 8 + 7 < n_ent) {
            *reinterpret_cast<float4*>(out) = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
            *reinterpret_cast<float4*>(out + 4) = make_float4(acc[i][4], acc[i][5], acc[i][6], acc[i][7]);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (e0 + tx * 8 + j < n_ent) out[j] = acc[i][j];
        }
    }
}

constexpr int KMAX = NGDB_MAX_TOPK;

__device__ __forceinline__ bool before(float d, int i, float d2, int i2) { return d < d2 || (d == d2 && i < i2); }

// one workgroup per query: merges the chunk's distances into the query's running top-k
__global__ __launch_bounds__(256) void topk_kernel(const float* __restrict__ dist, int ld, const int32_t* __restrict__ root_off,
                                                   int ent_base, int n_ent, int k, bool first_chunk,
                                                   float* __restrict__ out_dist, int32_t* __restrict__ out_ids) {
    __shared__ float ld_[256][KMAX + 1];
    __shared__ int li_[256][KMAX + 1];
    __shared__ float wd[4];
    __shared__ int wi[4];
    const int q = blockIdx.x, t = threadIdx.x;
    const int r0 = root_off[q], nb = root_off[q + 1] - r0;

    float bd[KMAX];
    int bi[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
        bd[j] = INFINITY;
        bi[j] = INT_MAX;
    }
    auto insert = [&](float dv, int id) {
        if (!before(dv, id, bd[KMAX - 1], bi[KMAX - 1])) return;
#pragma unroll
        for (int j = KMAX - 1; j >= 1; --j) {
            const bool shift = before(dv, id, bd[j - 1], bi[j - 1]);
            const bool here = !shift && before(dv, id, bd[j], bi[j]);
            const float nd = shift ? bd[j - 1] : (here ? dv : bd[j]);
            const int ni = shift ? bi[j - 1] : (here ? id : bi[j]);
            bd[j] = nd;
            bi[j] = ni;
        }
        if (before(dv, id, bd[0], bi[0])) {
            bd[0] = dv;
            bi[0] = id;
        }
    };
    if (!first_chunk && t < k) {
        const int id = out_ids[(size_t)q * k + t];
        if (id >= 0) insert(out_dist[(size_t)q * k + t], id);
    }
    for (int e = t; e < n_ent; e += 256) {
        float dv = dist[(size_t)r0 * ld + e];
        for (int b = 1; b < nb; ++b) dv = fminf(dv, dist[(size_t)(r0 + b) * ld + e]);
        insert(dv, ent_base + e);
    }
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
        ld_[t][j] = bd[j];
        li_[t][j] = bi[j];
    }
    ld_[t][KMAX] = INFINITY;
    li_[t][KMAX] = INT_MAX;
    int head = 0;
    for (int r = 0; r < k; ++r) {
        float cd = ld_[t][head];
        int ci = li_[t][head];
        float md = cd;
        int mi = ci;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const float od = __shfl_xor(md, off, 64);
            const int oi = __shfl_xor(mi, off, 64);
            if (before(od, oi, md, mi)) {
                md = od;
                mi = oi;
            }
        }
        __syncthreads();                 // wd / wi of the previous round have been read
        if ((t & 63) == 0) {
            wd[t >> 6] = md;
            wi[t >> 6] = mi;
        }
        __syncthreads();
        md = wd[0];
        mi = wi[0];
#pragma unroll
        for (int w = 1; w < 4; ++w)
            if (before(wd[w], wi[w], md, mi)) {
                md = wd[w];
                mi = wi[w];
            }
        if (ci == mi && cd == md && mi != INT_MAX) ++head;     // ids are unique: exactly one list advances
        if (t == 0) {
            out_dist[(size_t)q * k + r] = md;
            out_ids[(size_t)q * k + r] = mi == INT_MAX ? -1 : mi;
        }
    }
}

// ---------------------------------------------------------------- filtered ranks of listed answers
// query of answer a: largest q with ans_off[q] <= a
__device__ __forceinline__ int query_of_answer(const int32_t* __restrict__ ans_off, int n_queries, int a) {
    int lo = 0, hi = n_queries;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (ans_off[mid] <= a) lo = mid; else hi = mid;
    }
    return lo;
}

// thr[a] = min over the branch rows of a's query of dist[row, a - a0], a0 <= a < a0 + cnt
__global__ __launch_bounds__(256) void answer_dist_kernel(const float* __restrict__ dist, int ld,
                                                          const int32_t* __restrict__ root_off,
                                                          const int32_t* __restrict__ ans_off, int n_queries, int a0,
                                                          int cnt, float* __restrict__ thr) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= cnt) return;
    const int q = query_of_answer(ans_off, n_queries, a0 + i);
    float v = INFINITY;
    for (int r = root_off[q]; r < root_off[q + 1]; ++r) v = fminf(v, dist[(size_t)r * ld + i]);
    thr[a0 + i] = v;
}

constexpr int CNT_SLAB = 8192;    // entities per workgroup of the counting pass
constexpr int CNT_TILE = 256;     // answers whose counters a workgroup holds at once

// count[a] += number of entities of the slab strictly closer to a's query than thr[a].
// Grid (slabs, queries).  A wavefront compares 64 entities with one threshold at a time and
// counts by ballot; the per-wavefront counters live in LDS, one integer atomic per answer and
// workgroup reaches global memory (integer sums do not depend on the order).
__global__ __launch_bounds__(256) void count_less_kernel(const float* __restrict__ dist, int ld,
                                                         const int32_t* __restrict__ root_off,
                                                         const int32_t* __restrict__ ans_off,
                                                         const float* __restrict__ thr, int n_ent,
                                                         int32_t* __restrict__ count) {
    __shared__ float s_thr[CNT_TILE];
    __shared__ int32_t s_cnt[4][CNT_TILE];
    const int q = blockIdx.y;
    const int a_lo = ans_off[q], a_hi = ans_off[q + 1];
    if (a_lo >= a_hi) return;                                         // uniform
    const int r_lo = root_off[q], r_hi = root_off[q + 1];
    const int e_lo = blockIdx.x * CNT_SLAB, e_hi = min(n_ent, e_lo + CNT_SLAB);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int t0 = a_lo; t0 < a_hi; t0 += CNT_TILE) {
        const int nt = min(CNT_TILE, a_hi - t0);
        __syncthreads();
        for (int j = threadIdx.x; j < nt; j += 256) s_thr[j] = thr[t0 + j];
        for (int j = lane; j < nt; j += 64) s_cnt[wave][j] = 0;
        __syncthreads();
        for (int e = e_lo + threadIdx.x; e - (int)threadIdx.x < e_hi; e += 256) {   // whole wavefronts iterate together
            float v = INFINITY;                                       // entities past the end are closer to nothing
            if (e < e_hi)
                for (int r = r_lo; r < r_hi; ++r) v = fminf(v, dist[(size_t)r * ld + e]);
            for (int j = 0; j < nt; ++j) {
                const int c = __popcll(__ballot(v < s_thr[j]));
                if (lane == 0) s_cnt[wave][j] += c;
            }
        }
        __syncthreads();
        for (int j = threadIdx.x; j < nt; j += 256) {
            const int c = (s_cnt[0][j] + s_cnt[1][j]) + (s_cnt[2][j] + s_cnt[3][j]);
            if (c) atomicAdd(&count[t0 + j], c);
        }
    }
}

// rank[a] = 1 + count[a] - #{other listed answers b of the same query with thr[b] < thr[a]}
__global__ __launch_bounds__(256) void finish_rank_kernel(const int32_t* __restrict__ count,
                                                          const float* __restrict__ thr,
                                                          const int32_t* __restrict__ ans_off, int n_queries,
                                                          int n_ans, int32_t* __restrict__ rank) {
    const int a = blockIdx.x * blockDim.x + threadIdx.x;
    if (a >= n_ans) return;
    const int q = query_of_answer(ans_off, n_queries, a);
    const float t = thr[a];
    int closer = 0;
    for (int b = ans_off[q]; b < ans_off[q + 1]; ++b) closer += thr[b] < t ? 1 : 0;
    rank[a] = 1 + count[a] - closer;
}

// out[0] = mean reciprocal rank, out[1..3] = Hit@1, @3, @10: per query the mean over its first
// n_take[q] listed answers (all if n_take is null), then the mean over the queries that have one.
// One workgroup, fixed summation order.
__global__ __launch_bounds__(256) void rank_metrics_kernel(const int32_t* __restrict__ rank,
                                                           const int32_t* __restrict__ ans_off,
                                                           const int32_t* __restrict__ n_take, int n_queries,
                                                           float* __restrict__ out) {
    __shared__ float part[256][5];
    float acc[5] = {0.f, 0.f, 0.f, 0.f, 0.f};      // MRR, H@1, H@3, H@10, queries counted
    for (int q = threadIdx.x; q < n_queries; q += 256) {
        const int lo = ans_off[q];
        const int n = n_take ? min(n_take[q], ans_off[q + 1] - lo) : ans_off[q + 1] - lo;
        if (n <= 0) continue;
        float rr = 0.f, h1 = 0.f, h3 = 0.f, h10 = 0.f;
        for (int j = 0; j < n; ++j) {
            const int r = rank[lo + j];
            rr += 1.f / (float)r;
            h1 += r <= 1 ? 1.f : 0.f;
            h3 += r <= 3 ? 1.f : 0.f;
            h10 += r <= 10 ? 1.f : 0.f;
        }
        const float inv = 1.f / (float)n;
        acc[0] += rr * inv; acc[1] += h1 * inv; acc[2] += h3 * inv; acc[3] += h10 * inv; acc[4] += 1.f;
    }
    for (int k = 0; k < 5; ++k) part[threadIdx.x][k] = acc[k];
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off)
            for (int k = 0; k < 5; ++k) part[threadIdx.x][k] += part[threadIdx.x + off][k];
        __syncthreads();
    }
    if (threadIdx.x < 4) out[threadIdx.x] = part[0][4] > 0.f ? part[0][threadIdx.x] / part[0][4] : 0.f;
}

__global__ __launch_bounds__(256) void fill_zero_i32_kernel(int32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

}  // namespace

hipError_t launch_l1_tile(const float* act, const float* off, float alpha, const int32_t* row_ids, int n_rows,
                          const float* Emat, const int32_t* ent_ids, int n_ent, int d, float* dist, int ld, hipStream_t s,
                          const uint16_t* Emat16) {
    if (n_rows <= 0 || n_ent <= 0) return hipSuccess;
    if ((d & 3) || (ld & 3) || (off && !(alpha >= 0.f && alpha <= 1.f))) return hipErrorInvalidValue;
    dim3 grid((n_ent + TE - 1) / TE, (n_rows + TQ - 1) / TQ);
    if (off)
        hipLaunchKernelGGL((l1_tile_kernel<true>), grid, dim3(256), 0, s, act, off, alpha, row_ids, n_rows, Emat, Emat16,
                           ent_ids, n_ent, d, dist, ld);
    else
        hipLaunchKernelGGL((l1_tile_kernel<false>), grid, dim3(256), 0, s, act, off, alpha, row_ids, n_rows, Emat, Emat16,
                           ent_ids, n_ent, d, dist, ld);
    return hipGetLastError();
}

hipError_t launch_answer_dist(const float* dist, int ld, const int32_t* root_off, const int32_t* ans_off, int n_queries,
                              int a0, int cnt, float* thr, hipStream_t s) {
    if (cnt <= 0) return hipSuccess;
    hipLaunchKernelGGL(answer_dist_kernel, dim3((cnt + 255) / 256), dim3(256), 0, s, dist, ld, root_off, ans_off,
                       n_queries, a0, cnt, thr);
    return hipGetLastError();
}

hipError_t launch_count_less(const float* dist, int ld, const int32_t* root_off, const int32_t* ans_off,
                             const float* thr, int n_queries, int n_ent, int32_t* count, hipStream_t s) {
    if (n_queries <= 0 || n_ent <= 0) return hipSuccess;
    if (n_queries > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(count_less_kernel, dim3((n_ent + CNT_SLAB - 1) / CNT_SLAB, n_queries), dim3(256), 0, s, dist, ld,
                       root_off, ans_off, thr, n_ent, count);
    return hipGetLastError();
}

hipError_t launch_finish_rank(const int32_t* count, const float* thr, const int32_t* ans_off, int n_queries, int n_ans,
                              int32_t* rank, hipStream_t s) {
    if (n_ans <= 0) return hipSuccess;
    hipLaunchKernelGGL(finish_rank_kernel, dim3((n_ans + 255) / 256), dim3(256), 0, s, count, thr, ans_off, n_queries,
                       n_ans, rank);
    return hipGetLastError();
}

hipError_t launch_rank_metrics(const int32_t* rank, const int32_t* ans_off, const int32_t* n_take, int n_queries,
                               float* out, hipStream_t s) {
    hipLaunchKernelGGL(rank_metrics_kernel, dim3(1), dim3(256), 0, s, rank, ans_off, n_take, n_queries, out);
    return hipGetLastError();
}

hipError_t launch_fill_zero_i32(int32_t* p, int n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_zero_i32_kernel, dim3((n + 255) / 256), dim3(256), 0, s, p, n);
    return hipGetLastError();
}

hipError_t launch_topk_merge(const float* dist, int ld, const int32_t* root_off, int n_queries, int ent_base, int n_ent,
                             int k, bool first_chunk, float* out_dist, int32_t* out_ids, hipStream_t s) {
    if (n_queries <= 0) return hipSuccess;
    if (k < 1 || k > KMAX) return hipErrorInvalidValue;
    hipLaunchKernelGGL(topk_kernel, dim3(n_queries), dim3(256), 0, s, dist, ld, root_off, ent_base, n_ent, k,
                       first_chunk, out_dist, out_ids);
    return hipGetLastError();
}

}  // namespace ngdb
