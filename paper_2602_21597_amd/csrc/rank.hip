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

__global__ __launch_bounds__(256) void l1_tile_kernel(const float* __restrict__ act, const int32_t* __restrict__ row_ids,
                                                      int n_rows, const float* __restrict__ Emat, int n_ent, int d,
                                                      float* __restrict__ dist, int ld) {
    __shared__ __attribute__((aligned(16))) float Ys[2][DC][LDT];
    __shared__ __attribute__((aligned(16))) float Es[2][DC][LDT];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int e0 = blockIdx.x * TE, r0 = blockIdx.y * TQ;

    // loader: 128 rows x 16 coordinates = 512 float4, two per thread and operand
    const float* yrow[2];
    const float* erow[2];
    int lrow[2], lkq[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int idx = tid + i * 256;
        lrow[i] = idx >> 2;
        lkq[i] = idx & 3;
        const int r = min(r0 + lrow[i], n_rows - 1);          // clamped rows are computed and never stored
        yrow[i] = act + (size_t)row_ids[r] * d;
        erow[i] = Emat + (size_t)min(e0 + lrow[i], n_ent - 1) * d;
    }
    float4 ry[2], re[2];
    auto issue = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int kc = min(k0 + lkq[i] * 4, d - 4);
            ry[i] = *reinterpret_cast<const float4*>(yrow[i] + kc);
            re[i] = *reinterpret_cast<const float4*>(erow[i] + kc);
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
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i][j] += fabsf(yv[i] - ev[j]);
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

}  // namespace

hipError_t launch_l1_tile(const float* act, const int32_t* row_ids, int n_rows, const float* Emat, int n_ent, int d,
                          float* dist, int ld, hipStream_t s) {
    if (n_rows <= 0 || n_ent <= 0) return hipSuccess;
    if ((d & 3) || (ld & 3)) return hipErrorInvalidValue;
    dim3 grid((n_ent + TE - 1) / TE, (n_rows + TQ - 1) / TQ);
    hipLaunchKernelGGL(l1_tile_kernel, grid, dim3(256), 0, s, act, row_ids, n_rows, Emat, n_ent, d, dist, ld);
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
