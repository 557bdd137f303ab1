// Segmented scatter-add of embedding-table gradients fused with the row-sparse
// Adam update (Sec. 4.2: scatter through precomputed offsets; Alg. 1,
// OptimizerStep).  One wavefront owns one touched row: it reads the row once,
// sums the row's contributions in index order (no atomics), and writes the
// parameter and both moments back -- 6 row transfers per touched row, which is
// the algorithmic minimum for Adam.
//
// A contribution is either a gradient row of the arena (anchors; projections
// for the relation table) or a (query, candidate) pair of the scoring pass, for
// which dL/dE[e] = coef * sign(y_win - E[e]) is rebuilt from the 4-byte
// coefficient, the winning branch's embedding (cache resident) and the row the
// wavefront already holds.
#include "common.h"

namespace ngdb {
namespace {

template <int NCH>
__global__ __launch_bounds__(256) void table_kernel(const TableArgs a, const AdamHyper hp) {
    const int lane = threadIdx.x & 63;
    const int d4 = a.d >> 2;
    const int n_uniq = *a.n_uniq_dev;
    const int wave_global = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);

    for (int u = wave_global; u < n_uniq; u += n_waves) {
        const int32_t row = a.uniq[u];
        const int t0 = a.seg_off[u], t1 = a.seg_off[u + 1];
        float4* prow = reinterpret_cast<float4*>(a.P + (size_t)row * a.d);
        float4 p[NCH], g[NCH];
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            const int col = ch * 64 + lane;
            p[ch] = col < d4 ? prow[col] : zero4;
            g[ch] = zero4;
        }
        for (int t = t0; t < t1; ++t) {
            const int32_t c = a.src[t];
            if (a.src_is_row || c < a.n_rowsrc) {
                const float4* grow =
                    reinterpret_cast<const float4*>(a.dact + (size_t)(a.src_is_row ? c : a.row_base + c) * a.d);
#pragma unroll
                for (int ch = 0; ch < NCH; ++ch) {
                    const int col = ch * 64 + lane;
                    if (col < d4) {
                        const float4 x = grow[col];
                        g[ch].x += x.x; g[ch].y += x.y; g[ch].z += x.z; g[ch].w += x.w;
                    }
                }
            } else {
                int pair;
                const int r = c - a.n_rowsrc;
                if (r < a.B) {
                    pair = r * (a.K + 1);                      // the query's positive
                } else {
                    const int q = (r - a.B) / a.K;
                    pair = q * (a.K + 1) + 1 + ((r - a.B) - q * a.K);
                }
                const float coef = a.coef[pair];
                const float4* y = reinterpret_cast<const float4*>(a.act + (size_t)a.win[pair] * a.d);
#pragma unroll
                for (int ch = 0; ch < NCH; ++ch) {
                    const int col = ch * 64 + lane;
                    if (col < d4) {
                        const float4 yy = y[col];
                        g[ch].x += coef * sgn(yy.x - p[ch].x);
                        g[ch].y += coef * sgn(yy.y - p[ch].y);
                        g[ch].z += coef * sgn(yy.z - p[ch].z);
                        g[ch].w += coef * sgn(yy.w - p[ch].w);
                    }
                }
            }
        }
        if (a.g_out) {
            float4* orow = reinterpret_cast<float4*>(a.g_out + (size_t)u * a.d);
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const int col = ch * 64 + lane;
                if (col < d4) orow[col] = g[ch];
            }
            continue;
        }
        float4* mrow = reinterpret_cast<float4*>(a.Mo + (size_t)row * a.d);
        float4* vrow = reinterpret_cast<float4*>(a.Vo + (size_t)row * a.d);
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            const int col = ch * 64 + lane;
            if (col < d4) {
                float4 m = mrow[col], v = vrow[col];
                const float b1 = hp.beta1, b2 = hp.beta2;
#define NGDB_ADAM(F)                                                             \
    m.F = b1 * m.F + (1.f - b1) * g[ch].F;                                       \
    v.F = b2 * v.F + (1.f - b2) * g[ch].F * g[ch].F;                             \
    p[ch].F -= hp.lr * (m.F / hp.bc1) / (sqrtf(v.F / hp.bc2) + hp.eps);
                NGDB_ADAM(x) NGDB_ADAM(y) NGDB_ADAM(z) NGDB_ADAM(w)
#undef NGDB_ADAM
                mrow[col] = m;
                vrow[col] = v;
                prow[col] = p[ch];
            }
        }
    }
}

}  // namespace

hipError_t launch_table_update(const TableArgs& a, const AdamHyper& hp, hipStream_t s) {
    // the number of touched rows is only known on the device: a fixed grid walks them
    const int blocks = 256 * 8;
    if (a.d <= 256) hipLaunchKernelGGL(table_kernel<1>, dim3(blocks), dim3(256), 0, s, a, hp);
    else if (a.d <= 512) hipLaunchKernelGGL(table_kernel<2>, dim3(blocks), dim3(256), 0, s, a, hp);
    else if (a.d <= 1024) hipLaunchKernelGGL(table_kernel<4>, dim3(blocks), dim3(256), 0, s, a, hp);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace ngdb
