// Segmented scatter-add of embedding-table gradients fused with the row-sparse
// Adam update (Sec. 4.2: scatter through precomputed offsets; Alg. 1,
// OptimizerStep).  One wavefront owns one touched row: it reads the row and its
// two moments once, sums the row's contributions in index order (no atomics),
// and writes all three back -- 6 row transfers per touched row, the algorithmic
// minimum for Adam.
//
// A contribution is either a gradient row of the arena (anchors; projections
// for the relation table) or a (query, candidate) pair of the scoring pass, for
// which dL/dE[e] = coef * sign(y_win - Ef[e]) is rebuilt from the 4-byte
// coefficient and either (plain tables) the winning branch's embedding, which is
// cache resident, and the row the wavefront already holds, or (text features,
// where the scored row Ef[e] is not the table row) the sign codes the scoring
// kernel left, 2 bits per coordinate.  Measured on the 2.5 M-entity shape, the
// first costs no HBM traffic at all, the second 2 x d/4 bytes per pair but
// spares reading the fused row.
// A small kernel first resolves the sorted contribution numbers into
// (coefficient, source) records laid out in segment order, so that the row
// kernel reads them with one coalesced load per 64 contributions instead of
// chasing dependent indices per contribution; inside a segment the gradient rows
// come first (anchors sort before positives and negatives), so the two kinds are
// walked by two branch-free loops with several sources in flight.
#include <algorithm>
#include "common.h"

namespace ngdb {
namespace {

// rec_row[t] >= 0: pair contribution (rec_coef[t] = dL/ds): the row of act of the pair's
// winning branch if win is given, else the pair number; rec_row[t] < 0: row -1-rec_row[t]
// of dact (gradient row, added as is).  With loss_terms, one more workgroup (the last) sums the
// B per-query loss terms into loss[0] = loss_scale * sum (the step's loss; a launch saved).
__global__ __launch_bounds__(256) void resolve_kernel(const int32_t* __restrict__ src, int64_t n, int n_rowsrc,
                                                      int row_base, int B, int K, const float* __restrict__ coef,
                                                      const int32_t* __restrict__ win, float* __restrict__ rec_coef,
                                                      int32_t* __restrict__ rec_row,
                                                      const float* __restrict__ loss_terms, float loss_scale,
                                                      float* __restrict__ loss) {
    const int walkers = (int)gridDim.x - (loss_terms ? 1 : 0);
    if ((int)blockIdx.x == walkers) {      // (only with loss_terms)
        __shared__ float part[4];
        float s = 0.f;
        for (int i = threadIdx.x; i < B; i += 256) s += loss_terms[i];
        s = wave_sum(s);
        if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
        __syncthreads();
        if (threadIdx.x == 0) loss[0] = loss_scale * ((part[0] + part[1]) + (part[2] + part[3]));
        return;
    }
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < n; t += (int64_t)walkers * blockDim.x) {
        const int32_t c = src[t];
        if (c < n_rowsrc) {
            rec_coef[t] = 0.f;
            rec_row[t] = -1 - (row_base + c);
        } else {
            const int r = c - n_rowsrc;
            int pair;
            if (r < B) {
                pair = r * (K + 1);                       // the query's positive
            } else {
                const int q = (r - B) / K;
                pair = q * (K + 1) + 1 + ((r - B) - q * K);
            }
            rec_coef[t] = coef[pair];
            rec_row[t] = win ? win[pair] : pair;
        }
    }
}

constexpr int G = 4;    // gradient rows in flight per wavefront
constexpr int GP = 8;   // pairs in flight per wavefront

__device__ __forceinline__ uint32_t bf16_bits(float x) { return f32_to_bf16_bits(x); }
// sign code (1 = +, 2 = -, 0 = none) -> c, -c, 0
__device__ __forceinline__ float signed_coef(uint32_t code, float c) { return code == 1u ? c : (code == 2u ? -c : 0.f); }

template <int NCH>
__device__ __forceinline__ uint32_t load_mask(const void* mask, size_t idx) {
    if (NCH == 1) return reinterpret_cast<const uint8_t*>(mask)[idx];
    if (NCH == 2) return reinterpret_cast<const uint16_t*>(mask)[idx];
    return reinterpret_cast<const uint32_t*>(mask)[idx];
}

// SEM (text-feature fusion): pair signs come from the sign codes, and the row gradient is
// also stored as bf16 (input of the projection's gradient).
// BOX (box family, entity table): a pair's sign is weighted 1 where the row lies outside the
// winning box in that coordinate and alpha where it lies inside.
// SH (plain vector family): the scoring pass reads a bf16 copy of the table; pair signs are taken
// against the rounded row and the updated row is rounded into the copy.
// NT (tables far larger than the caches: every touched row is read once and written once per step):
// parameter and moment rows move with non-temporal loads and stores.  Measured on the bare access
// pattern (three rows read and written back per touched row, 2 M of 2.5 M rows): 4.8 against
// 4.2 TB/s; on tables that fit the last-level cache the hint would push them out of it.
typedef float table_f4 __attribute__((ext_vector_type(4)));
template <bool NT>
__device__ __forceinline__ float4 row_load(const float4* p) {
    if (!NT) return *p;
    const table_f4 v = __builtin_nontemporal_load(reinterpret_cast<const table_f4*>(p));
    return make_float4(v[0], v[1], v[2], v[3]);
}
template <bool NT>
__device__ __forceinline__ void row_store(float4* p, float4 v) {
    if (!NT) { *p = v; return; }
    const table_f4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<table_f4*>(p));
}

// UPD: the pass applies Adam (known when the kernel is chosen; otherwise a.g_out decides at run time).
// With the choice open, the stores of either path count as "maybe issued" for the compiler, and the
// wait for the next row's parameter rows, requested before them, also waits for the stores.
template <int NCH, bool SEM, bool BOX, bool SH, bool NT = false, bool UPD = false>
__device__ __forceinline__ void table_rows(const TableArgs& a, const AdamHyper& hp, int wave_global, int n_waves) {
    const int lane = threadIdx.x & 63;
    const int d4 = a.d >> 2;
    const int n_uniq = *a.n_uniq_dev;
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    const bool update = UPD || a.g_out == nullptr;
    const float step1 = hp.lr / hp.bc1, ibc2 = 1.f / hp.bc2;   // lr / (1 - beta1^t), 1 / (1 - beta2^t): once per wavefront
    bool col_ok[NCH];
    int colc[NCH];
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
        col_ok[ch] = ch * 64 + lane < d4;
        colc[ch] = min(ch * 64 + lane, d4 - 1);       // clamped: loads never branch
    }

    // The wavefront's next row is requested while the current one is finished: its index entries
    // during the walk over the current segment, its parameter and moment rows before the update
    // arithmetic and the stores of the current row (the registers of the segment walk are free
    // then).  Past the last row the requests repeat it and are not used.
    int32_t row_n = 0;
    int t0_n = 0, t1_n = 0;
    float4 p_n[NCH], m_n[NCH], v_n[NCH];
#define NGDB_FETCH_INDEX(uu)                                   \
    do {                                                       \
        const int uc = min((uu), n_uniq - 1);                  \
        row_n = a.uniq[uc];                                    \
        t0_n = a.seg_off[uc];                                  \
        t1_n = a.seg_off[uc + 1];                              \
    } while (0)
#define NGDB_FETCH_ROWS()                                                                                      \
    _Pragma("unroll") for (int ch = 0; ch < NCH; ++ch) {                                                      \
        if (update || !SEM) p_n[ch] = row_load<NT>(reinterpret_cast<const float4*>(a.P + (size_t)row_n * a.d) + colc[ch]); \
        if (update) {                                                                                          \
            m_n[ch] = row_load<NT>(reinterpret_cast<const float4*>(a.Mo + (size_t)row_n * a.d) + colc[ch]);    \
            v_n[ch] = row_load<NT>(reinterpret_cast<const float4*>(a.Vo + (size_t)row_n * a.d) + colc[ch]);    \
        }                                                                                                      \
    }
    if (wave_global < n_uniq) {
        NGDB_FETCH_INDEX(wave_global);
        NGDB_FETCH_ROWS()
    }
    for (int u = wave_global; u < n_uniq; u += n_waves) {
        const int32_t row = row_n;
        const int t0 = t0_n, t1 = t1_n;
        float4* prow = reinterpret_cast<float4*>(a.P + (size_t)row * a.d);
        float4* mrow = reinterpret_cast<float4*>(a.Mo + (size_t)row * a.d);
        float4* vrow = reinterpret_cast<float4*>(a.Vo + (size_t)row * a.d);
        float4 p[NCH], m[NCH], v[NCH], g[NCH];
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            if (update || !SEM) p[ch] = p_n[ch];
            if (update) {
                m[ch] = m_n[ch];
                v[ch] = v_n[ch];
            }
            g[ch] = zero4;
        }
        NGDB_FETCH_INDEX(u + n_waves);
        // SH: the row as the scoring pass read it (rounded to bf16)
        float4 psr[SH ? NCH : 1];
        if (SH) {
#pragma unroll
            for (int ch = 0; ch < (SH ? NCH : 1); ++ch) {
                psr[ch].x = bf16_round_f32(p[ch].x); psr[ch].y = bf16_round_f32(p[ch].y);
                psr[ch].z = bf16_round_f32(p[ch].z); psr[ch].w = bf16_round_f32(p[ch].w);
            }
        }
#define NGDB_PS(ch) (SH ? psr[SH ? (ch) : 0] : p[ch])
        for (int base = t0; base < t1; base += 64) {
            const int n = min(64, t1 - base);
            const int tl = base + min(lane, n - 1);
            const int32_t my_row = a.rec_row[tl];
            const float my_coef = a.rec_coef ? a.rec_coef[tl] : 0.f;
            // gradient rows come first in a segment
            const int n_rows = __popcll(__ballot(my_row < 0 && lane < n));
            for (int j0 = 0; j0 < n_rows; j0 += G) {
                float4 x[G][NCH];
                float wgt[G];
#pragma unroll
                for (int q = 0; q < G; ++q) {
                    const int j = min(j0 + q, n_rows - 1);
                    const int32_t r = lane_value(my_row, j);
                    wgt[q] = j0 + q < n_rows ? 1.f : 0.f;        // padding entries of the last group add nothing
                    const float4* srow = reinterpret_cast<const float4*>(a.dact + (size_t)(-1 - r) * a.d);
#pragma unroll
                    for (int ch = 0; ch < NCH; ++ch) x[q][ch] = srow[colc[ch]];
                }
#pragma unroll
                for (int q = 0; q < G; ++q)
#pragma unroll
                    for (int ch = 0; ch < NCH; ++ch) {
                        g[ch].x += wgt[q] * x[q][ch].x;
                        g[ch].y += wgt[q] * x[q][ch].y;
                        g[ch].z += wgt[q] * x[q][ch].z;
                        g[ch].w += wgt[q] * x[q][ch].w;
                    }
            }
            if (!SEM) {
                for (int j0 = n_rows; j0 < n; j0 += G) {
                    float4 x[G][NCH], xo[BOX ? G : 1][NCH];
                    float cf[G];
#pragma unroll
                    for (int q = 0; q < G; ++q) {
                        const int j = min(j0 + q, n - 1);
                        const int32_t r = lane_value(my_row, j);
                        cf[q] = j0 + q < n ? lane_value(my_coef, j) : 0.f;
                        const float4* srow = reinterpret_cast<const float4*>(a.act + (size_t)r * a.d);
#pragma unroll
                        for (int ch = 0; ch < NCH; ++ch) x[q][ch] = srow[colc[ch]];
                        if (BOX) {
                            const float4* orow = reinterpret_cast<const float4*>(a.off + (size_t)r * a.d);
#pragma unroll
                            for (int ch = 0; ch < NCH; ++ch) xo[q][ch] = orow[colc[ch]];
                        }
                    }
#pragma unroll
                    for (int q = 0; q < G; ++q)
#pragma unroll
                        for (int ch = 0; ch < NCH; ++ch) {
                            if (BOX) {
                                const float ca = cf[q] * a.alpha;
                                const float dx = x[q][ch].x - NGDB_PS(ch).x, dy = x[q][ch].y - NGDB_PS(ch).y,
                                            dz = x[q][ch].z - NGDB_PS(ch).z, dw = x[q][ch].w - NGDB_PS(ch).w;
                                g[ch].x += signed_by(fabsf(dx) > xo[q][ch].x ? cf[q] : ca, dx);
                                g[ch].y += signed_by(fabsf(dy) > xo[q][ch].y ? cf[q] : ca, dy);
                                g[ch].z += signed_by(fabsf(dz) > xo[q][ch].z ? cf[q] : ca, dz);
                                g[ch].w += signed_by(fabsf(dw) > xo[q][ch].w ? cf[q] : ca, dw);
                            } else {
                                g[ch].x += signed_by(cf[q], x[q][ch].x - NGDB_PS(ch).x);
                                g[ch].y += signed_by(cf[q], x[q][ch].y - NGDB_PS(ch).y);
                                g[ch].z += signed_by(cf[q], x[q][ch].z - NGDB_PS(ch).z);
                                g[ch].w += signed_by(cf[q], x[q][ch].w - NGDB_PS(ch).w);
                            }
                        }
                }
                continue;
            }
            for (int j0 = n_rows; j0 < n; j0 += GP) {
                uint32_t bits[GP];
                float cf[GP];
#pragma unroll
                for (int q = 0; q < GP; ++q) {
                    const int j = min(j0 + q, n - 1);
                    const int32_t pair = lane_value(my_row, j);
                    cf[q] = j0 + q < n ? lane_value(my_coef, j) : 0.f;
                    bits[q] = load_mask<NCH>(a.mask, (size_t)pair * 64 + lane);
                }
#pragma unroll
                for (int q = 0; q < GP; ++q)
#pragma unroll
                    for (int ch = 0; ch < NCH; ++ch) {
                        const uint32_t b = bits[q] >> (8 * ch);
                        g[ch].x += signed_coef(b & 3u, cf[q]);
                        g[ch].y += signed_coef((b >> 2) & 3u, cf[q]);
                        g[ch].z += signed_coef((b >> 4) & 3u, cf[q]);
                        g[ch].w += signed_coef((b >> 6) & 3u, cf[q]);
                    }
            }
        }
        NGDB_FETCH_ROWS()
        if (SEM) {
            uint2* brow = reinterpret_cast<uint2*>(a.g_bf16 + (size_t)u * a.d);
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch)
                if (col_ok[ch])
                    brow[ch * 64 + lane] = make_uint2(bf16_bits(g[ch].x) | (bf16_bits(g[ch].y) << 16),
                                                      bf16_bits(g[ch].z) | (bf16_bits(g[ch].w) << 16));
        }
        if (a.relu_gate) {
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                g[ch].x = p[ch].x > 0.f ? g[ch].x : 0.f;
                g[ch].y = p[ch].y > 0.f ? g[ch].y : 0.f;
                g[ch].z = p[ch].z > 0.f ? g[ch].z : 0.f;
                g[ch].w = p[ch].w > 0.f ? g[ch].w : 0.f;
            }
        }
        // Stores without a lane condition (plain rows of tables that stay in the caches): the lanes
        // past the end of the row hold, through their clamped loads, the values of its last four
        // coordinates and write those once more.  Under a condition the stores may or may not be
        // issued as far as the compiler can tell, and the next row's wait for its parameter rows,
        // requested before them, becomes a wait for the stores too.  (With text features the sign
        // codes of those lanes are not the last column's; tables streamed from HBM are faster with
        // that wait: 4.32 against 4.49 ms at 2 M touched rows.)
        constexpr bool ALL_LANES = !SEM && !NT;
        if (!update) {
            float4* orow = reinterpret_cast<float4*>(a.g_out + (size_t)u * a.d);
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                if (ALL_LANES) orow[colc[ch]] = g[ch];
                else if (col_ok[ch]) orow[ch * 64 + lane] = g[ch];
            }
            continue;
        }
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            const int at = ALL_LANES ? colc[ch] : ch * 64 + lane;
            if (ALL_LANES || col_ok[ch]) {
                // (reciprocal and square root by the hardware approximations, about 1 ulp each: the
                // correctly rounded forms cost some sixty instructions per coordinate, which made
                // this memory-bound kernel wait for its own arithmetic)
                const float b1 = hp.beta1, b2 = hp.beta2;
#define NGDB_ADAM(F)                                                             \
    m[ch].F = b1 * m[ch].F + (1.f - b1) * g[ch].F;                               \
    v[ch].F = b2 * v[ch].F + (1.f - b2) * g[ch].F * g[ch].F;                     \
    p[ch].F -= (step1 * m[ch].F) * fast_rcp(fast_sqrt(v[ch].F * ibc2) + hp.eps);
                NGDB_ADAM(x) NGDB_ADAM(y) NGDB_ADAM(z) NGDB_ADAM(w)
#undef NGDB_ADAM
                row_store<NT>(mrow + at, m[ch]);
                row_store<NT>(vrow + at, v[ch]);
                row_store<NT>(prow + at, p[ch]);
                if (SH)
                    reinterpret_cast<uint2*>(a.shadow + (size_t)row * a.d)[at] =
                        make_uint2(bf16_bits(p[ch].x) | (bf16_bits(p[ch].y) << 16),
                                   bf16_bits(p[ch].z) | (bf16_bits(p[ch].w) << 16));
            }
        }
    }
}

#undef NGDB_PS
#undef NGDB_FETCH_INDEX
#undef NGDB_FETCH_ROWS

// Small steps (the launch, not the bytes, is what a table update costs there): the last
// main_blocks workgroups walk the rows of the main table; the ones before them those of up to two
// small plain tables of the same width (the relation tables, whose launches of their own would
// each add their latency to the step's tail).  Large tables keep table_kernel: there this
// kernel measured 3 % slower on the entity table than the launches it saves are worth.
// one table per launch
template <int NCH, bool SEM, bool BOX, bool SH, bool NT, bool UPD>
__global__ __launch_bounds__(256) void table_kernel(const TableArgs a, const AdamHyper hp) {
    table_rows<NCH, SEM, BOX, SH, NT, UPD>(a, hp, (int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6),
                                  (int)((gridDim.x * blockDim.x) >> 6));
}

// (box family at d <= 512: every pair re-reads two cached rows, and a fourth wavefront per SIMD
// costs more in cache misses than it hides: held at three)
template <int NCH, bool SEM, bool BOX, bool SH, bool UPD>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, (BOX && NCH == 2) ? 3 : 8)))
void table_group_kernel(const TableArgs a, const TableTail tail, const AdamHyper hp) {
    const int b = (int)blockIdx.x;
    const int mb = b - tail.blocks[0] - tail.blocks[1];
    if (mb >= 0) {
        // (the wavefront's number is the same in all its lanes: kept in a scalar register)
        table_rows<NCH, SEM, BOX, SH, false, UPD>(a, hp, __builtin_amdgcn_readfirstlane((int)((mb * blockDim.x + threadIdx.x) >> 6)),
                                                  tail.main_blocks * 4);
        return;
    }
    const int k = b < tail.blocks[0] ? 0 : 1;
    const int lb = k ? b - tail.blocks[0] : b;
    table_rows<NCH, false, false, false, false, UPD>(tail.job[k], hp,
                                                     __builtin_amdgcn_readfirstlane((int)((lb * blockDim.x + threadIdx.x) >> 6)),
                                                     tail.blocks[k] * 4);
}


}  // namespace

hipError_t launch_resolve(const int32_t* src, int64_t n, int n_rowsrc, int row_base, int B, int K, const float* coef,
                          const int32_t* win, float* rec_coef, int32_t* rec_row, const float* loss_terms,
                          float loss_scale, float* loss, hipStream_t s) {
    if (n <= 0) return loss_terms ? launch_loss_reduce(loss_terms, B, loss_scale, loss, s) : hipSuccess;
    const unsigned blocks = (unsigned)std::min<int64_t>((n + 255) / 256, 4096) + (loss_terms ? 1 : 0);
    hipLaunchKernelGGL(resolve_kernel, dim3(blocks), dim3(256), 0, s, src, n, n_rowsrc, row_base, B, K, coef, win,
                       rec_coef, rec_row, loss_terms, loss_scale, loss);
    return hipGetLastError();
}

hipError_t launch_table_update(const TableArgs& a, const AdamHyper& hp, hipStream_t s, const TableArgs* small,
                               int n_small, int small_rows) {
    // the number of touched rows is only known on the device: a fixed grid walks them
    TableTail tail{};
    tail.main_blocks = 256 * 8;
    if (n_small < 0 || n_small > 2 || (n_small > 0 && !small)) return hipErrorInvalidValue;
    for (int k = 0; k < n_small; ++k) {
        const TableArgs& t = small[k];
        if (t.d != a.d || t.g_bf16 || t.mask || t.off || t.shadow) return hipErrorInvalidValue;   // plain tables only
        tail.job[k] = t;
        tail.blocks[k] = std::max(1, std::min(256, (small_rows + 3) / 4));
    }
    const int blocks = tail.main_blocks + tail.blocks[0] + tail.blocks[1];
    if (a.d > 1024 || (a.g_bf16 != nullptr) != (a.mask != nullptr)) return hipErrorInvalidValue;
    const bool sem = a.g_bf16 != nullptr, box = a.off != nullptr;
    if (sem && (box || a.relu_gate)) return hipErrorInvalidValue;
    if (a.shadow && (sem || box)) return hipErrorInvalidValue;
    bool upd = a.g_out == nullptr;        // every table of the launch is updated in place
    for (int k = 0; k < n_small; ++k) upd = upd && small[k].g_out == nullptr;
#define NGDB_TABLE_U(NCH, SEM_, BOX_, SH_, UPD_)                                                              \
    do {                                                                                                      \
        if (n_small) hipLaunchKernelGGL((table_group_kernel<NCH, SEM_, BOX_, SH_, UPD_>), dim3(blocks), dim3(256), 0, s, a, tail, hp); \
        else if (a.streaming) hipLaunchKernelGGL((table_kernel<NCH, SEM_, BOX_, SH_, true, false>), dim3(tail.main_blocks), dim3(256), 0, s, a, hp); \
        else hipLaunchKernelGGL((table_kernel<NCH, SEM_, BOX_, SH_, false, UPD_>), dim3(tail.main_blocks), dim3(256), 0, s, a, hp); \
    } while (0)
#define NGDB_TABLE_V(NCH, SEM_, BOX_, SH_)                                                                     \
    do {                                                                                                      \
        if (upd) NGDB_TABLE_U(NCH, SEM_, BOX_, SH_, true);                                                    \
        else NGDB_TABLE_U(NCH, SEM_, BOX_, SH_, false);                                                       \
    } while (0)
#define NGDB_TABLE(NCH)                                   \
    do {                                                  \
        if (sem) NGDB_TABLE_V(NCH, true, false, false);   \
        else if (box) NGDB_TABLE_V(NCH, false, true, false); \
        else if (a.shadow) NGDB_TABLE_V(NCH, false, false, true); \
        else NGDB_TABLE_V(NCH, false, false, false);      \
    } while (0)
    if (a.d <= 256) NGDB_TABLE(1);
    else if (a.d <= 512) NGDB_TABLE(2);
    else NGDB_TABLE(4);
#undef NGDB_TABLE
#undef NGDB_TABLE_V
#undef NGDB_TABLE_U
    return hipGetLastError();
}

}  // namespace ngdb
