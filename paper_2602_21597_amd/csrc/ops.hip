// Memory-bound pieces around the grouped MLPs (the row gathers through the plan's
// precomputed references, Sec. 4.2 "Efficient Tensor Indexing", are fused into the
// contraction kernel's operand loads): the attention
// pooling of the intersection classes C_k (Sec. 4.3), column sums for the bias
// gradients, dense Adam (Alg. 1, OptimizerStep) and the final loss reduction.
#include "common.h"

namespace ngdb {
namespace {

// y_i = sum_j softmax_j(att_j)_c * x_j,c : one thread per (member, coordinate); the cardinality
// classes of one level are the jobs of one launch (blockIdx.y).  The loops over inputs run to
// the compile-time maximum under a predicate, so the per-input values stay in registers.
template <bool BWD>
__global__ __launch_bounds__(256) void inter_kernel(const InterJobs jobs) {
    const InterJob jb = jobs.job[blockIdx.y];
    const int d = jobs.d, n = jb.n, k = jb.k;
    const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (size_t)n * d) return;
    const int i = (int)(t / d), c = (int)(t % d);
    float a[NGDB_MAX_CARD], x[NGDB_MAX_CARD];
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < NGDB_MAX_CARD; ++j) {
        const size_t row = (size_t)min(j, k - 1) * n + i;
        a[j] = jb.Att[row * d + c];
        x[j] = jb.X[row * d + c];
        if (j < k) mx = fmaxf(mx, a[j]);
    }
    float den = 0.f;
#pragma unroll
    for (int j = 0; j < NGDB_MAX_CARD; ++j) {
        a[j] = j < k ? expf(a[j] - mx) : 0.f;
        den += a[j];
    }
    const float inv = 1.f / den;
    if (!BWD) {
        float y = 0.f;
#pragma unroll
        for (int j = 0; j < NGDB_MAX_CARD; ++j) y += a[j] * inv * x[j];
        jb.out[(size_t)(jb.out_row ? jb.out_row[i] : i) * d + c] = y;
    } else {
        const float dy = jb.dY[(size_t)i * d + c];
        float tall = 0.f;
#pragma unroll
        for (int j = 0; j < NGDB_MAX_CARD; ++j) tall += a[j] * inv * x[j] * dy;
#pragma unroll
        for (int j = 0; j < NGDB_MAX_CARD; ++j) {
            if (j < k) {
                const size_t row = (size_t)j * n + i;
                const float w = a[j] * inv;
                jb.dAtt[row * d + c] = w * (dy * x[j] - tall);
                jb.Dx[row * d + c] = w * dy;
            }
        }
    }
}

// column sums of up to COLSUM_MAX_JOBS matrices in a fixed order, two steps: partial
// sums over chunks of rows (one workgroup per 64 columns x chunk x matrix), then the
// chunks are added up per column
__global__ __launch_bounds__(256) void colsum_part_kernel(const ColsumJobs jobs) {
    __shared__ float red[4][64];
    const ColsumJob j = jobs.job[blockIdx.z];
    const int c = blockIdx.x * 64 + threadIdx.x;
    const int lo = blockIdx.y * j.chunk_rows, hi = min(j.rows, lo + j.chunk_rows);
    if (blockIdx.y >= j.chunks || blockIdx.x * 64 >= j.cols) return;     // uniform per workgroup
    float s0 = 0.f, s1 = 0.f;
    if (c < j.cols) {
        int m = lo + threadIdx.y;
        for (; m + 4 < hi; m += 8) {
            s0 += j.X[(size_t)m * j.ld + c];
            s1 += j.X[(size_t)(m + 4) * j.ld + c];
        }
        if (m < hi) s0 += j.X[(size_t)m * j.ld + c];
    }
    red[threadIdx.y][threadIdx.x] = s0 + s1;
    __syncthreads();
    if (threadIdx.y == 0 && c < j.cols)
        j.part[(size_t)blockIdx.y * j.cols + c] =
            (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}

__global__ __launch_bounds__(256) void colsum_final_kernel(const ColsumJobs jobs) {
    const ColsumJob j = jobs.job[blockIdx.y];
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= j.cols) return;
    // four running sums (fixed assignment of chunks to sums): the loads of a round do not wait for one another
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    int k = 0;
    for (; k + 4 <= j.chunks; k += 4) {
        s0 += j.part[(size_t)(k + 0) * j.cols + c];
        s1 += j.part[(size_t)(k + 1) * j.cols + c];
        s2 += j.part[(size_t)(k + 2) * j.cols + c];
        s3 += j.part[(size_t)(k + 3) * j.cols + c];
    }
    for (; k < j.chunks; ++k) s0 += j.part[(size_t)k * j.cols + c];
    j.out[c] = (s0 + s1) + (s2 + s3);
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float* p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0.f;
}

__global__ __launch_bounds__(256) void copy_kernel(float4* __restrict__ dst, const float4* __restrict__ src, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

// Calibration kernels: plain access patterns of the memory-bound kernels of the step, without their
// arithmetic, to measure what this machine delivers for each pattern.
__global__ __launch_bounds__(256) void read_kernel(const float4* __restrict__ src, size_t n, float* __restrict__ sink) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const float4 v = src[i];
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    const float t = (acc.x + acc.y) + (acc.z + acc.w);
    if (t == 1.2345e-30f) sink[0] = t;      // keeps the loads alive; never true for the calibration data
}
__global__ __launch_bounds__(256) void write_kernel(float4* __restrict__ dst, size_t n) {
    const float4 v = make_float4(1.f, 2.f, 3.f, 4.f);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = v;
}
// One wavefront per listed row of a [*, row_floats] table, float4 pieces 64 lanes apart, the next
// row requested before the current one is consumed (the scoring kernel's gather).
template <int NCH>
__global__ __launch_bounds__(256) void gather_rows_kernel(const float* __restrict__ table, const int32_t* __restrict__ rows,
                                                         int64_t n_rows, int row_floats, float* __restrict__ sink) {
    const int lane = threadIdx.x & 63, d4 = row_floats >> 2;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float4 cur[NCH], nxt[NCH];
    int64_t i = wave;
    if (i < n_rows) {
        const float4* r = reinterpret_cast<const float4*>(table + (size_t)rows[i] * row_floats);
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) cur[ch] = r[min(ch * 64 + lane, d4 - 1)];
    }
    for (; i < n_rows; i += n_waves) {
        const float4* r = reinterpret_cast<const float4*>(table + (size_t)rows[min(i + n_waves, n_rows - 1)] * row_floats);
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) nxt[ch] = r[min(ch * 64 + lane, d4 - 1)];
#pragma unroll
        for (int ch = 0; ch < NCH; ++ch) {
            acc.x += cur[ch].x; acc.y += cur[ch].y; acc.z += cur[ch].z; acc.w += cur[ch].w;
            cur[ch] = nxt[ch];
        }
    }
    const float t = (acc.x + acc.y) + (acc.z + acc.w);
    if (t == 1.2345e-30f) sink[0] = t;
}
// One wavefront per listed row: the row of each of three equally shaped tables (laid out one after
// the other) is read and written back changed (the table kernel's traffic without its gradients).
typedef float ops_f4 __attribute__((ext_vector_type(4)));
template <bool NT>
__device__ __forceinline__ float4 ld4(const float4* p) {
    if (!NT) return *p;
    const ops_f4 v = __builtin_nontemporal_load(reinterpret_cast<const ops_f4*>(p));
    return make_float4(v[0], v[1], v[2], v[3]);
}
template <bool NT>
__device__ __forceinline__ void st4(float4* p, float4 v) {
    if (!NT) { *p = v; return; }
    const ops_f4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<ops_f4*>(p));
}
__global__ __launch_bounds__(256) void copy_nt_kernel(float4* __restrict__ dst, const float4* __restrict__ src, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        st4<true>(dst + i, ld4<true>(src + i));
}
template <int NCH, bool NT = false>
__global__ __launch_bounds__(256) void update_rows_kernel(float* __restrict__ tables, size_t table_floats,
                                                         const int32_t* __restrict__ rows, int64_t n_rows, int row_floats) {
    const int lane = threadIdx.x & 63, d4 = row_floats >> 2;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t i = wave; i < n_rows; i += n_waves) {
        const size_t at = (size_t)rows[i] * row_floats;
        float4 x[3][NCH];
#pragma unroll
        for (int t = 0; t < 3; ++t)
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch)
                x[t][ch] = ld4<NT>(reinterpret_cast<const float4*>(tables + t * table_floats + at) + min(ch * 64 + lane, d4 - 1));
#pragma unroll
        for (int t = 0; t < 3; ++t)
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch)
                if (ch * 64 + lane < d4) {
                    float4 v = x[t][ch];
                    v.x += 1.f; v.y += 1.f; v.z += 1.f; v.w += 1.f;
                    st4<NT>(reinterpret_cast<float4*>(tables + t * table_floats + at) + ch * 64 + lane, v);
                }
    }
}

__global__ __launch_bounds__(256) void dense_adam_kernel(const DenseAdamJob job, const AdamHyper hp) {
    const int t = blockIdx.y;
    float* __restrict__ p = job.p[t];
    float* __restrict__ m = job.m[t];
    float* __restrict__ v = job.v[t];
    const float* __restrict__ g = job.g[t];
    const int64_t n = job.n[t];
    const int chunks = job.chunks[t];
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        float gi;
        if (chunks > 0) {     // partial column sums, added up as colsum_final_kernel does
            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
            int k = 0;
            for (; k + 4 <= chunks; k += 4) {
                s0 += g[(size_t)(k + 0) * n + i];
                s1 += g[(size_t)(k + 1) * n + i];
                s2 += g[(size_t)(k + 2) * n + i];
                s3 += g[(size_t)(k + 3) * n + i];
            }
            for (; k < chunks; ++k) s0 += g[(size_t)k * n + i];
            gi = (s0 + s1) + (s2 + s3);
            job.gsum[t][i] = gi;
        } else {
            gi = g[i];
        }
        const float mi = hp.beta1 * m[i] + (1.f - hp.beta1) * gi;
        const float vi = hp.beta2 * v[i] + (1.f - hp.beta2) * gi * gi;
        m[i] = mi;
        v[i] = vi;
        p[i] -= hp.lr * (mi / hp.bc1) / (sqrtf(vi / hp.bc2) + hp.eps);
    }
}

__global__ __launch_bounds__(256) void loss_reduce_kernel(const float* __restrict__ terms, int n, float scale,
                                                          float* __restrict__ loss) {
    __shared__ float part[4];
    float s = 0.f;
    for (int i = threadIdx.x; i < n; i += 256) s += terms[i];
    s = wave_sum(s);
    if (lane_id() == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) loss[0] = scale * ((part[0] + part[1]) + (part[2] + part[3]));
}

}  // namespace

hipError_t launch_inter(const InterJobs& jobs, bool backward, hipStream_t s) {
    if (jobs.count <= 0) return hipSuccess;
    if (jobs.count > INTER_MAX_JOBS) return hipErrorInvalidValue;
    size_t most = 0;
    for (int i = 0; i < jobs.count; ++i) {
        if (jobs.job[i].n <= 0 || jobs.job[i].k < 1 || jobs.job[i].k > NGDB_MAX_CARD) return hipErrorInvalidValue;
        most = std::max(most, (size_t)jobs.job[i].n * jobs.d);
    }
    const dim3 grid((unsigned)((most + 255) / 256), jobs.count);
    if (backward) hipLaunchKernelGGL((inter_kernel<true>), grid, dim3(256), 0, s, jobs);
    else hipLaunchKernelGGL((inter_kernel<false>), grid, dim3(256), 0, s, jobs);
    return hipGetLastError();
}

hipError_t launch_colsums(ColsumJobs& jobs, hipStream_t s, bool finish) {
    if (jobs.count <= 0) return hipSuccess;
    int max_cols = 0, max_chunks = 1;
    for (int i = 0; i < jobs.count; ++i) {
        ColsumJob& j = jobs.job[i];
        j.chunk_rows = std::max(32, (j.rows + COLSUM_MAX_CHUNKS - 1) / COLSUM_MAX_CHUNKS);
        j.chunks = std::max(1, (j.rows + j.chunk_rows - 1) / j.chunk_rows);
        max_cols = std::max(max_cols, j.cols);
        max_chunks = std::max(max_chunks, j.chunks);
    }
    hipLaunchKernelGGL(colsum_part_kernel, dim3((max_cols + 63) / 64, max_chunks, jobs.count), dim3(64, 4), 0, s, jobs);
    if (!finish) return hipGetLastError();
    hipLaunchKernelGGL(colsum_final_kernel, dim3((max_cols + 255) / 256, jobs.count), dim3(256), 0, s, jobs);
    return hipGetLastError();
}

hipError_t launch_fill_zero(float* p, size_t n, hipStream_t s) {
    if (n == 0) return hipSuccess;
    const unsigned blocks = (unsigned)std::min<size_t>((n + 255) / 256, 4096);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, s, p, n);
    return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
    if (bytes == 0) return hipSuccess;
    if (bytes & 15) return hipErrorInvalidValue;
    const size_t n = bytes / 16;
    const unsigned blocks = (unsigned)std::min<size_t>((n + 255) / 256, 256 * 32);
    hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, s, static_cast<float4*>(dst),
                       static_cast<const float4*>(src), n);
    return hipGetLastError();
}

hipError_t launch_stream_pattern(int mode, void* dst, const void* src, size_t bytes, const int32_t* rows, int64_t n_rows,
                                 int row_floats, hipStream_t s) {
    const unsigned full = 256 * 32;      // workgroups of four wavefronts: eight wavefronts per SIMD everywhere
    if (mode == 0) return launch_copy(dst, src, bytes, s);
    if (mode == 1 || mode == 2) {
        if (bytes & 15) return hipErrorInvalidValue;
        const size_t n = bytes / 16;
        const unsigned blocks = (unsigned)std::min<size_t>((n + 255) / 256, full);
        if (mode == 1) hipLaunchKernelGGL(read_kernel, dim3(blocks), dim3(256), 0, s, static_cast<const float4*>(src), n,
                                          static_cast<float*>(dst));
        else hipLaunchKernelGGL(write_kernel, dim3(blocks), dim3(256), 0, s, static_cast<float4*>(dst), n);
        return hipGetLastError();
    }
    if (mode == 5) {     // the copy with non-temporal loads and stores
        if (bytes & 15) return hipErrorInvalidValue;
        const size_t n = bytes / 16;
        hipLaunchKernelGGL(copy_nt_kernel, dim3((unsigned)std::min<size_t>((n + 255) / 256, full)), dim3(256), 0, s,
                           static_cast<float4*>(dst), static_cast<const float4*>(src), n);
        return hipGetLastError();
    }
    if ((mode != 3 && mode != 4 && mode != 6) || !rows || n_rows <= 0 || row_floats < 4 || (row_floats & 3) || row_floats > 1024)
        return hipErrorInvalidValue;
    const unsigned blocks = (unsigned)std::min<int64_t>((n_rows + 3) / 4, full);
    const int nch = row_floats <= 256 ? 1 : (row_floats <= 512 ? 2 : 4);
#define NGDB_PATTERN(NCH)                                                                                          \
    do {                                                                                                          \
        if (mode == 3) hipLaunchKernelGGL((gather_rows_kernel<NCH>), dim3(blocks), dim3(256), 0, s,                \
                                          static_cast<const float*>(src), rows, n_rows, row_floats, static_cast<float*>(dst)); \
        else if (mode == 4) hipLaunchKernelGGL((update_rows_kernel<NCH>), dim3(blocks), dim3(256), 0, s,          \
                                               static_cast<float*>(dst), bytes / 12, rows, n_rows, row_floats);    \
        else hipLaunchKernelGGL((update_rows_kernel<NCH, true>), dim3(blocks), dim3(256), 0, s,                    \
                                static_cast<float*>(dst), bytes / 12, rows, n_rows, row_floats);                   \
    } while (0)
    if (nch == 1) NGDB_PATTERN(1);
    else if (nch == 2) NGDB_PATTERN(2);
    else NGDB_PATTERN(4);
#undef NGDB_PATTERN
    return hipGetLastError();
}

hipError_t launch_dense_adam(const DenseAdamJob& job, const AdamHyper& hp, hipStream_t s) {
    if (job.count <= 0) return hipSuccess;
    int64_t mx = 0;
    for (int t = 0; t < job.count; ++t) mx = std::max(mx, job.n[t]);
    const unsigned bx = (unsigned)std::min<int64_t>((mx + 255) / 256, 512);
    hipLaunchKernelGGL(dense_adam_kernel, dim3(bx, job.count), dim3(256), 0, s, job, hp);
    return hipGetLastError();
}

hipError_t launch_loss_reduce(const float* terms, int n, float scale, float* loss, hipStream_t s) {
    hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(256), 0, s, terms, n, scale, loss);
    return hipGetLastError();
}

}  // namespace ngdb
