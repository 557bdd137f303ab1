// Box-embedding operator family (the paper's Sec. 5.1 lists the box model among the
// backbones trained on the framework): the two operator pieces that are not MLPs.
// Projections translate the centre and widen the offset by the relation's rows, and
// the offset of an intersection is the smallest input offset shrunk by a gate
// computed from all inputs.  Both are memory bound: one thread per (member, 4
// coordinates) or (member, coordinate), rows read and written once.
#include "common.h"

namespace ngdb {
namespace {

template <bool BWD>
__device__ __forceinline__ void proj_body(const BoxProjArgs& a, size_t t) {
    const int d4 = a.d >> 2;
    if (t >= (size_t)a.n * d4) return;
    const int i = (int)(t / d4), c = (int)(t % d4);
    const size_t out = ((size_t)(a.out_base + i) * a.d >> 2) + c;
    if (BWD) {
        const size_t in = ((size_t)a.gslot[i] * a.d >> 2) + c;
        reinterpret_cast<float4*>(a.dact_c)[in] = reinterpret_cast<const float4*>(a.dact_c)[out];
        reinterpret_cast<float4*>(a.dact_o)[in] = reinterpret_cast<const float4*>(a.dact_o)[out];
        return;
    }
    const int32_t ref = a.ref[i];
    const size_t r = ((size_t)a.rel[i] * a.d >> 2) + c;
    float4 x, o = make_float4(0.f, 0.f, 0.f, 0.f);
    if (ref >= 0) {
        const size_t in = ((size_t)ref * a.d >> 2) + c;
        x = reinterpret_cast<const float4*>(a.act_c)[in];
        o = reinterpret_cast<const float4*>(a.act_o)[in];
    } else {
        x = reinterpret_cast<const float4*>(a.E)[((size_t)(-1 - ref) * a.d >> 2) + c];
    }
    const float4 rc = reinterpret_cast<const float4*>(a.Rc)[r];
    const float4 ro = reinterpret_cast<const float4*>(a.Ro)[r];
    x.x += rc.x; x.y += rc.y; x.z += rc.z; x.w += rc.w;
    o.x += fmaxf(ro.x, 0.f); o.y += fmaxf(ro.y, 0.f); o.z += fmaxf(ro.z, 0.f); o.w += fmaxf(ro.w, 0.f);
    reinterpret_cast<float4*>(a.act_c)[out] = x;
    reinterpret_cast<float4*>(a.act_o)[out] = o;
}

template <bool BWD>
__global__ __launch_bounds__(256) void box_proj_kernel(const BoxProjArgs a) {
    proj_body<BWD>(a, (size_t)blockIdx.x * blockDim.x + threadIdx.x);
}

// one thread per (member, coordinate); the cardinality classes of one level are the jobs of
// one launch (blockIdx.y), inputs walked to the compile-time maximum under a predicate
template <bool BWD>
__device__ __forceinline__ void offset_pool(const InterJob& jb, int d, int i, int c) {
    const int n = jb.n, k = jb.k;
    float mean = 0.f, mn = INFINITY;
    int arg = 0;
#pragma unroll
    for (int j = 0; j < NGDB_MAX_CARD; ++j) {
        const size_t row = (size_t)min(j, k - 1) * n + i;
        const float g = jb.Att[row * d + c];
        const float x = jb.X[row * d + c];
        if (j < k) {
            mean += g;
            if (x < mn) {       // strict: equal offsets keep the lower input
                mn = x;
                arg = j;
            }
        }
    }
    const float gate = sigmoid_f(mean / (float)k);
    if (!BWD) {
        jb.out[(size_t)i * d + c] = mn * gate;
    } else {
        const float dy = jb.dY[(size_t)i * d + c];
        const float dpre = dy * mn * gate * (1.f - gate) / (float)k;
#pragma unroll
        for (int j = 0; j < NGDB_MAX_CARD; ++j) {
            if (j < k) {
                const size_t row = (size_t)j * n + i;
                jb.dAtt[row * d + c] = dpre;
                jb.Dx[row * d + c] = j == arg ? dy * gate : 0.f;
            }
        }
    }
}

// attention pooling of the centres (as inter_kernel of the vector family)
template <bool BWD>
__device__ __forceinline__ void centre_pool(const InterJob& jb, int d, int i, int c) {
    const int n = jb.n, k = jb.k;
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
        jb.out[(size_t)i * d + c] = y;
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

template <bool BWD>
__global__ __launch_bounds__(256) void box_offset_kernel(const InterJobs jobs) {
    const InterJob jb = jobs.job[blockIdx.y];
    const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (size_t)jb.n * jobs.d) return;
    offset_pool<BWD>(jb, jobs.d, (int)(t / jobs.d), (int)(t % jobs.d));
}

// centre and offset jobs of one level in one launch (the job kind is uniform per workgroup)
template <bool BWD>
__global__ __launch_bounds__(256) void box_pool_kernel(const BoxPoolJobs bj) {
    const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if ((int)blockIdx.y == bj.jobs.count) {     // the projections riding along
        proj_body<BWD>(bj.proj, t);
        return;
    }
    const InterJob jb = bj.jobs.job[blockIdx.y];
    const int d = bj.jobs.d;
    if (t >= (size_t)jb.n * d) return;
    if ((bj.gate_mask >> blockIdx.y) & 1u) offset_pool<BWD>(jb, d, (int)(t / d), (int)(t % d));
    else centre_pool<BWD>(jb, d, (int)(t / d), (int)(t % d));
}

}  // namespace

hipError_t launch_box_proj(const BoxProjArgs& a, bool backward, hipStream_t s) {
    if (a.n <= 0) return hipSuccess;
    if (a.d & 3) return hipErrorInvalidValue;
    const size_t work = (size_t)a.n * (a.d >> 2);
    const dim3 grid((unsigned)((work + 255) / 256));
    if (backward) hipLaunchKernelGGL((box_proj_kernel<true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((box_proj_kernel<false>), grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_box_offset(const InterJobs& jobs, bool backward, hipStream_t s) {
    if (jobs.count <= 0) return hipSuccess;
    if (jobs.count > INTER_MAX_JOBS) return hipErrorInvalidValue;
    size_t most = 0;
    for (int i = 0; i < jobs.count; ++i) {
        if (jobs.job[i].n <= 0 || jobs.job[i].k < 1 || jobs.job[i].k > NGDB_MAX_CARD) return hipErrorInvalidValue;
        most = std::max(most, (size_t)jobs.job[i].n * jobs.d);
    }
    const dim3 grid((unsigned)((most + 255) / 256), jobs.count);
    if (backward) hipLaunchKernelGGL((box_offset_kernel<true>), grid, dim3(256), 0, s, jobs);
    else hipLaunchKernelGGL((box_offset_kernel<false>), grid, dim3(256), 0, s, jobs);
    return hipGetLastError();
}

hipError_t launch_box_pool(const BoxPoolJobs& bj, bool backward, hipStream_t s) {
    const InterJobs& jobs = bj.jobs;
    if (jobs.count <= 0) return hipSuccess;
    if (jobs.count > INTER_MAX_JOBS) return hipErrorInvalidValue;
    size_t most = 0;
    for (int i = 0; i < jobs.count; ++i) {
        if (jobs.job[i].n <= 0 || jobs.job[i].k < 1 || jobs.job[i].k > NGDB_MAX_CARD) return hipErrorInvalidValue;
        most = std::max(most, (size_t)jobs.job[i].n * jobs.d);
    }
    if (bj.has_proj) {
        if (bj.proj.n <= 0 || (bj.proj.d & 3)) return hipErrorInvalidValue;
        most = std::max(most, (size_t)bj.proj.n * (bj.proj.d >> 2));
    }
    const dim3 grid((unsigned)((most + 255) / 256), jobs.count + (bj.has_proj ? 1 : 0));
    if (backward) hipLaunchKernelGGL((box_pool_kernel<true>), grid, dim3(256), 0, s, bj);
    else hipLaunchKernelGGL((box_pool_kernel<false>), grid, dim3(256), 0, s, bj);
    return hipGetLastError();
}

}  // namespace ngdb
