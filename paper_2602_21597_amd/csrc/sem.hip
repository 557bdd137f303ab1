// Text-feature fusion of entity rows (Sec. 4.4: the frozen encoder's outputs are
// cached in HBM as H_sem, a batch gathers its rows and a learned linear map
// brings them to the embedding width):
//     Ef[e] = E[e] + bf16(Wp) * H_sem[e]
// computed once per step for the entity rows the batch touches (the rows of the
// gradient index, so every repeated negative is projected once), with
// bf16 16x16x32 MFMA blocks and fp32 accumulation; and the gradient of the
// projection, dWp = sum over touched rows of g_row (x) H_sem[row], as a
// contraction over the touched rows split over workgroups and summed in a
// fixed order.
//
// Both kernels stage 64-wide k slices through LDS in rows of 128 bytes whose
// 16-byte chunks are XOR-swizzled, so that the 16 rows one MFMA operand fetch
// touches and the 8 rows one transposing store touches fall on different banks.
#include "common.h"

namespace ngdb {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int KS = 64;          // k extent of one staged slice (bf16 elements), 8 chunks of 8
constexpr int TN = 80;          // embedding coordinates per workgroup tile (5 MFMA blocks)

// LDS rows of W bf16 values; the low three bits of the 16-byte chunk index are swizzled by the row
__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row ^ (row >> 3)) & 7); }
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <int W = KS>
__device__ __forceinline__ u32x4* lds_chunk(uint16_t* base, int row, int chunk) {
    return reinterpret_cast<u32x4*>(base + row * W + swz(row, chunk) * 8);
}
template <int W = KS>
__device__ __forceinline__ bf16x8 frag(const uint16_t* base, int row, int chunk) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(base + row * W + swz(row, chunk) * 8));
}
__device__ __forceinline__ uint32_t to_bf16_bits(float x) {   // round to nearest, ties to even
    const uint32_t b = __float_as_uint(x);
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

__global__ __launch_bounds__(256) void cast_bf16_kernel(const float* __restrict__ x, uint16_t* __restrict__ y, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        y[i] = (uint16_t)to_bf16_bits(x[i]);
}

// inv[contribution number] = position of its entity in the list of touched rows
__global__ __launch_bounds__(256) void inverse_index_kernel(const int32_t* __restrict__ src,
                                                            const int32_t* __restrict__ seg_off,
                                                            const int32_t* __restrict__ n_uniq_dev, int64_t n,
                                                            int32_t* __restrict__ inv) {
    const int n_uniq = *n_uniq_dev;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < n; t += (int64_t)gridDim.x * blockDim.x) {
        int lo = 0, hi = n_uniq;                    // largest u with seg_off[u] <= t
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if ((int64_t)seg_off[mid] <= t) lo = mid; else hi = mid;
        }
        inv[src[t]] = lo;
    }
}

// operator input references with anchors redirected to their fused row
__global__ __launch_bounds__(256) void translate_refs_kernel(const int32_t* __restrict__ in_ref,
                                                             const int32_t* __restrict__ in_gslot, int n, int n_slots,
                                                             const int32_t* __restrict__ inv, int32_t* __restrict__ out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t r = in_ref[i];
    out[i] = r >= 0 ? r : -1 - inv[in_gslot[i] - n_slots];
}

// ------------------------------------------------------------------ forward
// out[u, :] = E[id(u), :] + Wb * H[id(u), :].  Workgroup tile: BU rows x TN coordinates, k
// slices of KSF; wavefront w owns rows [w*BU/4, (w+1)*BU/4).  The slice width sets how much of
// a gathered feature row one request covers, BU the registers per lane: the kernel waits on
// HBM, so the shape is chosen for bytes in flight per compute unit, not for MFMA reuse.
template <int BU, int KSF>
__global__ __launch_bounds__(256) void sem_fuse_kernel(const SemFuseArgs a) {
    constexpr int CPR = KSF / 8;                 // 16-byte chunks per LDS row
    constexpr int RPP = 256 / CPR;               // rows covered by one pass of the 256 threads
    constexpr int LH = BU / RPP;                 // feature chunks per thread and slice
    constexpr int LW = (TN + RPP - 1) / RPP;     // projection chunks per thread and slice
    constexpr int RB = BU / 64;                  // 16-row MFMA blocks per wavefront
    __shared__ __attribute__((aligned(16))) uint16_t Hs[BU * KSF];
    __shared__ __attribute__((aligned(16))) uint16_t Ws[LW * RPP * KSF];   // TN rows used
    const int n_rows = a.n_rows_dev ? min(*a.n_rows_dev, a.n_rows) : a.n_rows;
    const int n_tiles = (a.d + TN - 1) / TN;
    // workgroups are dealt round-robin to the 8 dies: the coordinate tiles of one
    // row tile go to the same die one after the other and share its L2
    const int die = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int u0 = ((j / n_tiles) * 8 + die) * BU;
    const int n0 = (j % n_tiles) * TN;
    if (u0 >= n_rows) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = tid / CPR, lchunk = tid % CPR;

    const uint16_t* hrow[LH];
#pragma unroll
    for (int i = 0; i < LH; ++i) {
        const int u = min(u0 + lrow + RPP * i, n_rows - 1);
        const int64_t id = a.ids ? a.ids[u] : a.id_base + u;
        hrow[i] = a.H + id * a.ds + lchunk * 8;
    }
    const uint16_t* wrow[LW];
#pragma unroll
    for (int i = 0; i < LW; ++i)
        wrow[i] = a.Wb + (size_t)min(n0 + min(lrow + RPP * i, TN - 1), a.d - 1) * a.ds + lchunk * 8;

    u32x4 rh[LH], rw[LW];
#pragma unroll
    for (int i = 0; i < LH; ++i) rh[i] = *reinterpret_cast<const u32x4*>(hrow[i]);
#pragma unroll
    for (int i = 0; i < LW; ++i) rw[i] = *reinterpret_cast<const u32x4*>(wrow[i]);

    // The accumulators start from the structural rows, requested together with the first
    // slice: a lane holds, per block, 4 consecutive coordinates of one row (clamped addresses;
    // rows and coordinates past the end are never stored).
    floatx4 acc[RB][5];
#pragma unroll
    for (int bu = 0; bu < RB; ++bu) {
        const int u = min(u0 + wave * (BU / 4) + bu * 16 + (lane & 15), n_rows - 1);
        const int64_t id = a.ids ? a.ids[u] : a.id_base + u;
        const float* erow = a.E + id * a.d;
#pragma unroll
        for (int bn = 0; bn < 5; ++bn) {
            const float4 e = *reinterpret_cast<const float4*>(erow + min(n0 + bn * 16 + (lane >> 4) * 4, a.d - 4));
            acc[bu][bn] = floatx4{e.x, e.y, e.z, e.w};
        }
    }

    for (int k0 = 0; k0 < a.ds; k0 += KSF) {
#pragma unroll
        for (int i = 0; i < LH; ++i) *lds_chunk<KSF>(Hs, lrow + RPP * i, lchunk) = rh[i];
#pragma unroll
        for (int i = 0; i < LW; ++i) *lds_chunk<KSF>(Ws, lrow + RPP * i, lchunk) = rw[i];
        __syncthreads();
        {   // next slice (the last iteration re-reads its own: no branch around the loads)
            const int kn = min(k0 + KSF, a.ds - KSF);
#pragma unroll
            for (int i = 0; i < LH; ++i) rh[i] = *reinterpret_cast<const u32x4*>(hrow[i] + kn);
#pragma unroll
            for (int i = 0; i < LW; ++i) rw[i] = *reinterpret_cast<const u32x4*>(wrow[i] + kn);
        }
#pragma unroll
        for (int kk = 0; kk < KSF / 32; ++kk) {
            const int chunk = kk * 4 + (lane >> 4);
            bf16x8 fh[RB], fw[5];
#pragma unroll
            for (int bu = 0; bu < RB; ++bu) fh[bu] = frag<KSF>(Hs, wave * (BU / 4) + bu * 16 + (lane & 15), chunk);
#pragma unroll
            for (int bn = 0; bn < 5; ++bn) fw[bn] = frag<KSF>(Ws, bn * 16 + (lane & 15), chunk);
#pragma unroll
            for (int bu = 0; bu < RB; ++bu)
#pragma unroll
                for (int bn = 0; bn < 5; ++bn)
                    acc[bu][bn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[bn], fh[bu], acc[bu][bn], 0, 0, 0);
        }
        __syncthreads();
    }
    // a lane holds, per block, 4 consecutive coordinates of one row
#pragma unroll
    for (int bu = 0; bu < RB; ++bu) {
        const int u = u0 + wave * (BU / 4) + bu * 16 + (lane & 15);
        if (u >= n_rows) continue;
        float* orow = a.out + (size_t)u * a.d;
#pragma unroll
        for (int bn = 0; bn < 5; ++bn) {
            const int n = n0 + bn * 16 + (lane >> 4) * 4;
            if (n >= a.d) continue;
            *reinterpret_cast<float4*>(orow + n) =
                make_float4(acc[bu][bn][0], acc[bu][bn][1], acc[bu][bn][2], acc[bu][bn][3]);
        }
    }
}

// ------------------------------------------------------------------ gradient of Wp
// 8 rows x 8 bf16 held by one thread (x[j] = row j) -> y[i] = column i over the 8 rows
__device__ __forceinline__ void transpose8x8(const uint4 (&x)[8], uint4 (&y)[8]) {
    uint32_t in[8][4], out[8][4];
#pragma unroll
    for (int j = 0; j < 8; ++j) { in[j][0] = x[j].x; in[j][1] = x[j].y; in[j][2] = x[j].z; in[j][3] = x[j].w; }
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const uint32_t lo = in[2 * p][i >> 1], hi = in[2 * p + 1][i >> 1];
            out[i][p] = (i & 1) ? ((lo >> 16) | (hi & 0xFFFF0000u)) : ((lo & 0xFFFFu) | (hi << 16));
        }
#pragma unroll
    for (int i = 0; i < 8; ++i) y[i] = make_uint4(out[i][0], out[i][1], out[i][2], out[i][3]);
}

constexpr int WG_SEM = 256;     // text-feature coordinates per workgroup tile of the gradient

// loads of one 64-row stage, written as force-inlined functions over register arrays
__device__ __forceinline__ void wgrad_load_ids(const SemWgradArgs& a, int s, int ug, int n_rows, int32_t (&ids)[8]) {
#pragma unroll
    for (int q = 0; q < 8; ++q) ids[q] = a.ids[min(s * KS + ug * 8 + q, n_rows - 1)];
}
__device__ __forceinline__ void wgrad_load_data(const SemWgradArgs& a, int s, const int32_t (&ids)[8], int hcol,
                                                bool g_thread, int gug, int gcol, int n_rows, uint4 (&rh)[8],
                                                uint4 (&rg)[8]) {
#pragma unroll
    for (int q = 0; q < 8; ++q) rh[q] = *reinterpret_cast<const uint4*>(a.H + (size_t)ids[q] * a.ds + hcol);
    if (g_thread) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int u = min(s * KS + gug * 8 + q, n_rows - 1);
            rg[q] = *reinterpret_cast<const uint4*>(a.G + (size_t)u * a.d + gcol);
        }
    }
}

// partial[split, m, n] = sum over the split's rows u of G[u, m] * H[id(u), n]
__global__ __launch_bounds__(256) void sem_wgrad_kernel(const SemWgradArgs a) {
    __shared__ __attribute__((aligned(16))) uint16_t Ht[WG_SEM * KS];   // [n][u]
    __shared__ __attribute__((aligned(16))) uint16_t Gt[TN * KS];       // [m][u]
    const int n_rows = min(*a.n_rows_dev, a.n_rows);
    const int m_tiles = (a.d + TN - 1) / TN, n_tiles = (a.ds + WG_SEM - 1) / WG_SEM;
    const int tiles = m_tiles * n_tiles;
    const int die = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int split = (j / tiles) * 8 + die;
    if (split >= a.n_splits) return;
    const int tile = j % tiles;
    const int m0 = (tile % m_tiles) * TN, n0 = (tile / m_tiles) * WG_SEM;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    const int stages = (n_rows + KS - 1) / KS;
    const int per_split = (stages + a.n_splits - 1) / a.n_splits;
    const int s_lo = split * per_split, s_hi = min(stages, s_lo + per_split);

    // H: thread = (8 feature coordinates ng, 8 rows ug); G: threads 0..79 = (8 coordinates mg, 8 rows ug)
    const int ng = tid & 31, ug = tid >> 5;
    const int hcol = min(n0 + ng * 8, a.ds - 8);
    const bool g_thread = tid < (TN / 8) * 8;
    const int mg = tid % (TN / 8), gug = tid / (TN / 8);
    const bool g_col_ok = g_thread && m0 + mg * 8 < a.d;
    const int gcol = min(m0 + mg * 8, a.d - 8);

    floatx4 acc[4][5];
#pragma unroll
    for (int bn = 0; bn < 4; ++bn)
#pragma unroll
        for (int bm = 0; bm < 5; ++bm) acc[bn][bm] = floatx4{0.f, 0.f, 0.f, 0.f};

    int32_t ids[8];
    uint4 rh[8], rg[8];
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
    if (s_lo < s_hi) {
        wgrad_load_ids(a, s_lo, ug, n_rows, ids);
        wgrad_load_data(a, s_lo, ids, hcol, g_thread, gug, gcol, n_rows, rh, rg);
        if (s_lo + 1 < s_hi) wgrad_load_ids(a, s_lo + 1, ug, n_rows, ids);
    }
    for (int s = s_lo; s < s_hi; ++s) {
        {   // transpose to [coordinate][row]; rows past the end contribute zeros through G
            uint4 t[8];
            transpose8x8(rh, t);
#pragma unroll
            for (int i = 0; i < 8; ++i) *lds_chunk(Ht, ng * 8 + i, ug) = u32x4{t[i].x, t[i].y, t[i].z, t[i].w};
            if (g_thread) {
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    if (!g_col_ok || s * KS + gug * 8 + q >= n_rows) rg[q] = zero;
                transpose8x8(rg, t);
#pragma unroll
                for (int i = 0; i < 8; ++i) *lds_chunk(Gt, mg * 8 + i, gug) = u32x4{t[i].x, t[i].y, t[i].z, t[i].w};
            }
        }
        __syncthreads();
        if (s + 1 < s_hi) {
            wgrad_load_data(a, s + 1, ids, hcol, g_thread, gug, gcol, n_rows, rh, rg);
            if (s + 2 < s_hi) wgrad_load_ids(a, s + 2, ug, n_rows, ids);
        }
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int chunk = kk * 4 + (lane >> 4);
            bf16x8 fh[4], fg[5];
#pragma unroll
            for (int bn = 0; bn < 4; ++bn) fh[bn] = frag(Ht, wave * 64 + bn * 16 + (lane & 15), chunk);
#pragma unroll
            for (int bm = 0; bm < 5; ++bm) fg[bm] = frag(Gt, bm * 16 + (lane & 15), chunk);
#pragma unroll
            for (int bn = 0; bn < 4; ++bn)
#pragma unroll
                for (int bm = 0; bm < 5; ++bm)
                    acc[bn][bm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fh[bn], fg[bm], acc[bn][bm], 0, 0, 0);
        }
        __syncthreads();
    }
    // a lane holds, per block, 4 consecutive feature coordinates n of one embedding coordinate m
#pragma unroll
    for (int bm = 0; bm < 5; ++bm) {
        const int m = m0 + bm * 16 + (lane & 15);
        if (m >= a.d) continue;
        float* prow = a.partial + ((size_t)split * a.d + m) * a.ds;
#pragma unroll
        for (int bn = 0; bn < 4; ++bn) {
            const int n = n0 + wave * 64 + bn * 16 + (lane >> 4) * 4;
            if (n >= a.ds) continue;
            *reinterpret_cast<float4*>(prow + n) =
                make_float4(acc[bn][bm][0], acc[bn][bm][1], acc[bn][bm][2], acc[bn][bm][3]);
        }
    }
}

__global__ __launch_bounds__(256) void sem_wgrad_reduce_kernel(const float* __restrict__ partial, int n_splits,
                                                               int64_t n4, float* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n4) return;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int k = 0; k < n_splits; ++k) {
        const float4 v = reinterpret_cast<const float4*>(partial)[(size_t)k * n4 + i];
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    reinterpret_cast<float4*>(out)[i] = s;
}

}  // namespace

hipError_t launch_cast_bf16(const float* x, uint16_t* y, int64_t n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    const unsigned blocks = (unsigned)std::min<int64_t>((n + 255) / 256, 2048);
    hipLaunchKernelGGL(cast_bf16_kernel, dim3(blocks), dim3(256), 0, s, x, y, n);
    return hipGetLastError();
}

hipError_t launch_inverse_index(const int32_t* src, const int32_t* seg_off, const int32_t* n_uniq_dev, int64_t n,
                                int32_t* inv, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    const unsigned blocks = (unsigned)std::min<int64_t>((n + 255) / 256, 4096);
    hipLaunchKernelGGL(inverse_index_kernel, dim3(blocks), dim3(256), 0, s, src, seg_off, n_uniq_dev, n, inv);
    return hipGetLastError();
}

hipError_t launch_translate_refs(const int32_t* in_ref, const int32_t* in_gslot, int n, int n_slots,
                                 const int32_t* inv, int32_t* out, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(translate_refs_kernel, dim3((n + 255) / 256), dim3(256), 0, s, in_ref, in_gslot, n, n_slots,
                       inv, out);
    return hipGetLastError();
}

template <int BU, int KSF>
hipError_t launch_sem_fuse_as(const SemFuseArgs& a, hipStream_t s) {
    const int64_t u_tiles = (a.n_rows + BU - 1) / BU;
    const int64_t n_tiles = (a.d + TN - 1) / TN;
    const int64_t blocks = ((u_tiles + 7) / 8) * 8 * n_tiles;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL((sem_fuse_kernel<BU, KSF>), dim3((unsigned)blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_sem_fuse(const SemFuseArgs& a, hipStream_t s) {
    if (a.n_rows <= 0) return hipSuccess;
    if (a.ds <= 0 || a.ds % KS || a.d % 4) return hipErrorInvalidValue;
    return launch_sem_fuse_as<256, 64>(a, s);
}

int sem_wgrad_splits(int64_t n_rows_bound, int d, int ds) {
    const int tiles = ((d + TN - 1) / TN) * ((ds + WG_SEM - 1) / WG_SEM);
    const int64_t stages = (n_rows_bound + KS - 1) / KS;
    // one resident set of workgroups, no second round: 2 workgroups of this kernel fit a compute
    // unit (224 VGPRs), 256 units
    const int cap = std::max(8, (512 / tiles) / 8 * 8);
    return (int)std::max<int64_t>(1, std::min<int64_t>(stages / 4, cap));
}

hipError_t launch_sem_wgrad(const SemWgradArgs& a, float* out, hipStream_t s) {
    if (a.ds <= 0 || a.ds % KS || a.d % 8 || a.n_splits < 1) return hipErrorInvalidValue;
    const int tiles = ((a.d + TN - 1) / TN) * ((a.ds + WG_SEM - 1) / WG_SEM);
    const int blocks = ((a.n_splits + 7) / 8) * 8 * tiles;
    hipLaunchKernelGGL(sem_wgrad_kernel, dim3(blocks), dim3(256), 0, s, a);
    const int64_t n4 = (int64_t)a.d * a.ds / 4;
    hipLaunchKernelGGL(sem_wgrad_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s,
                       (const float*)a.partial, a.n_splits, n4, out);
    return hipGetLastError();
}

}  // namespace ngdb
