// fp32 MFMA GEMM for the grouped operator MLPs (forward, data-gradient and
// weight-gradient contractions of Sec. 4.1's batched kernels).  One workgroup of
// four wavefronts computes a BM x BN tile; every wavefront owns a (BM/2) x (BN/2)
// sub-tile made of 32x32 MFMA blocks (v_mfma_f32_32x32x2_f32).  Operand tiles go
// through LDS k-major, double buffered, so that each MFMA operand is one
// conflict-free 4-byte LDS read per lane.
#include "common.h"

namespace ngdb {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 16;    // k extent of one LDS tile
constexpr int PAD = 4;    // keeps rows 16-byte aligned and spreads banks

template <int BM, int BN, bool AK, bool BKC>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmArgs a) {
    __shared__ __attribute__((aligned(16))) float As[2][BK][BM + PAD];
    __shared__ __attribute__((aligned(16))) float Bs[2][BK][BN + PAD];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int m0 = blockIdx.y * BM;
    const int n0 = blockIdx.x * BN;
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 32, TN = WN / 32;
    const int wm0 = (wave >> 1) * WM;
    const int wn0 = (wave & 1) * WN;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    constexpr int LA = BM * BK / 4 / 256;
    constexpr int LB = BN * BK / 4 / 256;
    static_assert(LA >= 1 && LB >= 1, "tile too small for 256 threads");
    float4 ra[LA], rb[LB];
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);

    auto load_tiles = [&](int k0) {
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int idx = tid + i * 256;
            if (AK) {
                const int m = idx / (BK / 4), kq = idx % (BK / 4);
                const int gm = m0 + m, gk = k0 + kq * 4;
                ra[i] = (gm < a.M && gk < a.K)
                            ? *reinterpret_cast<const float4*>(a.A + (size_t)gm * a.lda + gk) : zero4;
            } else {
                const int k = idx / (BM / 4), mq = idx % (BM / 4);
                const int gk = k0 + k, gm = m0 + mq * 4;
                ra[i] = (gk < a.K && gm < a.M)
                            ? *reinterpret_cast<const float4*>(a.A + (size_t)gk * a.lda + gm) : zero4;
            }
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int idx = tid + i * 256;
            if (BKC) {
                const int n = idx / (BK / 4), kq = idx % (BK / 4);
                const int gn = n0 + n, gk = k0 + kq * 4;
                rb[i] = (gn < a.N && gk < a.K)
                            ? *reinterpret_cast<const float4*>(a.B + (size_t)gn * a.ldb + gk) : zero4;
            } else {
                const int k = idx / (BN / 4), nq = idx % (BN / 4);
                const int gk = k0 + k, gn = n0 + nq * 4;
                rb[i] = (gk < a.K && gn < a.N)
                            ? *reinterpret_cast<const float4*>(a.B + (size_t)gk * a.ldb + gn) : zero4;
            }
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int idx = tid + i * 256;
            if (AK) {
                const int m = idx / (BK / 4), kq = idx % (BK / 4);
                As[buf][kq * 4 + 0][m] = ra[i].x;
                As[buf][kq * 4 + 1][m] = ra[i].y;
                As[buf][kq * 4 + 2][m] = ra[i].z;
                As[buf][kq * 4 + 3][m] = ra[i].w;
            } else {
                const int k = idx / (BM / 4), mq = idx % (BM / 4);
                *reinterpret_cast<float4*>(&As[buf][k][mq * 4]) = ra[i];
            }
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int idx = tid + i * 256;
            if (BKC) {
                const int n = idx / (BK / 4), kq = idx % (BK / 4);
                Bs[buf][kq * 4 + 0][n] = rb[i].x;
                Bs[buf][kq * 4 + 1][n] = rb[i].y;
                Bs[buf][kq * 4 + 2][n] = rb[i].z;
                Bs[buf][kq * 4 + 3][n] = rb[i].w;
            } else {
                const int k = idx / (BN / 4), nq = idx % (BN / 4);
                *reinterpret_cast<float4*>(&Bs[buf][k][nq * 4]) = rb[i];
            }
        }
    };

    const int nk = (a.K + BK - 1) / BK;
    load_tiles(0);
    store_tiles(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_tiles((kt + 1) * BK);
#pragma unroll
        for (int kk = 0; kk < BK / 2; ++kk) {
            const int krow = kk * 2 + (lane >> 5);
            float av[TM], bv[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) av[i] = As[buf][krow][wm0 + i * 32 + (lane & 31)];
#pragma unroll
            for (int j = 0; j < TN; ++j) bv[j] = Bs[buf][krow][wn0 + j * 32 + (lane & 31)];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_tiles(buf ^ 1);
        __syncthreads();
    }

    // accumulator layout of the 32x32 block: lane owns column (lane & 31) and the
    // rows 8*(r/4) + 4*(lane/32) + r%4, r = 0..15
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn0 + j * 32 + (lane & 31);
            if (col >= a.N) continue;
            const float bias = a.bias ? a.bias[col] : 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm0 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                if (row >= a.M) continue;
                float v = acc[i][j][r] + bias;
                if (a.relu) v = fmaxf(v, 0.f);
                if (a.mask) v = a.mask[(size_t)row * a.ldmask + col] > 0.f ? v : 0.f;
                if (a.addend) v += a.addend[(size_t)row * a.ldadd + col];
                const int orow = a.dst_row ? a.dst_row[row] : row;
                a.C[(size_t)orow * a.ldc + col] = v;
            }
        }
}

template <int BM, int BN>
hipError_t dispatch_layout(const GemmArgs& a, hipStream_t s) {
    dim3 grid((a.N + BN - 1) / BN, (a.M + BM - 1) / BM);
    dim3 block(256);
    if (a.a_kcontig && a.b_kcontig)
        hipLaunchKernelGGL((gemm_kernel<BM, BN, true, true>), grid, block, 0, s, a);
    else if (a.a_kcontig && !a.b_kcontig)
        hipLaunchKernelGGL((gemm_kernel<BM, BN, true, false>), grid, block, 0, s, a);
    else if (!a.a_kcontig && !a.b_kcontig)
        hipLaunchKernelGGL((gemm_kernel<BM, BN, false, false>), grid, block, 0, s, a);
    else
        hipLaunchKernelGGL((gemm_kernel<BM, BN, false, true>), grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s) {
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    // float4 operand loads: leading dimensions and the contiguous extents must be multiples of 4
    if ((a.lda & 3) || (a.ldb & 3)) return hipErrorInvalidValue;
    if ((a.a_kcontig ? a.K : a.M) & 3) return hipErrorInvalidValue;
    if ((a.b_kcontig ? a.K : a.N) & 3) return hipErrorInvalidValue;
    // larger row tile once there are enough tiles to cover the 256 compute units
    const long tiles128 = (long)((a.M + 127) / 128) * ((a.N + 63) / 64);
    if (tiles128 >= 512) return dispatch_layout<128, 64>(a, s);
    return dispatch_layout<64, 64>(a, s);
}

}  // namespace ngdb
