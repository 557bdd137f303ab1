// fp32 MFMA GEMM for the grouped operator MLPs (forward, data-gradient and
// weight-gradient contractions of Sec. 4.1's batched kernels).
//
// The groups of one batch are small next to the chip (a few hundred to a few
// thousand rows against 256 compute units), so a contraction is latency bound,
// not throughput bound: what matters is the length of the dependent chain
// "global load -> LDS -> MFMA" of one workgroup.  Therefore the k extent is
// split over the wavefronts of a workgroup: every wavefront walks its own
// k-tiles (tile w, w+NW, ...) through a private LDS staging area and
// accumulates the whole BM x BN output tile with 32x32x2 MFMA blocks; the NW
// partial tiles are then summed through LDS in a fixed order (deterministic) and
// the epilogue is applied to the sum.  The A operand can be assembled on the fly
// from row references (gather of operator inputs fused into the first layer).
//
// Results are fp32 either way, but the products are formed on one of two routes: fp32
// MFMA blocks, or (SPLIT) bf16 MFMA blocks on operands that are split, while a tile is
// staged, into three bf16 pieces whose sum is the fp32 value exactly; six of the nine
// partial products are kept.  The matrix unit then needs 2.7 times less time per tile.
// On the split route the small tile can take operands that were split beforehand (BP: the
// weights, once per pass, by weight_pieces_kernel; AP: the hidden rows, by the epilogue of
// the launch that produced them): such pieces lie in global memory tile by tile in the lane
// order of the MFMA and go from there straight into its operand registers.
#include "common.h"

namespace ngdb {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 16;    // k extent of one staged tile
constexpr int PAD = 4;    // keeps LDS rows 16-byte aligned and spreads banks

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int BM, int BN, int NW, bool SPLIT = false, bool BP = false, bool AP = false>
struct Smem {
    // SPLIT: per wavefront and operand three bf16 pieces of a [32][BK] tile (BP, AP: that operand
    // comes ready-made from global memory and is not staged)
    static constexpr int STAGE = SPLIT ? NW * ((AP ? 0 : BM / 32) + (BP ? 0 : BN / 32)) * 960 : NW * BK * (BM + PAD + BN + PAD);   // floats
    // partial tiles held in LDS at once: all of them in the small tile (one barrier less than folding
    // the upper half of the wavefronts into the lower half first, 34 KB for eight)
    static constexpr int NR = (NW > 4 && BM * BN > 32 * 32) ? NW / 2 : NW;
    static constexpr int REDUCE = NR * BM * (BN + 1);
    static constexpr int FLOATS = STAGE > REDUCE ? STAGE : REDUCE;
};

// Operand staging is written as force-inlined functions over register arrays of
// compile-time size (no lambdas, no run-time indices) so that the tiles in
// flight stay in VGPRs.  Issuing a tile is nothing but address arithmetic and
// loads: addresses are clamped into the operand, never branched on, and nothing
// touches the loaded values before the tile is staged, so the loads of the next
// tile stay in flight while the current one is multiplied.
// A 16-byte load from global memory.  Row pointers picked at run time among several bases lose their
// address space, and the loads through them would be FLAT ones: those count as LDS operations as
// well, so every LDS read of the current tile would wait for the tile requested ahead.
// (through a built-in vector type: float4 is a class, and copying one goes through a generic reference)
__device__ __forceinline__ float4 load_global4(const float* p) {
    typedef float floatx4 __attribute__((ext_vector_type(4)));
    typedef const floatx4 __attribute__((address_space(1))) * global_floatx4;
    const floatx4 v = *(global_floatx4)p;
    return make_float4(v.x, v.y, v.z, v.w);
}

template <int BM, int LA, bool AK>
__device__ __forceinline__ void issue_a(const GemmArgs& a, int lane, int m0, int k0, bool has_add,
                                        const float* const (&arow)[LA], const float* const (&aadd)[LA],
                                        float4 (&ra)[LA], float4 (&rd)[LA]) {
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int idx = lane + i * 64;
        if (AK) {
            const int gkc = min(k0 + (idx % (BK / 4)) * 4, a.K - 4);
            ra[i] = load_global4(arow[i] + gkc);
            if (has_add) rd[i] = load_global4(aadd[i] + gkc);
        } else {
            const int gk = k0 + idx / (BM / 4), gm = m0 + (idx % (BM / 4)) * 4;
            ra[i] = load_global4(a.A + (size_t)min(gk, a.K - 1) * a.lda + min(gm, a.M - 4));
        }
    }
}

template <int BN, int LB, bool BKC>
__device__ __forceinline__ void issue_b(const GemmArgs& a, int lane, int n0, int k0, float4 (&rb)[LB]) {
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int idx = lane + i * 64;
        const float* p;
        if (BKC) {
            const int gn = n0 + idx / (BK / 4), gk = k0 + (idx % (BK / 4)) * 4;
            p = a.B + (size_t)min(gn, a.N - 1) * a.ldb + min(gk, a.K - 4);
        } else {
            const int gk = k0 + idx / (BN / 4), gn = n0 + (idx % (BN / 4)) * 4;
            p = a.B + (size_t)min(gk, a.K - 1) * a.ldb + min(gn, a.N - 4);
        }
        rb[i] = load_global4(p);
    }
}

// registers -> this wavefront's LDS tile [BK][LD].  Here the values are completed:
// relation row added, entries outside the operand zeroed, assembled A rows copied out.
template <int BM, int LA, int LD, bool AK>
__device__ __forceinline__ void stage_a(const GemmArgs& a, float* __restrict__ dst, int lane, int m0, int k0,
                                        bool has_add, bool copy_out, const bool (&avalid)[LA],
                                        const float4 (&ra)[LA], const float4 (&rd)[LA]) {
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int idx = lane + i * 64;
        float4 v = ra[i];
        if (AK) {
            const int m = idx / (BK / 4), kq = idx % (BK / 4);
            const int gk = k0 + kq * 4;
            if (has_add) { v.x += rd[i].x; v.y += rd[i].y; v.z += rd[i].z; v.w += rd[i].w; }
            const bool ok = avalid[i] && gk < a.K;
            v.x = ok ? v.x : 0.f; v.y = ok ? v.y : 0.f; v.z = ok ? v.z : 0.f; v.w = ok ? v.w : 0.f;
            if (copy_out && ok) *reinterpret_cast<float4*>(a.a_copy + (size_t)(m0 + m) * a.lda + gk) = v;
            dst[(kq * 4 + 0) * LD + m] = v.x;
            dst[(kq * 4 + 1) * LD + m] = v.y;
            dst[(kq * 4 + 2) * LD + m] = v.z;
            dst[(kq * 4 + 3) * LD + m] = v.w;
        } else {
            const int k = idx / (BM / 4), mq = idx % (BM / 4);
            const bool ok = k0 + k < a.K && m0 + mq * 4 < a.M;
            v.x = ok ? v.x : 0.f; v.y = ok ? v.y : 0.f; v.z = ok ? v.z : 0.f; v.w = ok ? v.w : 0.f;
            *reinterpret_cast<float4*>(&dst[k * LD + mq * 4]) = v;
        }
    }
}

template <int BN, int LB, int LD, bool BKC>
__device__ __forceinline__ void stage_b(const GemmArgs& a, float* __restrict__ dst, int lane, int n0, int k0,
                                        const float4 (&rb)[LB]) {
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int idx = lane + i * 64;
        float4 v = rb[i];
        if (BKC) {
            const int n = idx / (BK / 4), kq = idx % (BK / 4);
            const bool ok = n0 + n < a.N && k0 + kq * 4 < a.K;
            v.x = ok ? v.x : 0.f; v.y = ok ? v.y : 0.f; v.z = ok ? v.z : 0.f; v.w = ok ? v.w : 0.f;
            dst[(kq * 4 + 0) * LD + n] = v.x;
            dst[(kq * 4 + 1) * LD + n] = v.y;
            dst[(kq * 4 + 2) * LD + n] = v.z;
            dst[(kq * 4 + 3) * LD + n] = v.w;
        } else {
            const int k = idx / (BN / 4), nq = idx % (BN / 4);
            const bool ok = k0 + k < a.K && n0 + nq * 4 < a.N;
            v.x = ok ? v.x : 0.f; v.y = ok ? v.y : 0.f; v.z = ok ? v.z : 0.f; v.w = ok ? v.w : 0.f;
            *reinterpret_cast<float4*>(&dst[k * LD + nq * 4]) = v;
        }
    }
}

// An fp32 value is the exact sum of three bf16 values: x rounded to bf16, the remainder rounded
// to bf16, and what is then left (at most 6 bits).  Rounding is to nearest (the hardware
// conversion), so the pieces carry signs of their own and nothing is biased: with pieces cut off
// instead, every product would come out a little short, and the scores, whose loss weights
// depend on them exponentially, would shift in one direction.  A product of two fp32 values is a
// sum of nine bf16 products, of which the six largest are kept; the three left out are below
// 2^-23 of the product (second piece at most 2^-8, third at most 2^-16 of the value), with
// either sign.  bf16 products are exact in the fp32 accumulator of the matrix unit,
// which multiplies bf16 sixteen times as fast as fp32.
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t cvt_pk(float first, float second) {   // first in the lower half
    const floatx2 v = {first, second};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
// pieces of two values, packed pairwise: h, m, l words
__device__ __forceinline__ void split2(float a, float b, uint32_t& h, uint32_t& m, uint32_t& l) {
    h = cvt_pk(a, b);
    const float ra = a - __uint_as_float(h << 16), rb = b - __uint_as_float(h & 0xffff0000u);
    m = cvt_pk(ra, rb);
    l = cvt_pk(ra - __uint_as_float(m << 16), rb - __uint_as_float(m & 0xffff0000u));
}
struct Pieces {
    uint2 h, m, l;     // 4 consecutive k each, bf16 bit patterns
};
__device__ __forceinline__ Pieces split3(float4 v) {
    Pieces p;
    split2(v.x, v.y, p.h.x, p.m.x, p.l.x);
    split2(v.z, v.w, p.h.y, p.m.y, p.l.y);
    return p;
}
// Pieces of a [32][BK] tile in LDS: 16-byte units (8 consecutive k of a row); unit index
// = k-half * 32 + row, piece after piece -- the operand layout of the 32x32x16 bf16 MFMA
// (lane = k-half * 32 + row reads unit `lane`).  In the tiles of an operand that is staged from
// its k-strided layout (GAPS) one unit is left empty after every four: the 32-bit stores of that
// staging then spread over all banks (8-way conflicts without the gaps; the 64-bit stores of the
// k-contiguous staging need none and are slower with them).  Room per piece: 80 units = 640
// bf16 either way; the three pieces of 32 rows take 1920.
template <bool GAPS>
__device__ __forceinline__ int unit_at(int u) { return (GAPS ? u + (u >> 2) : u) * 8; }
constexpr int PIECE = 640, SUBTILE = 3 * PIECE;
__device__ __forceinline__ void store_pieces(uint16_t* tile, int row, int kq, const Pieces& p) {
    uint16_t* at = tile + unit_at<false>((kq >> 1) * 32 + row) + (kq & 1) * 4;
    *reinterpret_cast<uint2*>(at) = p.h;
    *reinterpret_cast<uint2*>(at + PIECE) = p.m;
    *reinterpret_cast<uint2*>(at + 2 * PIECE) = p.l;
}

// Operand stored with k as the slow index ([K][X], X = rows or columns of the output): a lane
// takes two consecutive k of four consecutive x (8 lanes cover 128 contiguous bytes), so that
// the pieces of a (k, k+1) pair fill one 32-bit word of the tile.
__device__ __forceinline__ void issue_strided(const float* base, int ld, int K, int X, int k0, int x0, int lane,
                                              float4 (&r)[2]) {
    const int gk = k0 + 2 * (lane >> 3), gx = min(x0 + (lane & 7) * 4, X - 4);
    r[0] = load_global4(base + (size_t)min(gk, K - 1) * ld + gx);
    r[1] = load_global4(base + (size_t)min(gk + 1, K - 1) * ld + gx);
}
__device__ __forceinline__ void stage_strided(uint16_t* tile, int K, int X, int k0, int x0, int lane,
                                              const float4 (&r)[2]) {
    const int kp = lane >> 3, q = lane & 7;
    const bool okx = x0 + q * 4 < X;
    const bool ok0 = okx && k0 + 2 * kp < K, ok1 = okx && k0 + 2 * kp + 1 < K;
    const float e[4] = {r[0].x, r[0].y, r[0].z, r[0].w}, o[4] = {r[1].x, r[1].y, r[1].z, r[1].w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        uint32_t h, m, l;
        split2(ok0 ? e[j] : 0.f, ok1 ? o[j] : 0.f, h, m, l);
        uint32_t* at = reinterpret_cast<uint32_t*>(tile + unit_at<true>((kp >> 2) * 32 + q * 4 + j) + (kp & 3) * 2);
        at[0] = h;
        at[PIECE / 2] = m;
        at[PIECE] = l;
    }
}

// Weight matrices as ready-made B operands of the bf16 MFMA block: the three bf16 pieces of every
// value (see split3), laid out tile by tile in the order the lanes of a wavefront consume them.
// Tile (nb, kt) covers rows n = nb*32 .. +31 and k = kt*16 .. +15 of the operand B[n][k]; it holds
// per piece 64 x 16 bytes: lane l's eight values B[nb*32 + (l & 31)][kt*16 + (l >> 5)*8 + 0..7].
// A wavefront fetches a piece of a tile with one fully coalesced 1 KiB load straight into the
// registers of the MFMA: no staging through LDS, no arithmetic.  Tiles beyond the matrix (the
// launcher pads the tile grid to what its kernels walk) hold zeros, so the consumers need no bounds.
constexpr int WTILE = 3 * 512;            // bf16 values of one tile
// One workgroup reads a block of 32 rows x 64 columns of a row-major matrix W [R][C] (coalesced),
// and writes the tiles that block contributes to both operand forms: B[n = row][k = column]
// (four tiles along k) and B[n = column][k = row] (two tile rows x two k-tiles).
__global__ __launch_bounds__(256) void weight_pieces_kernel(const PieceJobs J) {
    __shared__ float blk[32][65];
    int j = 0;
#pragma unroll
    for (int i = 1; i < PIECE_MAX_JOBS; ++i)
        if (i < J.count && (int)blockIdx.x >= J.block0[i]) j = i;
    PieceJob jb = J.job[0];
#pragma unroll
    for (int i = 1; i < PIECE_MAX_JOBS; ++i)
        if (i == j) jb = J.job[i];
    const int b = (int)blockIdx.x - J.block0[j];
    const int cblocks = (jb.C + 63) / 64;
    const int r0 = (b / cblocks) * 32, c0 = (b % cblocks) * 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int q = 0; q < 2; ++q) {         // 512 float4 of the block, 16 per row
        const int idx = tid + q * 256, r = idx >> 4, c4 = (idx & 15) * 4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r0 + r < jb.R && c0 + c4 < jb.C) v = *reinterpret_cast<const float4*>(jb.W + (size_t)(r0 + r) * jb.C + c0 + c4);
        blk[r][c4 + 0] = v.x; blk[r][c4 + 1] = v.y; blk[r][c4 + 2] = v.z; blk[r][c4 + 3] = v.w;
    }
    __syncthreads();
    float v[8];
    // B[n = row][k = column]: wavefront w writes k-tile w of the block
    {
        const int kt = c0 / 16 + wave, KT = (jb.C + 15) / 16;
        if (kt < KT) {
            const int n = lane & 31, kk = wave * 16 + (lane >> 5) * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = blk[n][kk + e];
            const Pieces p0 = split3(make_float4(v[0], v[1], v[2], v[3])), p1 = split3(make_float4(v[4], v[5], v[6], v[7]));
            uint16_t* out = jb.out_rk + ((size_t)(r0 / 32) * KT + kt) * WTILE + lane * 8;
            *reinterpret_cast<uint4*>(out) = make_uint4(p0.h.x, p0.h.y, p1.h.x, p1.h.y);
            *reinterpret_cast<uint4*>(out + 512) = make_uint4(p0.m.x, p0.m.y, p1.m.x, p1.m.y);
            *reinterpret_cast<uint4*>(out + 1024) = make_uint4(p0.l.x, p0.l.y, p1.l.x, p1.l.y);
        }
    }
    // B[n = column][k = row]: wavefront w writes tile row w / 2, k-tile w % 2 of the block
    {
        const int nb = c0 / 32 + (wave >> 1), kt = r0 / 16 + (wave & 1), KT = (jb.R + 15) / 16;
        if (nb < (jb.C + 31) / 32 && kt < KT) {
            const int n = (wave >> 1) * 32 + (lane & 31), kk = (wave & 1) * 16 + (lane >> 5) * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = blk[kk + e][n];
            const Pieces p0 = split3(make_float4(v[0], v[1], v[2], v[3])), p1 = split3(make_float4(v[4], v[5], v[6], v[7]));
            uint16_t* out = jb.out_ck + ((size_t)nb * KT + kt) * WTILE + lane * 8;
            *reinterpret_cast<uint4*>(out) = make_uint4(p0.h.x, p0.h.y, p1.h.x, p1.h.y);
            *reinterpret_cast<uint4*>(out + 512) = make_uint4(p0.m.x, p0.m.y, p1.m.x, p1.m.y);
            *reinterpret_cast<uint4*>(out + 1024) = make_uint4(p0.l.x, p0.l.y, p1.l.x, p1.l.y);
        }
    }
}

// (at: the lane's place in the first piece of a tile)
__device__ __forceinline__ bf16x8 piece_at(const uint16_t* at, int q) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(at + q * 512));
}

template <int BM, int BN, int NW, bool AK, bool BKC, bool SPLIT = false, int PF = 1, bool BP = false, bool AP = false>
__global__ __launch_bounds__(NW * 64) void gemm_kernel(const GemmGroup g) {
    static_assert(!BP || (SPLIT && AK), "B operand from split pieces: split route with k-contiguous A only");
    static_assert(!AP || (BP && BM == 32), "A operand from split pieces: with B from pieces, one block of rows");
    static_assert(!SPLIT || BK == 16, "split path: one 32x32x16 MFMA step per staged tile");
    __shared__ __attribute__((aligned(16))) float smem[Smem<BM, BN, NW, SPLIT, BP, AP>::FLOATS];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    // which problem of the group this workgroup works on (uniform, stays in scalar registers)
    int p = 0, first = g.tile_start[0], last = g.tile_start[1];
#pragma unroll
    for (int i = 1; i < GEMM_MAX_GROUP; ++i)
        if (i < g.count && (int)blockIdx.x >= g.tile_start[i]) {
            p = i;
            first = g.tile_start[i];
            last = g.tile_start[i + 1];
        }
    const GemmArgs& a = g.p[p];        // (the group lies in the kernel argument segment: a scalar load at a uniform offset)
    // Workgroups are dealt round-robin to the 8 dies, each with its own L2.  Every problem
    // owns a multiple of 8 workgroups, and die x takes the x-th eighth of the problem's
    // tiles, ordered so that this eighth is a slab along the longer output side: a die then
    // reads one slab of one operand and the whole of the other, not both whole.
    const int local = (int)blockIdx.x - first;
    const int per_die = (last - first) >> 3;
    const int tile = (local & 7) * per_die + (local >> 3);
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    if (tile >= tiles_m * tiles_n) return;
    const bool m_major = a.M >= a.N;
    const int m0 = (m_major ? tile / tiles_n : tile % tiles_m) * BM;
    const int n0 = (m_major ? tile % tiles_n : tile / tiles_m) * BN;
    const bool first_n_tile = n0 == 0;
    constexpr int TM = BM / 32, TN = BN / 32;
    constexpr int LDA = BM + PAD, LDB = BN + PAD;
    // (SPLIT: per 32 rows of an operand three pieces, SUBTILE bf16 = 960 floats)
    float* As = smem + (SPLIT ? wave * ((AP ? 0 : TM) + (BP ? 0 : TN)) * 960 : wave * BK * (LDA + LDB));     // [BK][LDA] of this wavefront
    float* Bs = As + (SPLIT ? (AP ? 0 : TM) * 960 : BK * LDA);                                      // [BK][LDB]

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    constexpr int LA = BM * BK / 4 / 64;   // float4 per lane per tile
    constexpr int LB = BN * BK / 4 / 64;
    float4 ra[PF][LA], rd[PF][LA], rb[PF][LB];
    bf16x8 bq[PF][BP ? BN / 32 : 1][3];       // BP: the B operand blocks of a tile, ready for the MFMA
    bf16x8 aq[PF][3];                         // AP: the A operand block likewise
    const bool has_add = AK && a.a_ref != nullptr && a.a_add_idx != nullptr;   // uniform
    const bool copy_out = AK && a.a_copy != nullptr && first_n_tile;           // uniform

    // rows of A (k-contiguous layout), possibly assembled from references: resolved once
    // per lane; rows past M point at row M-1 and are zeroed after the load
    const float* arow[LA];
    const float* aadd[LA];
    bool avalid[LA];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        arow[i] = a.A;
        aadd[i] = a.A;
        avalid[i] = false;
        if (AK && !AP) {
            const int gm = m0 + (lane + i * 64) / (BK / 4);
            avalid[i] = gm < a.M;
            const int gmc = min(gm, a.M - 1);
            if (a.a_ref) {
                const int32_t r = a.a_ref[gmc];
                arow[i] = r >= 0 ? a.a_base0 + (size_t)r * a.lda : a.a_base1 + (size_t)(-1 - r) * a.lda;
                if (a.a_add_idx) aadd[i] = a.a_add + (size_t)a.a_add_idx[gmc] * a.lda;
            } else {
                arow[i] = a.A + (size_t)gmc * a.lda;
            }
        }
    }

    // Epilogue operands of this thread's output elements (clamped addresses, uniform flags).
    // Small tiles (launches that are latency bound) request them here, ahead of the k loop, so
    // that nothing is waited for after the last MFMA; large tiles request them after the loop:
    // held across it they would cost the registers of a second resident wavefront per SIMD (the
    // 4-wavefront small tile with split arithmetic likewise: 5 instead of 4 wavefronts per SIMD).
    constexpr int EPT = BM * BN / (NW * 64);
    constexpr bool EARLY_EPILOGUE = BM * BN <= 32 * 32 && !(SPLIT && NW == 4) && PF == 1;
    float e_bias[EPT], e_mask[EPT], e_add[EPT];
    int e_orow[EPT];
    const bool has_bias = a.bias != nullptr, has_mask = a.mask != nullptr, has_addend = a.addend != nullptr,
               has_dst = a.dst_row != nullptr;
#define NGDB_LOAD_EPILOGUE()                                                                \
    _Pragma("unroll") for (int q = 0; q < EPT; ++q) {                                      \
        const int e = tid + q * NW * 64;                                                    \
        const int lr = e / BN, lc = e % BN;                                                 \
        const int row = min(m0 + lr, a.M - 1), col = min(n0 + lc, a.N - 1);                 \
        e_bias[q] = has_bias ? a.bias[col] : 0.f;                                           \
        e_mask[q] = has_mask ? a.mask[(size_t)row * a.ldmask + col] : 1.f;                  \
        e_add[q] = has_addend ? a.addend[(size_t)row * a.ldadd + col] : 0.f;                \
        e_orow[q] = has_dst ? a.dst_row[row] : row;                                         \
    }
    if (EARLY_EPILOGUE) { NGDB_LOAD_EPILOGUE() }

    // A wavefront stages its tiles in its own LDS area and LDS executes a wavefront's
    // instructions in order, so the k loop needs no workgroup barrier: wavefronts run
    // independently (their memory waits do not line up) and only over the tiles they own.
    const int nk = (a.K + BK - 1) / BK;
    const int rounds = nk > wave ? (nk - wave + NW - 1) / NW : 0;
    // (operands that come as fp32 values, to be staged, and operands that come as pieces)
#define NGDB_ISSUE_VALUES(u, kc)                                                             \
    if (AP) {                                                                                \
    } else if (SPLIT && !AK) {                                                               \
        _Pragma("unroll") for (int t = 0; t < TM; ++t)                                      \
            issue_strided(a.A, a.lda, a.K, a.M, kc, m0 + 32 * t, lane, reinterpret_cast<float4(&)[2]>(ra[u][2 * t])); \
    } else {                                                                                 \
        issue_a<BM, LA, AK>(a, lane, m0, kc, has_add, arow, aadd, ra[u], rd[u]);            \
    }                                                                                        \
    if (BP) {                                                                                \
    } else if (SPLIT && !BKC) {                                                              \
        _Pragma("unroll") for (int t = 0; t < TN; ++t)                                      \
            issue_strided(a.B, a.ldb, a.K, a.N, kc, n0 + 32 * t, lane, reinterpret_cast<float4(&)[2]>(rb[u][2 * t])); \
    } else {                                                                                 \
        issue_b<BN, LB, BKC>(a, lane, n0, kc, rb[u]);                                       \
    }
#define NGDB_ISSUE_PIECES(u, kc, live)                                                       \
    if (AP) {                                                                                \
        const uint16_t* at = (live) ? a.a_pieces + ((size_t)(m0 / 32) * a.a_kt + (kc) / BK) * WTILE + lane * 8 : a.a_pieces; \
        _Pragma("unroll") for (int q = 0; q < 3; ++q) aq[u][q] = piece_at(at, q);           \
    }                                                                                        \
    if (BP) {                                                                                \
        _Pragma("unroll") for (int j = 0; j < BN / 32; ++j) {                               \
            const uint16_t* at = (live) ? a.b_pieces + ((size_t)(n0 / 32 + j) * a.b_kt + (kc) / BK) * WTILE + lane * 8 : a.b_pieces; \
            _Pragma("unroll") for (int q = 0; q < 3; ++q) bq[u][BP ? j : 0][q] = piece_at(at, q); \
        }                                                                                    \
    }
    // PF tiles are in flight per wavefront.  With more than one, every stage of the loop requests
    // its next tile whether or not there is one (beyond the end: the first k-tile once more for the
    // staged values, one 16-byte word for all lanes for the pieces, neither used): with the same
    // loads on every path the compiler can wait for a stage's own loads alone (vmcnt = what was
    // requested after them), where a request under a condition makes it wait for everything outstanding.
#pragma unroll
    for (int u = 0; u < PF; ++u) {
        const bool live = u < rounds;
        const int kc = live ? (u * NW + wave) * BK : 0;
        if (SPLIT && PF > 1) {
            NGDB_ISSUE_VALUES(u, kc)
            NGDB_ISSUE_PIECES(u, kc, live)
        } else if (live) {
            NGDB_ISSUE_VALUES(u, kc)
            NGDB_ISSUE_PIECES(u, kc, true)
        }
    }
    for (int it0 = 0; SPLIT && it0 < rounds; it0 += PF) {
#pragma unroll
      for (int u = 0; u < PF; ++u) {
        const int it = it0 + u;
        const bool live_next = it + PF < rounds;
        const int knext = live_next ? ((it + PF) * NW + wave) * BK : 0;
        if (it < rounds) {
            const int kcur = (it * NW + wave) * BK;
            uint16_t* Ap = reinterpret_cast<uint16_t*>(As);
            uint16_t* Bp = reinterpret_cast<uint16_t*>(Bs);
            if (!AK) {
#pragma unroll
                for (int t = 0; t < TM; ++t)
                    stage_strided(Ap + t * SUBTILE, a.K, a.M, kcur, m0 + 32 * t, lane,
                                  reinterpret_cast<const float4(&)[2]>(ra[u][2 * t]));
            }
#pragma unroll
            for (int i = 0; AK && !AP && i < LA; ++i) {
                const int idx = lane + i * 64;
                const int m = idx / (BK / 4), kq = idx % (BK / 4);
                const int gk = kcur + kq * 4;
                float4 v = ra[u][i];
                if (has_add) { v.x += rd[u][i].x; v.y += rd[u][i].y; v.z += rd[u][i].z; v.w += rd[u][i].w; }
                const bool ok = avalid[i] && gk < a.K;
                v.x = ok ? v.x : 0.f; v.y = ok ? v.y : 0.f; v.z = ok ? v.z : 0.f; v.w = ok ? v.w : 0.f;
                if (copy_out && ok) *reinterpret_cast<float4*>(a.a_copy + (size_t)(m0 + m) * a.lda + gk) = v;
                store_pieces(Ap + (m >> 5) * SUBTILE, m & 31, kq, split3(v));
            }
            if (!BKC && !BP) {
#pragma unroll
                for (int t = 0; t < TN; ++t)
                    stage_strided(Bp + t * SUBTILE, a.K, a.N, kcur, n0 + 32 * t, lane,
                                  reinterpret_cast<const float4(&)[2]>(rb[u][2 * t]));
            }
#pragma unroll
            for (int i = 0; BKC && !BP && i < LB; ++i) {
                const int idx = lane + i * 64;
                const int n = idx / (BK / 4), kq = idx % (BK / 4);
                float4 v = rb[u][i];
                const bool ok = n0 + n < a.N && kcur + kq * 4 < a.K;
                v.x = ok ? v.x : 0.f; v.y = ok ? v.y : 0.f; v.z = ok ? v.z : 0.f; v.w = ok ? v.w : 0.f;
                store_pieces(Bp + (n >> 5) * SUBTILE, n & 31, kq, split3(v));
            }
            if (!AP) __builtin_amdgcn_wave_barrier();
            // Operands that came as pieces are multiplied from the registers they were loaded into, and
            // those registers are requested again only after the MFMAs: copied aside first, the compiler
            // would load into temporaries and wait for them in the middle of the MFMAs.
            bf16x8 ap[TM][3], bp[TN][3];
            if (AP) {
#pragma unroll
                for (int q = 0; q < 3; ++q) ap[0][q] = aq[u][q];
            }
            if (BP) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int q = 0; q < 3; ++q) bp[j][q] = bq[u][BP ? j : 0][q];
            }
            // the staged values' registers are free again: their next tile is under way during the MFMAs
            // (one tile in flight: nothing for the compiler to count, and no request beyond the end)
            if (PF == 1 && live_next) { NGDB_ISSUE_VALUES(u, knext) }
#pragma unroll
            for (int q = 0; q < 3; ++q) {
#pragma unroll
                for (int i = 0; !AP && i < TM; ++i)
                    ap[i][q] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Ap + i * SUBTILE + q * PIECE + unit_at<!AK>(lane)));
#pragma unroll
                for (int j = 0; !BP && j < TN; ++j)
                    bp[j][q] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(Bp + j * SUBTILE + q * PIECE + unit_at<!BKC>(lane)));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {   // smallest products first
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ap[i][2], bp[j][0], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ap[i][0], bp[j][2], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ap[i][1], bp[j][1], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ap[i][1], bp[j][0], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ap[i][0], bp[j][1], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ap[i][0], bp[j][0], acc[i][j], 0, 0, 0);
                }
            if (!AP) __builtin_amdgcn_wave_barrier();
        }
        __builtin_amdgcn_sched_barrier(0);
        if (PF > 1) { NGDB_ISSUE_VALUES(u, knext) }
        if (PF > 1 || live_next) {
            NGDB_ISSUE_PIECES(u, knext, live_next)
        }
      }
    }
    for (int it0 = 0; !SPLIT && it0 < rounds; it0 += PF) {
#pragma unroll
      for (int u = 0; u < PF; ++u) {
        const int it = it0 + u;
        if (it >= rounds) break;
        const int kcur = (it * NW + wave) * BK;
        stage_a<BM, LA, LDA, AK>(a, As, lane, m0, kcur, has_add, copy_out, avalid, ra[u], rd[u]);
        stage_b<BN, LB, LDB, BKC>(a, Bs, lane, n0, kcur, rb[u]);
        __builtin_amdgcn_wave_barrier();        // staged tile before its reads (compiler ordering only)
        if (it + PF < rounds) {
            const int kc = ((it + PF) * NW + wave) * BK;
            NGDB_ISSUE_VALUES(u, kc)
        }
        // all LDS operand reads of the tile are issued before the first MFMA, so that the
        // matrix pipe never waits for an LDS round trip between k steps
        float av[BK / 2][TM], bv[BK / 2][TN];
#pragma unroll
        for (int kk = 0; kk < BK / 2; ++kk) {
            const int krow = kk * 2 + (lane >> 5);
#pragma unroll
            for (int i = 0; i < TM; ++i) av[kk][i] = As[krow * LDA + i * 32 + (lane & 31)];
#pragma unroll
            for (int j = 0; j < TN; ++j) bv[kk][j] = Bs[krow * LDB + j * 32 + (lane & 31)];
        }
        __builtin_amdgcn_sched_barrier(0);      // keep the reads ahead of the MFMAs
#pragma unroll
        for (int kk = 0; kk < BK / 2; ++kk)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[kk][i], bv[kk][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_wave_barrier();        // reads of this tile before the next one is staged
      }
    }
    if (!EARLY_EPILOGUE) { NGDB_LOAD_EPILOGUE() }   // in flight during the reduction
#undef NGDB_LOAD_EPILOGUE
#undef NGDB_ISSUE_VALUES
#undef NGDB_ISSUE_PIECES
    __syncthreads();                            // the staging areas are reused for the reduction

    // partial tiles -> LDS.  Accumulator layout of a 32x32 block: lane owns column
    // (lane & 31) and rows 8*(r/4) + 4*(lane/32) + r%4, r = 0..15.
    constexpr int NR = Smem<BM, BN, NW, SPLIT, BP, AP>::NR;
    float* red = smem + (wave % NR) * BM * (BN + 1);
#define NGDB_ACC_TO_LDS()                                                                   \
    _Pragma("unroll") for (int i = 0; i < TM; ++i)                                         \
    _Pragma("unroll") for (int j = 0; j < TN; ++j)                                         \
    _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                       \
        const int row = i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);                  \
        red[row * (BN + 1) + j * 32 + (lane & 31)] = acc[i][j][r];                          \
    }
    if (NW > NR) {   // fold the upper half of the wavefronts into the lower half first
        if (wave >= NR) { NGDB_ACC_TO_LDS() }
        __syncthreads();
        if (wave < NR) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int row = i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                        acc[i][j][r] += red[row * (BN + 1) + j * 32 + (lane & 31)];
                    }
        }
        __syncthreads();
    }
    if (wave < NR) { NGDB_ACC_TO_LDS() }
#undef NGDB_ACC_TO_LDS
    __syncthreads();

    // epilogue: the partial tiles are summed, the operands requested before the k loop applied
    const bool emit = a.c_pieces != nullptr;    // uniform
#pragma unroll
    for (int q = 0; q < EPT; ++q) {
        const int e = tid + q * NW * 64;
        const int lr = e / BN, lc = e % BN;
        float v = smem[lr * (BN + 1) + lc];
#pragma unroll
        for (int w = 1; w < NR; ++w) v += smem[w * BM * (BN + 1) + lr * (BN + 1) + lc];
        v += e_bias[q];
        if (a.relu) v = fmaxf(v, 0.f);
        v = e_mask[q] > 0.f ? v : 0.f;
        v += e_add[q];
        const bool inside = m0 + lr < a.M && n0 + lc < a.N;
        if (inside) a.C[(size_t)e_orow[q] * a.ldc + n0 + lc] = v;
        // (a slot of the first partial tile is read by the thread that owns the element only)
        if (BM == 32 && BN == 32 && SPLIT && emit) smem[lr * (BN + 1) + lc] = inside ? v : 0.f;
    }
    // The output once more as bf16 pieces in tile order (zero beyond the matrix), for the launch that
    // takes it as its A operand: block row m0/32, k-tiles n0/16 and n0/16 + 1; a lane of the first
    // two wavefronts splits eight consecutive values of a row.
    if (BM == 32 && BN == 32 && SPLIT && emit) {
        __syncthreads();
        if (tid < 128) {
            const int lr = tid & 31, u = tid >> 5;
            float x[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) x[j] = smem[lr * (BN + 1) + u * 8 + j];
            const Pieces p0 = split3(make_float4(x[0], x[1], x[2], x[3])), p1 = split3(make_float4(x[4], x[5], x[6], x[7]));
            uint16_t* out = a.c_pieces + ((size_t)(m0 / 32) * a.c_kt + n0 / 16 + (u >> 1)) * WTILE + ((u & 1) * 32 + lr) * 8;
            *reinterpret_cast<uint4*>(out) = make_uint4(p0.h.x, p0.h.y, p1.h.x, p1.h.y);
            *reinterpret_cast<uint4*>(out + 512) = make_uint4(p0.m.x, p0.m.y, p1.m.x, p1.m.y);
            *reinterpret_cast<uint4*>(out + 1024) = make_uint4(p0.l.x, p0.l.y, p1.l.x, p1.l.y);
        }
    }
}

template <int BM, int BN, int NW, bool SPLIT = false>
hipError_t dispatch_layout(GemmGroup& g, hipStream_t s) {
    int tiles = 0;
    for (int i = 0; i < g.count; ++i) {
        g.tile_start[i] = tiles;
        tiles += (((g.p[i].M + BM - 1) / BM) * ((g.p[i].N + BN - 1) / BN) + 7) / 8 * 8;
    }
    for (int i = g.count; i <= GEMM_MAX_GROUP; ++i) g.tile_start[i] = tiles;
    dim3 grid(tiles), block(NW * 64);
    const GemmArgs& a = g.p[0];
    if (a.a_kcontig && a.b_kcontig)
        hipLaunchKernelGGL((gemm_kernel<BM, BN, NW, true, true, SPLIT>), grid, block, 0, s, g);
    else if (a.a_kcontig && !a.b_kcontig)
        hipLaunchKernelGGL((gemm_kernel<BM, BN, NW, true, false, SPLIT>), grid, block, 0, s, g);
    else if (!a.a_kcontig && !a.b_kcontig)
        hipLaunchKernelGGL((gemm_kernel<BM, BN, NW, false, false, SPLIT>), grid, block, 0, s, g);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

template <int NW, bool AP, int PF>
hipError_t dispatch_pieces(GemmGroup& g, hipStream_t s) {
    constexpr int BM = 32, BN = 32;
    int tiles = 0;
    for (int i = 0; i < g.count; ++i) {
        g.tile_start[i] = tiles;
        tiles += (((g.p[i].M + BM - 1) / BM) * ((g.p[i].N + BN - 1) / BN) + 7) / 8 * 8;
    }
    for (int i = g.count; i <= GEMM_MAX_GROUP; ++i) g.tile_start[i] = tiles;
    hipLaunchKernelGGL((gemm_kernel<BM, BN, NW, true, true, true, PF, true, AP>), dim3(tiles), dim3(NW * 64), 0, s, g);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_group(const GemmArgs* problems, int count, hipStream_t s, int* route, bool* emitted) {
    if (route) *route = GEMM_FP32;
    if (emitted) *emitted = false;
    GemmGroup g{};
    uint16_t* c_pieces[GEMM_MAX_GROUP] = {};
    long blocks_small = 0;
    int max_k = 0;
    for (int i = 0; i < count; ++i) {
        const GemmArgs& a = problems[i];
        if (a.M <= 0 || a.N <= 0) continue;
        if (g.count == GEMM_MAX_GROUP) return hipErrorInvalidValue;
        // float4 operand loads: leading dimensions and the contiguous extents must be multiples of 4
        if ((a.lda & 3) || (a.ldb & 3)) return hipErrorInvalidValue;
        if ((a.a_kcontig ? a.K : a.M) & 3) return hipErrorInvalidValue;
        if ((a.b_kcontig ? a.K : a.N) & 3) return hipErrorInvalidValue;
        if (a.a_ref && !a.a_kcontig) return hipErrorInvalidValue;
        if (g.count && (a.a_kcontig != g.p[0].a_kcontig || a.b_kcontig != g.p[0].b_kcontig))
            return hipErrorInvalidValue;   // one operand layout per launch
        if (g.count && a.arith != g.p[0].arith) return hipErrorInvalidValue;
        c_pieces[g.count] = a.c_pieces;
        g.p[g.count] = a;
        g.p[g.count++].c_pieces = nullptr;    // (only the kernels chosen below for ready-made B operands write them)
        blocks_small += (long)((a.M + 31) / 32) * ((a.N + 63) / 64);
        max_k = std::max(max_k, a.K);
    }
    if (g.count == 0) return hipSuccess;
    const int arith = g.p[0].arith;
    const bool auto_split = arith == GEMM_AUTO && g.p[0].a_kcontig && max_k >= 128;
    // weight gradients (k = all rows of an operator type) of a mid-size step: the large tile with
    // the split route beats the small tile with fp32 MFMAs although it leaves compute units idle
    const bool wgrad_big_tile = arith == GEMM_AUTO && !g.p[0].a_kcontig && max_k >= 512 && blocks_small >= 512;
    // (with the B operands ready-made the small tile holds its own up to twice the size: 0.516 + 0.388
    // against 0.537 + 0.416 ms for the forward and backward launches of 4096 queries at h = 800)
    bool b_ready = g.p[0].a_kcontig;
    for (int i = 0; i < g.count; ++i) b_ready = b_ready && g.p[i].b_pieces != nullptr && g.p[i].b_kt >= (g.p[i].K + 15) / 16;
    const long big_at = b_ready && auto_split ? 4096 : 2048;
    if ((blocks_small >= big_at || wgrad_big_tile) && arith != GEMM_SPLIT) {
        // (in the large tile every staged value feeds two MFMA blocks: there the split pays for
        // the weight gradients too)
        const bool big_split = arith == GEMM_AUTO && max_k >= 128;
        if (route && big_split) *route = GEMM_SPLIT;
        return big_split ? dispatch_layout<64, 64, 4, true>(g, s) : dispatch_layout<64, 64, 4>(g, s);
    }
    // below that the launches of a step do not fill the chip: the smallest tile the MFMA block
    // allows spreads a launch over the most compute units (a tile's MFMA work runs on one)
    // (more than two such tiles per compute unit: 4 wavefronts per tile keep them all resident)
    // fp32 operands as three bf16 pieces each (six bf16 MFMAs per k-tile instead of eight fp32
    // ones that take twice as long each): launches whose A operand is k-contiguous, i.e. the
    // forward and data-gradient contractions.  With k as the slow index of both operands (weight
    // gradients) splitting and transposing the pieces costs more than the matrix unit saves.
    // (with a k extent below 128 the matrix unit is idle either way and the splitting only adds work)
    if (arith == GEMM_SPLIT || auto_split) {
        if (route) *route = GEMM_SPLIT;
        // every B operand comes ready-made (weights split once per pass): no staging of B at all
        bool all_pieces = g.p[0].a_kcontig;
        for (int i = 0; i < g.count; ++i) all_pieces = all_pieces && g.p[i].b_pieces != nullptr && g.p[i].b_kt >= (g.p[i].K + 15) / 16;
        if (all_pieces) {
            // ... and the A operand too where the launch before left its output as pieces
            bool a_too = true;
            for (int i = 0; i < g.count; ++i)
                a_too = a_too && g.p[i].a_pieces != nullptr && !g.p[i].a_ref && !g.p[i].a_copy && g.p[i].a_kt >= (g.p[i].K + 15) / 16;
            // (only from launches that leave compute units idle: in a larger one the extra stores cost
            // more than the launch after it saves)
            if (emitted && blocks_small * 2 <= 512) {
                *emitted = true;
                for (int i = 0; i < g.count; ++i)
                    *emitted = *emitted && c_pieces[i] != nullptr && !g.p[i].dst_row && g.p[i].c_kt >= 2 * ((g.p[i].N + 31) / 32);
                for (int i = 0; i < g.count; ++i)
                    if (*emitted) g.p[i].c_pieces = c_pieces[i];
            }
            if (blocks_small * 2 > 512) return a_too ? dispatch_pieces<4, true, 2>(g, s) : dispatch_pieces<4, false, 1>(g, s);
            return a_too ? dispatch_pieces<8, true, 2>(g, s) : dispatch_pieces<8, false, 1>(g, s);
        }
        if (blocks_small * 2 > 512) return dispatch_layout<32, 32, 4, true>(g, s);
        return dispatch_layout<32, 32, 8, true>(g, s);
    }
    if (blocks_small * 2 > 512) return dispatch_layout<32, 32, 4>(g, s);
    return dispatch_layout<32, 32, 8>(g, s);
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s) { return launch_gemm_group(&a, 1, s, nullptr); }

hipError_t launch_weight_pieces(PieceJobs& J, hipStream_t s) {
    if (J.count <= 0) return hipSuccess;
    if (J.count > PIECE_MAX_JOBS) return hipErrorInvalidValue;
    int blocks = 0;
    for (int i = 0; i < J.count; ++i) {
        if ((J.job[i].C & 3) || J.job[i].R <= 0 || J.job[i].C <= 0) return hipErrorInvalidValue;
        J.block0[i] = blocks;
        blocks += ((J.job[i].R + 31) / 32) * ((J.job[i].C + 63) / 64);
    }
    J.block0[J.count] = blocks;
    hipLaunchKernelGGL(weight_pieces_kernel, dim3(blocks), dim3(256), 0, s, J);
    return hipGetLastError();
}

}  // namespace ngdb
