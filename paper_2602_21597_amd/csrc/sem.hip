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
// Both kernels bring their operand rows from global memory straight into LDS
// (direct loads, a few stages ahead, counted and waited for by hand) and keep one
// workgroup of large tiles per compute unit: what limits them is how many cache
// lines a compute unit has in flight, so every row piece is brought in as few
// times as the accumulator registers allow.  The gradient's operands both have
// the contraction index (rows) as the slow one: they are fetched from LDS with
// the transposing read of gfx950 instead of being transposed on the way in.
#include "common.h"

namespace ngdb {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int KS = 64;          // the feature width is a multiple of this
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
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

// ---- building blocks of the projection kernels (gfx950)
// A direct load from global memory into LDS: lane l's bytes land at lds_base + l * size, whatever
// global address the lane gives; lds_base is wave-uniform (it travels in M0).  The loads are
// issued from inline assembly and waited for by hand (s_waitcnt vmcnt): left to the compiler,
// every LDS read after such a load would wait for all of them, also those of the stages ahead.
__device__ __forceinline__ void lds_load16(const void* gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(gptr) : "memory");
}
__device__ __forceinline__ void lds_load4(const void* gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(gptr) : "memory");
}
// at most n vector-memory operations of this wavefront still in flight (they complete in order)
template <int N>
__device__ __forceinline__ void wait_vm() {
    static_assert(N >= 0 && N < 64, "vmcnt has 6 bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}
// Transposing LDS read of 16-bit values: within 16 lanes, lane 4r + c gives the address of 4
// consecutive values of row r (c-th group of 4 columns); lane i receives column i of the
// 4 x 16 block: rows 0..3.  Two of them make the 8 consecutive k of a 16x16x32 MFMA operand
// from a tile that is stored with k as the slow index.
typedef short short4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ short4v read_tr(const uint16_t* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)p);
}
__device__ __forceinline__ bf16x8 join8(short4v a, short4v b) {
    typedef short short8v __attribute__((ext_vector_type(8)));
    return __builtin_bit_cast(bf16x8, short8v{a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]});
}

// ------------------------------------------------------------------ forward
// out[u, :] = E[id(u), :] + Wb * H[id(u), :].  Workgroup tile: 256 rows x 208 coordinates (two
// tiles cover d = 400, so a feature row is brought into LDS twice), k stages of 64 = 128 bytes of
// every row = one cache line per row and stage.  What bounds the kernel is the number of cache
// lines a compute unit can have in flight (its L1 miss queue: about 35 GB/s per unit at the
// latency of an L2 hit under load, whatever the LDS could buffer), so every request is a whole
// line, the tile is as wide as the accumulators allow, and two stages in LDS (one being multiplied,
// one landing) are as good as more.
// A stage is 64 direct loads of 1 KiB, 8 per wavefront: load l of an area covers rows 8l .. 8l+7,
// 128 bytes each; a lane's 16 bytes land at its lane number, so the lane picks the column that
// belongs there: column c of row r is stored at c ^ (r / 2 % 8), which spreads the 16 rows x 16
// bytes one MFMA operand fetch touches over all banks.
constexpr int SF_BU = 256, SF_N = 208, SF_NBLK = SF_N / 16, SF_KS = 64;
constexpr int SF_NW = 8;                                      // wavefronts: 32 rows x 208 coordinates each (104 accumulator registers)
constexpr int SF_HL = SF_BU / 8, SF_WL = 32;                  // loads per stage: feature rows, weight rows (26 used)
constexpr int SF_STAGE = (SF_HL + SF_WL) * 1024, SF_NB = 2, SF_PER_WAVE = (SF_HL + SF_WL) / SF_NW;
__global__ __launch_bounds__(SF_NW * 64) void sem_fuse_kernel(const SemFuseArgs a) {
    __shared__ __attribute__((aligned(1024))) unsigned char tiles[SF_NB * SF_STAGE];
    const int n_rows = a.n_rows_dev ? min(*a.n_rows_dev, a.n_rows) : a.n_rows;
    const int n_tiles = (a.d + SF_N - 1) / SF_N;
    // workgroups are dealt round-robin to the 8 dies: the coordinate tiles of one
    // row tile go to the same die one after the other and share its L2
    const int die = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int u0 = ((j / n_tiles) * 8 + die) * SF_BU;
    const int n0 = (j % n_tiles) * SF_N;
    if (u0 >= n_rows) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // entity of a row of the tile (rows past the end: the last row's); the row numbers are read
    // unconditionally (from a valid address when the rows are consecutive entities)
    const bool listed = a.ids != nullptr;
    const int32_t* id_src = listed ? a.ids : reinterpret_cast<const int32_t*>(a.E);
    constexpr int HQ = SF_HL / SF_NW, WQ = SF_WL / SF_NW;     // loads per wavefront: 4 + 4
    int urow[HQ + 2];
#pragma unroll
    for (int q = 0; q < HQ; ++q) urow[q] = min(u0 + (wave + SF_NW * q) * 8 + (lane >> 3), n_rows - 1);   // feature rows this lane fetches
#pragma unroll
    for (int q = 0; q < 2; ++q) urow[HQ + q] = min(u0 + wave * 32 + q * 16 + (lane & 15), n_rows - 1);   // rows of its accumulator blocks
    int32_t listed_id[HQ + 2];
#pragma unroll
    for (int q = 0; q < HQ + 2; ++q) listed_id[q] = id_src[listed ? urow[q] : 0];
    int64_t ent[HQ + 2];
#pragma unroll
    for (int q = 0; q < HQ + 2; ++q) ent[q] = listed ? (int64_t)listed_id[q] : a.id_base + urow[q];
    // sources of this lane's loads at k = 0 (row r of the area = 8 * load + lane / 8, stored column lane % 8)
    const uint16_t* src[SF_PER_WAVE];
#pragma unroll
    for (int q = 0; q < HQ; ++q) {
        const int r = (wave + SF_NW * q) * 8 + (lane >> 3);
        src[q] = a.H + ent[q] * a.ds + ((lane & 7) ^ ((r >> 1) & 7)) * 8;
    }
#pragma unroll
    for (int q = 0; q < WQ; ++q) {
        const int r = (wave + SF_NW * q) * 8 + (lane >> 3);          // (rows past the tile's 208: padding, the last row again)
        src[HQ + q] = a.Wb + (size_t)min(n0 + min(r, SF_N - 1), a.d - 1) * a.ds + ((lane & 7) ^ ((r >> 1) & 7)) * 8;
    }
    // The accumulators start from the structural rows: a lane holds, per block, 4 consecutive
    // coordinates of one row (clamped addresses; rows and coordinates past the end are never stored).
    floatx4 acc[2][SF_NBLK];
#pragma unroll
    for (int bu = 0; bu < 2; ++bu) {
        const float* erow = a.E + ent[HQ + bu] * a.d;
#pragma unroll
        for (int bn = 0; bn < SF_NBLK; ++bn) {
            const float4 e = *reinterpret_cast<const float4*>(erow + min(n0 + bn * 16 + (lane >> 4) * 4, a.d - 4));
            acc[bu][bn] = floatx4{e.x, e.y, e.z, e.w};
        }
    }
    const uint32_t tiles_at = lds_addr(tiles);
    const int stages = a.ds / SF_KS;
    auto issue = [&](int s) {                // (stages past the end fetch the last one again; nobody reads them)
        const int k0 = min(s, stages - 1) * SF_KS;
        const uint32_t base = tiles_at + (uint32_t)(s % SF_NB) * SF_STAGE;
#pragma unroll
        for (int q = 0; q < HQ; ++q) lds_load16(src[q] + k0, base + (uint32_t)(wave + SF_NW * q) * 1024u);
#pragma unroll
        for (int q = 0; q < WQ; ++q) lds_load16(src[HQ + q] + k0, base + (uint32_t)(SF_HL + wave + SF_NW * q) * 1024u);
    };
    issue(0);
    issue(1);
    // The structural rows have to be in their registers before the loop: the compiler's own count of
    // loads in flight does not know the direct loads, and its waits inside the loop would throttle them.
    wait_vm<0>();
    // operand fetch: row R = 16 b + lane % 16 of an area, columns 4 h + lane / 16 (h = which half of the stage's k)
    const int ri = lane & 15;
    int frag_at[2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
        frag_at[h] = (ri >> 3) * 1024 + (ri & 7) * 128 + (((4 * h + (lane >> 4)) ^ ((ri >> 1) & 7))) * 16;
    for (int s = 0; s < stages; ++s) {
        wait_vm<SF_PER_WAVE>();              // all but the next stage's loads: stage s is in LDS
        __syncthreads();                     // ... every wavefront's part of it
        const unsigned char* buf = tiles + (s % SF_NB) * SF_STAGE;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            bf16x8 fh[2], fw[SF_NBLK];
#pragma unroll
            for (int bu = 0; bu < 2; ++bu)
                fh[bu] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(buf + (wave * 2 + bu) * 2048 + frag_at[h]));
#pragma unroll
            for (int bn = 0; bn < SF_NBLK; ++bn)
                fw[bn] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(buf + SF_HL * 1024 + bn * 2048 + frag_at[h]));
#pragma unroll
            for (int bu = 0; bu < 2; ++bu)
#pragma unroll
                for (int bn = 0; bn < SF_NBLK; ++bn)
                    acc[bu][bn] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw[bn], fh[bu], acc[bu][bn], 0, 0, 0);
        }
        __syncthreads();                     // everybody is done with this buffer
        issue(s + 2);
    }
    wait_vm<0>();                            // the loads issued past the end land before the workgroup gives up its LDS
#pragma unroll
    for (int bu = 0; bu < 2; ++bu) {
        const int u = u0 + wave * 32 + bu * 16 + (lane & 15);
        if (u >= n_rows) continue;
        float* orow = a.out + (size_t)u * a.d;
#pragma unroll
        for (int bn = 0; bn < SF_NBLK; ++bn) {
            const int n = n0 + bn * 16 + (lane >> 4) * 4;
            if (n >= a.d) continue;
            *reinterpret_cast<float4*>(orow + n) =
                make_float4(acc[bu][bn][0], acc[bu][bn][1], acc[bu][bn][2], acc[bu][bn][3]);
        }
    }
}

// ------------------------------------------------------------------ gradient of Wp
constexpr int WG_SEM = 256;     // text-feature coordinates per workgroup tile of the gradient

// LDS of one 32-row stage: H rows [32][256 feature coordinates] at a pitch of 544 bytes (34
// chunks of 16: with 17 * 32 bytes per row the 16 consecutive rows one transposing read touches
// spread over all banks), G rows [32][208 embedding coordinates] at 416 bytes (13 * 32: likewise).
constexpr int WG_KS = 32;                                     // rows per stage = one MFMA step
constexpr int WG_M = 208, WG_MB = WG_M / 16;                  // embedding coordinates per workgroup tile, MFMA blocks
constexpr int WG_HP = 544, WG_GP = 2 * WG_M;                  // row pitches, bytes
constexpr int WG_HL = 19, WG_GL = 13;                         // wave-loads of 1 KiB per stage: H area (17 carry data), G area
constexpr int WG_STAGE = (WG_HL + WG_GL) * 1024;
constexpr int WG_NB = 4;                                      // stages in LDS: one multiplied, three in flight or landing
constexpr int WG_PER_WAVE = (WG_HL + WG_GL) / 4;              // data loads per wavefront and stage

// partial[split, m, n] = sum over the split's rows u of G[u, m] * H[id(u), n]
// Workgroup tile: 208 embedding x 256 feature coordinates (two tiles cover d = 400, so a feature
// row is brought into LDS twice per step and a gradient row four times; what bounds the kernel is
// the bytes a compute unit keeps in flight at the latency of a loaded memory system, so the tile
// is as large as the accumulators allow and LDS is all staging).  Rows travel from global memory straight into LDS
// (no registers, no transposition on the way): every wavefront issues 8 loads of 1 KiB per
// stage, up to three stages ahead of the one being multiplied, and one load of the row numbers
// two stages further; the operands of the MFMA blocks are fetched with transposing reads.
// One workgroup barrier per stage.
__global__ __launch_bounds__(256) void sem_wgrad_kernel(const SemWgradArgs a) {
    __shared__ __attribute__((aligned(1024))) unsigned char tiles[WG_NB * WG_STAGE];
    __shared__ __attribute__((aligned(256))) int32_t id_ring[4][3][64];     // per wavefront: row numbers of three stages
    const int n_rows = min(*a.n_rows_dev, a.n_rows);
    const int m_tiles = (a.d + WG_M - 1) / WG_M, n_tiles = (a.ds + WG_SEM - 1) / WG_SEM;
    const int tiles_mn = m_tiles * n_tiles;
    const int die = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int split = (j / tiles_mn) * 8 + die;
    if (split >= a.n_splits) return;
    const int tile = j % tiles_mn;
    const int m0 = (tile % m_tiles) * WG_M, n0 = (tile / m_tiles) * WG_SEM;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    const int stages = (n_rows + WG_KS - 1) / WG_KS;
    const int per_split = (stages + a.n_splits - 1) / a.n_splits;
    const int s_lo = split * per_split, s_hi = min(stages, s_lo + per_split);

    floatx4 acc[4][WG_MB];
#pragma unroll
    for (int bn = 0; bn < 4; ++bn)
#pragma unroll
        for (int bm = 0; bm < WG_MB; ++bm) acc[bn][bm] = floatx4{0.f, 0.f, 0.f, 0.f};

    if (s_lo < s_hi) {
        // What this lane fetches in each of its wavefront's loads of a stage (the same every stage).
        // The H tile is 32 rows x 34 chunks of 16 bytes = 17 loads of 64 chunks (chunk c = row c/34, column
        // c%34; columns 32 and 33 are padding and fetch columns 0 and 1 again), the G tile 32 x 26 = 13 loads.
        // Loads 0..18 of a stage go to the H area (17 carry the tile, 2 are padding), loads 19..31 are the G tile.
        constexpr int G_AT = WG_HL;                                       // the G tile starts at this KiB of the stage
        int row[WG_PER_WAVE], col[WG_PER_WAVE];
        bool is_h[WG_PER_WAVE];
#pragma unroll
        for (int q = 0; q < WG_PER_WAVE; ++q) {
            const int l = wave + 4 * q;                                   // load number within the stage, 0..31
            is_h[q] = l < G_AT;
            if (l < G_AT) {                                               // (loads 17, 18: padding, rows past the tile clamp to its last)
                const int c = l * 64 + lane;
                row[q] = min(c / 34, WG_KS - 1);
                col[q] = min(n0 + ((c % 34) & 31) * 8, a.ds - 8);
            } else {
                const int c = (l - G_AT) * 64 + lane;
                row[q] = min(c / (WG_GP / 16), WG_KS - 1);
                col[q] = min(m0 + (c % (WG_GP / 16)) * 8, a.d - 8);
            }
        }
        static_assert(WG_HL * 1024 >= WG_KS * WG_HP && WG_GL * 1024 >= WG_KS * WG_GP && (WG_HL + WG_GL) % 4 == 0, "stage layout");
        const uint32_t tiles_at = lds_addr(tiles), ring_at = lds_addr(&id_ring[wave][0][0]);
        auto issue_ids = [&](int s) {        // row numbers of stage s (rows past the end: the last row's)
            lds_load4(a.ids + min(s * WG_KS + (lane & (WG_KS - 1)), n_rows - 1), ring_at + (uint32_t)(s % 3) * 256u);
        };
        auto issue_data = [&](int s) {       // WG_PER_WAVE loads; needs the row numbers of stage s in the ring
            const uint32_t base = tiles_at + (uint32_t)(s % WG_NB) * WG_STAGE;
            const int32_t* ids = id_ring[wave][s % 3];
            int32_t id[WG_PER_WAVE];
#pragma unroll
            for (int q = 0; q < WG_PER_WAVE; ++q) id[q] = ids[row[q]];
#pragma unroll
            for (int q = 0; q < WG_PER_WAVE; ++q) {
                const uint16_t* src = is_h[q] ? a.H + (size_t)id[q] * a.ds + col[q]
                                              : a.G + (size_t)min(s * WG_KS + row[q], n_rows - 1) * a.d + col[q];
                lds_load16(src, base + (uint32_t)(wave + 4 * q) * 1024u);
            }
        };
        // prologue: in flight afterwards, oldest first:
        // data(s_lo) | ids(s_lo + 3) data(s_lo + 1) | ids(s_lo + 4) data(s_lo + 2)
        issue_ids(s_lo);
        issue_ids(s_lo + 1);
        issue_ids(s_lo + 2);
        wait_vm<0>();
        issue_data(s_lo);
        issue_ids(s_lo + 3);
        issue_data(s_lo + 1);
        issue_ids(s_lo + 4);
        issue_data(s_lo + 2);
        for (int s = s_lo; s < s_hi; ++s) {
            // all but the last two stages' loads and the row numbers between them:
            // stage s and the row numbers of stage s + 3 are in LDS
            wait_vm<2 * WG_PER_WAVE + 1>();
            __syncthreads();                 // ... those of every wavefront; and everybody is done with stage s - 1
            issue_ids(s + 5);
            issue_data(s + 3);               // into the buffer stage s - 1 was multiplied from (stages past the end fetch valid rows that nobody reads)
            unsigned char* buf = tiles + (s % WG_NB) * WG_STAGE;
            if ((s + 1) * WG_KS > n_rows) {  // rows past the end hold copies of the last row: they count as zeros through G
                uint32_t* g = reinterpret_cast<uint32_t*>(buf + G_AT * 1024);
                const int first = n_rows - s * WG_KS;
                for (int i = first * (WG_GP / 4) + tid; i < WG_KS * (WG_GP / 4); i += 256) g[i] = 0u;
                __syncthreads();
            }
            const uint16_t* Hs = reinterpret_cast<const uint16_t*>(buf);
            const uint16_t* Gs = reinterpret_cast<const uint16_t*>(buf + G_AT * 1024);
            // lane group g = lane / 16 reads rows 4g .. 4g+3 (first read) and 16 + 4g .. (second) of the 32 rows:
            // the order of the 32 products within an MFMA step is free as long as both operands agree
            const int row_in = (lane >> 4) * 4 + ((lane & 15) >> 2), col_in = (lane & 3) * 4;
            bf16x8 fh[4], fg[WG_MB];
            const uint16_t* hr = Hs + row_in * (WG_HP / 2) + wave * 64 + col_in;
            const uint16_t* gr = Gs + row_in * (WG_GP / 2) + col_in;
#pragma unroll
            for (int bn = 0; bn < 4; ++bn) fh[bn] = join8(read_tr(hr + bn * 16), read_tr(hr + 16 * (WG_HP / 2) + bn * 16));
#pragma unroll
            for (int bm = 0; bm < WG_MB; ++bm) fg[bm] = join8(read_tr(gr + bm * 16), read_tr(gr + 16 * (WG_GP / 2) + bm * 16));
#pragma unroll
            for (int bn = 0; bn < 4; ++bn)
#pragma unroll
                for (int bm = 0; bm < WG_MB; ++bm)
                    acc[bn][bm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fh[bn], fg[bm], acc[bn][bm], 0, 0, 0);
        }
        wait_vm<0>();                        // the loads issued past the end land before the workgroup gives up its LDS
    }
    // a lane holds, per block, 4 consecutive feature coordinates n of one embedding coordinate m
#pragma unroll
    for (int bm = 0; bm < WG_MB; ++bm) {
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

hipError_t launch_sem_fuse(const SemFuseArgs& a, hipStream_t s) {
    if (a.n_rows <= 0) return hipSuccess;
    if (a.ds <= 0 || a.ds % KS || a.d % 4) return hipErrorInvalidValue;
    const int64_t u_tiles = (a.n_rows + SF_BU - 1) / SF_BU;
    const int64_t n_tiles = (a.d + SF_N - 1) / SF_N;
    const int64_t blocks = ((u_tiles + 7) / 8) * 8 * n_tiles;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(sem_fuse_kernel, dim3((unsigned)blocks), dim3(SF_NW * 64), 0, s, a);
    return hipGetLastError();
}

int sem_wgrad_splits(int64_t n_rows_bound, int d, int ds) {
    const int tiles = ((d + WG_M - 1) / WG_M) * ((ds + WG_SEM - 1) / WG_SEM);
    const int64_t stages = (n_rows_bound + WG_KS - 1) / WG_KS;
    // one resident set of workgroups, no second round: the four stages in LDS leave room for one
    // workgroup per compute unit; the splits of a launch are dealt to the 8 dies in turn, 32
    // compute units each
    const int cap = std::max(1, 32 / tiles) * 8;
    return (int)std::max<int64_t>(1, std::min<int64_t>(stages / 4, cap));
}

hipError_t launch_sem_wgrad(const SemWgradArgs& a, float* out, hipStream_t s) {
    if (a.ds <= 0 || a.ds % KS || a.d % 8 || a.n_splits < 1) return hipErrorInvalidValue;
    const int tiles = ((a.d + WG_M - 1) / WG_M) * ((a.ds + WG_SEM - 1) / WG_SEM);
    const int blocks = ((a.n_splits + 7) / 8) * 8 * tiles;
    hipLaunchKernelGGL(sem_wgrad_kernel, dim3(blocks), dim3(256), 0, s, a);
    const int64_t n4 = (int64_t)a.d * a.ds / 4;
    hipLaunchKernelGGL(sem_wgrad_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s,
                       (const float*)a.partial, a.n_splits, n4, out);
    return hipGetLastError();
}

}  // namespace ngdb
