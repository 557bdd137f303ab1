// Device-side gradient index (Sec. 4.2 "Efficient Tensor Indexing"): the
// contributions to an embedding table -- anchors, positives, negatives -- are
// grouped by row id with a stable least-significant-digit radix sort, so that
// the scatter-add of the backward pass becomes one atomic-free segmented sum per
// touched row, in a fixed order.  Every pass is three kernels (per-tile digit
// histogram, exclusive scan of the digit-major histogram, stable scatter); no
// kernel contains a data-dependent wait.
#include "common.h"

namespace ngdb {
namespace {

constexpr int RADIX_BITS = 8;
constexpr int RADIX = 1 << RADIX_BITS;
constexpr int SORT_THREADS = 256;
constexpr int SORT_ITEMS = 4;                        // keys per thread
constexpr int SORT_TILE = SORT_THREADS * SORT_ITEMS; // keys per workgroup
constexpr int SCAN_THREADS = 256;
constexpr int SCAN_ITEMS = 8;
constexpr int SCAN_TILE = SCAN_THREADS * SCAN_ITEMS;

// keys[i] = i < n_head ? head[i] : tail[i - n_head]; vals[i] = i
__global__ __launch_bounds__(256) void assemble_kernel(const int32_t* __restrict__ head, int n_head,
                                                       const int32_t* __restrict__ tail, int64_t n,
                                                       int32_t* __restrict__ keys, int32_t* __restrict__ vals) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        keys[i] = i < n_head ? head[i] : tail[i - n_head];
        vals[i] = (int32_t)i;
    }
}

// hist[digit * n_tiles + tile] = number of keys of the tile with that digit
__global__ __launch_bounds__(SORT_THREADS) void hist_kernel(const int32_t* __restrict__ keys, int64_t n, int shift,
                                                            int n_tiles, int32_t* __restrict__ hist) {
    __shared__ int32_t h[RADIX];
    h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * SORT_TILE;
    for (int r = 0; r < SORT_ITEMS; ++r) {
        const int64_t i = base + (int64_t)r * SORT_THREADS + threadIdx.x;
        if (i < n) atomicAdd(&h[(keys[i] >> shift) & (RADIX - 1)], 1);
    }
    __syncthreads();
    hist[(size_t)threadIdx.x * n_tiles + blockIdx.x] = h[threadIdx.x];
}

// ---- exclusive scan of int32 in three steps: tile sums, scan of the sums, tile scan
__device__ __forceinline__ int32_t block_exclusive_scan(int32_t v, int32_t* total) {
    __shared__ int32_t wsum[SCAN_THREADS / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int32_t inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int32_t t = __shfl_up(inc, off, 64);
        if (lane >= off) inc += t;
    }
    __syncthreads();                      // wsum may still be read from a previous call
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    int32_t woff = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < SCAN_THREADS / 64; ++w) {
        if (w < wave) woff += wsum[w];
        tot += wsum[w];
    }
    *total = tot;
    return woff + inc - v;
}

template <bool HEADS>
__device__ __forceinline__ int32_t scan_input(const int32_t* __restrict__ in, int64_t i) {
    if (!HEADS) return in[i];
    return (i == 0 || in[i] != in[i - 1]) ? 1 : 0;   // segment head flag over sorted keys
}

template <bool HEADS>
__global__ __launch_bounds__(SCAN_THREADS) void scan_sums_kernel(const int32_t* __restrict__ in, int64_t n,
                                                                 int32_t* __restrict__ sums) {
    const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    int32_t s = 0;
    for (int k = 0; k < SCAN_ITEMS; ++k)
        if (base + k < n) s += scan_input<HEADS>(in, base + k);
    int32_t tot;
    block_exclusive_scan(s, &tot);
    if (threadIdx.x == 0) sums[blockIdx.x] = tot;
}

// one workgroup: exclusive scan of sums[0..m) in place, grand total to *total
__global__ __launch_bounds__(SCAN_THREADS) void scan_top_kernel(int32_t* __restrict__ sums, int m,
                                                                int32_t* __restrict__ total) {
    int32_t carry = 0;
    for (int base = 0; base < m; base += SCAN_THREADS) {
        const int i = base + threadIdx.x;
        const int32_t v = i < m ? sums[i] : 0;
        int32_t tot;
        const int32_t ex = block_exclusive_scan(v, &tot);
        if (i < m) sums[i] = carry + ex;
        carry += tot;
    }
    if (threadIdx.x == 0 && total) *total = carry;
}

// HEADS=false: out[i] = exclusive prefix.  HEADS=true: for every head position i
// with rank u: uniq[u] = keys[i], seg_off[u] = i; the last workgroup closes seg_off.
template <bool HEADS>
__global__ __launch_bounds__(SCAN_THREADS) void scan_apply_kernel(const int32_t* __restrict__ in, int64_t n,
                                                                  const int32_t* __restrict__ sums,
                                                                  int32_t* __restrict__ out,
                                                                  int32_t* __restrict__ seg_off,
                                                                  const int32_t* __restrict__ total) {
    const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    int32_t v[SCAN_ITEMS];
    int32_t s = 0;
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        v[k] = base + k < n ? scan_input<HEADS>(in, base + k) : 0;
        s += v[k];
    }
    int32_t tot;
    int32_t run = sums[blockIdx.x] + block_exclusive_scan(s, &tot);
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        if (base + k < n) {
            if (!HEADS) {
                out[base + k] = run;
            } else if (v[k]) {
                out[run] = in[base + k];
                seg_off[run] = (int32_t)(base + k);
            }
        }
        run += v[k];
    }
    if (HEADS && blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) seg_off[*total] = (int32_t)n;
}

// Stable scatter of one radix pass.  The tile is walked in rounds of 256
// consecutive keys (thread t takes key round*256 + t), so the order inside the
// tile is (round, wavefront, lane); the rank of a key among equal digits is
// running count of earlier rounds + counts of lower wavefronts + lower lanes.
__global__ __launch_bounds__(SORT_THREADS) void scatter_kernel(const int32_t* __restrict__ keys_in,
                                                               const int32_t* __restrict__ vals_in, int64_t n,
                                                               int shift, int n_tiles,
                                                               const int32_t* __restrict__ offs,
                                                               int32_t* __restrict__ keys_out,
                                                               int32_t* __restrict__ vals_out) {
    __shared__ int32_t running[RADIX];                    // global position of the next key per digit
    __shared__ int32_t wcnt[SORT_THREADS / 64][RADIX];    // per wavefront counts of the current round
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    running[threadIdx.x] = offs[(size_t)threadIdx.x * n_tiles + blockIdx.x];
    for (int w = 0; w < SORT_THREADS / 64; ++w) wcnt[w][threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * SORT_TILE;
    for (int r = 0; r < SORT_ITEMS; ++r) {
        const int64_t i = base + (int64_t)r * SORT_THREADS + threadIdx.x;
        const bool valid = i < n;
        int32_t key = 0, val = 0;
        if (valid) {
            key = keys_in[i];
            val = vals_in[i];
        }
        const int digit = (key >> shift) & (RADIX - 1);
        // lanes of this wavefront that hold a valid key with the same digit
        unsigned long long peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < RADIX_BITS; ++b) {
            const unsigned long long bal = __ballot((digit >> b) & 1);
            peers &= ((digit >> b) & 1) ? bal : ~bal;
        }
        const unsigned long long lower = peers & ((1ull << lane) - 1ull);
        const int rank_in_wave = __popcll(lower);
        if (valid && lower == 0ull) wcnt[wave][digit] = __popcll(peers);   // one writer per digit
        __syncthreads();
        int32_t pos = 0;
        if (valid) {
            pos = running[digit] + rank_in_wave;
            for (int w = 0; w < wave; ++w) pos += wcnt[w][digit];
        }
        __syncthreads();
        {   // thread t owns digit t: advance the running position, clear the round's counts
            int32_t add = 0;
            for (int w = 0; w < SORT_THREADS / 64; ++w) {
                add += wcnt[w][threadIdx.x];
                wcnt[w][threadIdx.x] = 0;
            }
            running[threadIdx.x] += add;
        }
        if (valid) {
            keys_out[pos] = key;
            vals_out[pos] = val;
        }
        __syncthreads();
    }
}

inline int tiles_of(int64_t n, int tile) { return (int)((n + tile - 1) / tile); }

// exclusive scan of in[0..n) into out (may alias), scratch `sums` of ceil(n/SCAN_TILE) ints
hipError_t scan_exclusive(const int32_t* in, int32_t* out, int64_t n, int32_t* sums, hipStream_t s) {
    const int nt = tiles_of(n, SCAN_TILE);
    hipLaunchKernelGGL((scan_sums_kernel<false>), dim3(nt), dim3(SCAN_THREADS), 0, s, in, n, sums);
    hipLaunchKernelGGL(scan_top_kernel, dim3(1), dim3(SCAN_THREADS), 0, s, sums, nt, (int32_t*)nullptr);
    hipLaunchKernelGGL((scan_apply_kernel<false>), dim3(nt), dim3(SCAN_THREADS), 0, s, in, n,
                       (const int32_t*)sums, out, (int32_t*)nullptr, (const int32_t*)nullptr);
    return hipGetLastError();
}

}  // namespace

size_t index_hist_elems(int64_t n_keys) { return (size_t)RADIX * tiles_of(std::max<int64_t>(n_keys, 1), SORT_TILE); }

size_t index_scan_tmp_elems(int64_t n_keys) {
    const int64_t a = tiles_of((int64_t)index_hist_elems(n_keys), SCAN_TILE);
    const int64_t b = tiles_of(std::max<int64_t>(n_keys, 1), SCAN_TILE);
    return (size_t)std::max(a, b) + 1;
}

hipError_t build_segment_index(const int32_t* head, int n_head, const int32_t* tail, int64_t n_tail,
                               int32_t key_bound, const IndexBuffers& buf, int32_t** src_out, hipStream_t s) {
    const int64_t n = (int64_t)n_head + n_tail;
    if (n <= 0) {
        // empty index: n_uniq = 0, seg_off[0] = 0
        hipLaunchKernelGGL(scan_top_kernel, dim3(1), dim3(SCAN_THREADS), 0, s, buf.seg_off, 0, buf.n_uniq);
        hipLaunchKernelGGL((scan_apply_kernel<true>), dim3(1), dim3(SCAN_THREADS), 0, s,
                           (const int32_t*)buf.keys_a, (int64_t)0, (const int32_t*)buf.scan_tmp, buf.uniq,
                           buf.seg_off, (const int32_t*)buf.n_uniq);
        *src_out = buf.vals_a;
        return hipGetLastError();
    }
    const unsigned gblocks = (unsigned)std::min<int64_t>((n + 255) / 256, 2048);
    hipLaunchKernelGGL(assemble_kernel, dim3(gblocks), dim3(256), 0, s, head, n_head, tail, n, buf.keys_a, buf.vals_a);

    int bits = 1;
    while (bits < 31 && (1ll << bits) < (long long)key_bound) ++bits;
    const int n_tiles = tiles_of(n, SORT_TILE);
    int32_t *kin = buf.keys_a, *kout = buf.keys_b, *vin = buf.vals_a, *vout = buf.vals_b;
    for (int shift = 0; shift < bits; shift += RADIX_BITS) {
        hipLaunchKernelGGL(hist_kernel, dim3(n_tiles), dim3(SORT_THREADS), 0, s, (const int32_t*)kin, n, shift,
                           n_tiles, buf.hist);
        hipError_t e = scan_exclusive(buf.hist, buf.hist, (int64_t)RADIX * n_tiles, buf.scan_tmp, s);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(scatter_kernel, dim3(n_tiles), dim3(SORT_THREADS), 0, s, (const int32_t*)kin,
                           (const int32_t*)vin, n, shift, n_tiles, (const int32_t*)buf.hist, kout, vout);
        std::swap(kin, kout);
        std::swap(vin, vout);
    }
    // segment heads over the sorted keys
    const int nt = tiles_of(n, SCAN_TILE);
    hipLaunchKernelGGL((scan_sums_kernel<true>), dim3(nt), dim3(SCAN_THREADS), 0, s, (const int32_t*)kin, n,
                       buf.scan_tmp);
    hipLaunchKernelGGL(scan_top_kernel, dim3(1), dim3(SCAN_THREADS), 0, s, buf.scan_tmp, nt, buf.n_uniq);
    hipLaunchKernelGGL((scan_apply_kernel<true>), dim3(nt), dim3(SCAN_THREADS), 0, s, (const int32_t*)kin, n,
                       (const int32_t*)buf.scan_tmp, buf.uniq, buf.seg_off, (const int32_t*)buf.n_uniq);
    *src_out = vin;
    return hipGetLastError();
}

}  // namespace ngdb
