// Stable LSD radix sort of (key, value) pairs, <= 8 bits per pass.
//
// Per pass, three launches over 2048-key tiles:
//   sort_count    per-tile digit histogram (one LDS add per distinct digit per wave,
//                 found by ballot matching), stored digit-major
//   sort_scan     one block per digit: exclusive scan of the digit's per-tile counts,
//                 and the digit's total
//   sort_scatter  each wave ranks its 512 consecutive keys against a wave-private
//                 running histogram in LDS (ballot matching keeps equal digits in
//                 order), adds tile and digit bases, writes the pairs
// Stability comes from wave -> tile -> digit prefix order; there are no spin-waits.
#include "radix_sort.h"

namespace fs {

constexpr int kSortWaveSpan = kWave * kSortItems;
constexpr int64_t kSortMaxGrid = 8192;       // 32 blocks per CU: enough to fill the chip, few enough to be cheap when idle

__device__ __forceinline__ int64_t sort_count_of(const int64_t* m_dev, int64_t m_max)
{
    if (m_dev == nullptr) return m_max;
    const int64_t m = *m_dev;
    return m < 0 ? 0 : (m < m_max ? m : m_max);
}

__global__ __launch_bounds__(kBlock) void sort_count_kernel(
    const uint32_t* __restrict__ keys, int64_t m_max, const int64_t* __restrict__ m_dev,
    int shift, int nbits, uint32_t* __restrict__ tile_hist /* [bins][tiles] */, int64_t tiles)
{
    __shared__ uint32_t hist[1 << kSortMaxDigitBits];
    const int64_t m = sort_count_of(m_dev, m_max);
    const int64_t used = (m + kSortTile - 1) / kSortTile;      // tiles that hold keys (m may live on the device)
    const int bins = 1 << nbits;
    const uint32_t mask = (uint32_t)bins - 1u;
    for (int64_t tile = blockIdx.x; tile < used; tile += gridDim.x) {
        const int64_t base = tile * kSortTile;
        for (int b = threadIdx.x; b < bins; b += kBlock) hist[b] = 0;
        __syncthreads();
#pragma unroll
        for (int it = 0; it < kSortItems; ++it) {
            const int64_t i = base + (int64_t)it * kBlock + threadIdx.x;
            const bool valid = i < m;
            const uint32_t digit = valid ? ((keys[i] >> shift) & mask) : 0u;
            const uint64_t same = match_bits(digit, nbits, valid);
            if (valid && popc_below(same) == 0) atomicAdd(&hist[digit], (uint32_t)__popcll(same));
        }
        __syncthreads();
        for (int b = threadIdx.x; b < bins; b += kBlock) tile_hist[(int64_t)b * tiles + tile] = hist[b];
        __syncthreads();
    }
}

__global__ __launch_bounds__(kBlock) void sort_scan_kernel(
    uint32_t* __restrict__ tile_hist, int64_t tiles, int64_t m_max, const int64_t* __restrict__ m_dev,
    uint32_t* __restrict__ totals)
{
    __shared__ uint32_t part[kBlock];
    const int64_t m = sort_count_of(m_dev, m_max);
    const int64_t used = (m + kSortTile - 1) / kSortTile;       // tiles that hold keys
    uint32_t* h = tile_hist + (int64_t)blockIdx.x * tiles;
    const int64_t per = (used + kBlock - 1) / kBlock;
    const int64_t lo = (int64_t)threadIdx.x * per < used ? (int64_t)threadIdx.x * per : used;
    const int64_t hi = lo + per < used ? lo + per : used;
    uint32_t sum = 0;
    for (int64_t k = lo; k < hi; ++k) sum += h[k];
    part[threadIdx.x] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int k = 0; k < kBlock; ++k) { const uint32_t v = part[k]; part[k] = run; run += v; }
        totals[blockIdx.x] = run;
    }
    __syncthreads();
    uint32_t run = part[threadIdx.x];
    for (int64_t k = lo; k < hi; ++k) { const uint32_t v = h[k]; h[k] = run; run += v; }
}

__global__ __launch_bounds__(kBlock) void sort_scatter_kernel(
    const uint32_t* __restrict__ keys, const uint32_t* __restrict__ vals,
    int64_t m_max, const int64_t* __restrict__ m_dev, int shift, int nbits,
    const uint32_t* __restrict__ tile_hist /* scanned */, int64_t tiles, const uint32_t* __restrict__ totals,
    uint32_t* __restrict__ keys_out, uint32_t* __restrict__ vals_out)
{
    __shared__ uint32_t digit_base[1 << kSortMaxDigitBits];
    __shared__ uint16_t wave_hist[kWavesPerBlock][1 << kSortMaxDigitBits];
    const int64_t m = sort_count_of(m_dev, m_max);
    const int64_t used = (m + kSortTile - 1) / kSortTile;
    const int bins = 1 << nbits;
    const uint32_t mask = (uint32_t)bins - 1u;
    const int w = wave_id();
    const int lane = lane_id();

    for (int64_t tile = blockIdx.x; tile < used; tile += gridDim.x) {
        const int64_t base = tile * kSortTile;
        // exclusive scan of the digit totals by the first wave (bins <= 256 = 4 per lane)
        if (w == 0) {
            uint32_t v[4];
            uint32_t sum = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int b = lane * 4 + q;
                v[q] = b < bins ? totals[b] : 0u;
                sum += v[q];
            }
            uint32_t incl = sum;
            for (int off = 1; off < kWave; off <<= 1) {
                const uint32_t up = __shfl_up(incl, off);
                if (lane >= off) incl += up;
            }
            uint32_t run = incl - sum;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int b = lane * 4 + q;
                if (b < bins) digit_base[b] = run + tile_hist[(int64_t)b * tiles + tile];
                run += v[q];
            }
        }
        for (int b = lane; b < bins; b += kWave) wave_hist[w][b] = 0;
        __syncthreads();

        uint32_t key[kSortItems];
        uint32_t val[kSortItems];
        uint32_t rank[kSortItems];
#pragma unroll
        for (int it = 0; it < kSortItems; ++it) {
            const int64_t i = base + (int64_t)w * kSortWaveSpan + it * kWave + lane;
            const bool valid = i < m;
            key[it] = valid ? keys[i] : 0u;
            val[it] = valid ? vals[i] : 0u;
        }
#pragma unroll
        for (int it = 0; it < kSortItems; ++it) {
            const int64_t i = base + (int64_t)w * kSortWaveSpan + it * kWave + lane;
            const bool valid = i < m;
            const uint32_t digit = (key[it] >> shift) & mask;
            const uint64_t same = match_bits(digit, nbits, valid);
            const uint32_t before = popc_below(same);
            uint32_t seen = 0;
            if (valid) seen = wave_hist[w][digit];
            __builtin_amdgcn_wave_barrier();
            rank[it] = seen + before;
            if (valid && before == 0) wave_hist[w][digit] = (uint16_t)(seen + __popcll(same));
            __builtin_amdgcn_wave_barrier();
        }
        __syncthreads();
        for (int b = threadIdx.x; b < bins; b += kBlock) {
            uint32_t run = 0;
#pragma unroll
            for (int k = 0; k < kWavesPerBlock; ++k) {
                const uint32_t v = wave_hist[k][b];
                wave_hist[k][b] = (uint16_t)run;
                run += v;
            }
        }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < kSortItems; ++it) {
            const int64_t i = base + (int64_t)w * kSortWaveSpan + it * kWave + lane;
            if (i < m) {
                const uint32_t digit = (key[it] >> shift) & mask;
                const uint32_t j = digit_base[digit] + wave_hist[w][digit] + rank[it];
                keys_out[j] = key[it];
                vals_out[j] = val[it];
            }
        }
        __syncthreads();
    }
}

static int64_t sort_tiles(int64_t m_max) { return (m_max + kSortTile - 1) / kSortTile; }

size_t radix_sort_scratch_bytes(int64_t m_max)
{
    Carver c(nullptr);
    c.take<uint32_t>((size_t)1 << kSortMaxDigitBits);
    c.take<uint32_t>(((size_t)1 << kSortMaxDigitBits) * (size_t)sort_tiles(m_max));
    return c.used;
}

fs_status radix_sort_pairs(uint32_t* keys_a, uint32_t* vals_a, uint32_t* keys_b, uint32_t* vals_b,
                           int64_t m_max, const int64_t* m_dev, int key_bits, void* scratch,
                           hipStream_t stream, uint32_t** keys_out, uint32_t** vals_out)
{
    *keys_out = keys_a;
    *vals_out = vals_a;
    if (m_max <= 0) return FS_OK;
    if (key_bits < 1) key_bits = 1;
    if (key_bits > 32) key_bits = 32;
    const int64_t tiles = sort_tiles(m_max);
    if (tiles > 0x7FFFFFFF) return FS_ERR_SIZE;
    Carver c(scratch);
    uint32_t* totals = c.take<uint32_t>((size_t)1 << kSortMaxDigitBits);
    uint32_t* tile_hist = c.take<uint32_t>(((size_t)1 << kSortMaxDigitBits) * (size_t)tiles);

    // blocks walk the tiles with a grid stride: when the pair count lives on the device the grid
    // is sized for m_max, and empty blocks would otherwise dominate a small sort
    const unsigned grid = (unsigned)(tiles < kSortMaxGrid ? tiles : kSortMaxGrid);
    const int passes = (key_bits + kSortMaxDigitBits - 1) / kSortMaxDigitBits;
    int shift = 0;
    uint32_t* src_k = keys_a; uint32_t* src_v = vals_a;
    uint32_t* dst_k = keys_b; uint32_t* dst_v = vals_b;
    for (int p = 0; p < passes; ++p) {
        // spread the bits evenly over the passes: 27 bits -> 7, 7, 7, 6
        const int left = key_bits - shift;
        const int nbits = (left + (passes - p) - 1) / (passes - p);
        FS_LAUNCH("sort_count", sort_count_kernel, dim3(grid), dim3(kBlock), stream,
                  src_k, m_max, m_dev, shift, nbits, tile_hist, tiles);
        FS_LAUNCH("sort_scan", sort_scan_kernel, dim3(1u << nbits), dim3(kBlock), stream,
                  tile_hist, tiles, m_max, m_dev, totals);
        FS_LAUNCH("sort_scatter", sort_scatter_kernel, dim3(grid), dim3(kBlock), stream,
                  src_k, src_v, m_max, m_dev, shift, nbits, tile_hist, tiles, totals, dst_k, dst_v);
        shift += nbits;
        uint32_t* t;
        t = src_k; src_k = dst_k; dst_k = t;
        t = src_v; src_v = dst_v; dst_v = t;
    }
    *keys_out = src_k;
    *vals_out = src_v;
    return FS_OK;
}

}  // namespace fs
