// Stable LSD radix sort of (key, value) pairs, up to 10 bits per pass (27-bit row ids: 3 passes).
//
// Per pass, four launches over 4096-pair tiles (blocks walk the tiles with a grid stride):
//   sort_count    per-tile digit histogram (one LDS add per distinct digit per wave, found by
//                 ballot matching), stored tile-major
//   sort_scan     exclusive scan of every digit's per-tile counts over the tiles (two levels,
//                 coalesced across digits), and the digits' totals; for small sorts the block that
//                 finishes its chunk of tiles last (a counter, no waiting) runs the second level,
//                 for large ones the second level is a launch of its own (sort_scan_chunks)
//   sort_scatter  each wave ranks its 1024 consecutive pairs against a wave-private running
//                 histogram in LDS (ballot matching keeps equal digits in order); the tile is put
//                 in digit order in LDS, then written out so that consecutive lanes write
//                 consecutive addresses of one digit's run
// Stability comes from wave -> tile -> digit prefix order; no block ever waits for another.
// The first pass can read (int64 row, int32 position) directly, validating them on the way.
#include "radix_sort.h"

namespace fs {

constexpr int kSortWaveSpan = kWave * kSortItems;
constexpr int kSortMaxBins = 1 << kSortMaxDigitBits;
constexpr int kSortStripe = 16;              // tiles per XCD stripe in the scatter
constexpr int64_t kSortMaxGrid = 8192;       // 32 blocks per CU: fills the chip, cheap when most are idle

__device__ __forceinline__ int64_t sort_count_of(const int64_t* m_dev, int64_t m_max)
{
    if (m_dev == nullptr) return m_max;
    const int64_t m = *m_dev;
    return m < 0 ? 0 : (m < m_max ? m : m_max);
}

struct PairReader {                           // pairs already in (keys, vals)
    const uint32_t* keys;
    const uint32_t* vals;
    __device__ __forceinline__ uint32_t key(int64_t i) const { return keys[i]; }
    __device__ __forceinline__ void pair(int64_t i, uint32_t* k, uint32_t* v, int32_t*) const
    {
        *k = keys[i];
        *v = vals[i];
    }
};

struct RowPosReader {                         // pairs are (rows[i], pos[i]), validated
    const int64_t* rows;
    const int32_t* pos;
    int64_t R;
    int64_t n;
    // one unsigned compare each also catches the negative values (R < 2^32, n < 2^31)
    __device__ __forceinline__ uint32_t key(int64_t i) const
    {
        const uint64_t r = (uint64_t)load_stream(rows + i);
        return r >= (uint64_t)R ? 0u : (uint32_t)r;
    }
    __device__ __forceinline__ void pair(int64_t i, uint32_t* k, uint32_t* v, int32_t* faults) const
    {
        uint64_t r = (uint64_t)load_stream(rows + i);
        uint32_t p = (uint32_t)load_stream(pos + i);
        if (r >= (uint64_t)R) { r = 0; *faults |= FS_DEV_BAD_ID; }
        if (p >= (uint32_t)n) { p = 0; *faults |= FS_DEV_BAD_ID; }
        *k = (uint32_t)r;
        *v = p;
    }
};

// One LDS add per distinct digit per wave: the lanes that hold the same digit are found with one
// ballot per bit (plain per-lane LDS adds serialise on the popular rows' digits and were slower).
template <int NBITS>
__device__ __forceinline__ void count_digit(uint32_t* hist, uint32_t digit, bool valid)
{
    const uint64_t same = match_bits_n<NBITS>(digit, valid);
    if (valid && popc_below(same) == 0) atomicAdd(&hist[digit], (uint32_t)__popcll(same));
}

template <typename Reader, int NBITS>
__global__ __launch_bounds__(kBlock) void sort_count_kernel(
    Reader in, int64_t m_max, const int64_t* __restrict__ m_dev,
    int shift, uint32_t* __restrict__ tile_hist /* [tiles][bins] */, uint32_t* __restrict__ scan_done)
{
    constexpr int bins = 1 << NBITS;
    __shared__ uint32_t hist[bins];
    if (blockIdx.x == 0 && threadIdx.x == 0) *scan_done = 0;    // the scan kernel that follows counts its finished blocks here
    const int64_t m = sort_count_of(m_dev, m_max);
    const int64_t used = (m + kSortTile - 1) / kSortTile;      // tiles that hold pairs (m may live on the device)
    constexpr uint32_t mask = (uint32_t)bins - 1u;
    for (int64_t tile = blockIdx.x; tile < used; tile += gridDim.x) {
        const int64_t base = tile * kSortTile;
        for (int b = threadIdx.x; b < bins; b += kBlock) hist[b] = 0;
        __syncthreads();
        if (base + kSortTile <= m) {                            // whole tile: unpredicated loads, all in flight
            uint32_t key[kSortItems];
#pragma unroll
            for (int it = 0; it < kSortItems; ++it) key[it] = in.key(base + (int64_t)it * kBlock + threadIdx.x);
#pragma unroll
            for (int it = 0; it < kSortItems; ++it) count_digit<NBITS>(hist, (key[it] >> shift) & mask, true);
        } else {
            for (int it = 0; it < kSortItems; ++it) {
                const int64_t i = base + (int64_t)it * kBlock + threadIdx.x;
                const bool valid = i < m;
                count_digit<NBITS>(hist, valid ? ((in.key(i) >> shift) & mask) : 0u, valid);
            }
        }
        __syncthreads();
        for (int b = threadIdx.x; b < bins; b += kBlock) tile_hist[tile * bins + b] = hist[b];
        __syncthreads();
    }
}

// Column-wise exclusive scan of tile_hist[tile][digit] over the tiles, in two levels so that every
// access is coalesced across digits.  Level 1: a block takes a chunk of 64 tiles; thread b walks
// the chunk's tiles for digit b, leaves the running prefix in place and the chunk's sum in
// chunk_sums[chunk][b].  Level 2 (one block): thread b walks the chunks for digit b: chunk_sums ->
// exclusive prefix, totals[b].
constexpr int kSortChunkTiles = 64;
constexpr int kSortFusedScanChunks = 16;     // up to this many chunks (4 M pairs) the scan's second level runs inside its first launch
constexpr int kSortFusedScanChunksDev = 1024;
constexpr int kScanAhead = 8;                // loads a scan thread keeps in flight (16 and 32 are slower)

__global__ __launch_bounds__(1024) void sort_scan_kernel(
    uint32_t* __restrict__ tile_hist, int bins, int64_t m_max, const int64_t* __restrict__ m_dev,
    uint32_t* __restrict__ chunk_sums, uint32_t* __restrict__ totals, uint32_t* __restrict__ scan_done, int fused)
{
    __shared__ bool is_last;
    const int64_t m = sort_count_of(m_dev, m_max);
    const int64_t used = (m + kSortTile - 1) / kSortTile;
    const int64_t chunks = (used + kSortChunkTiles - 1) / kSortChunkTiles;
    const int64_t t0 = (int64_t)blockIdx.x * kSortChunkTiles;
    if (t0 >= used) return;                                      // block-uniform: this block has no tiles
    const int64_t t1 = t0 + kSortChunkTiles < used ? t0 + kSortChunkTiles : used;
    for (int b = threadIdx.x; b < bins; b += blockDim.x) {       // launched with one thread per digit (up to 1024)
        uint32_t run = 0;
        int64_t t = t0;
        for (; t + kScanAhead <= t1; t += kScanAhead) {          // kScanAhead loads in flight: a thread's time is its rounds of loads
            uint32_t v[kScanAhead];
#pragma unroll
            for (int q = 0; q < kScanAhead; ++q) v[q] = tile_hist[(t + q) * bins + b];
#pragma unroll
            for (int q = 0; q < kScanAhead; ++q) { tile_hist[(t + q) * bins + b] = run; run += v[q]; }
        }
        for (; t < t1; ++t) { const uint32_t v = tile_hist[t * bins + b]; tile_hist[t * bins + b] = run; run += v; }
        chunk_sums[(int64_t)blockIdx.x * bins + b] = run;
    }
    if (!fused) return;                                          // block-uniform: level 2 is a launch of its own
    // Level 2 needs every block's chunk sums.  Each block publishes its own (fence), then takes a ticket;
    // the block that draws the last ticket sees all of them (fence) and runs the second level.  Nobody waits.
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) is_last = atomicAdd(scan_done, 1u) == (uint32_t)(chunks - 1);
    __syncthreads();
    if (!is_last) return;
    __threadfence();
    for (int b = threadIdx.x; b < bins; b += blockDim.x) {       // thread b walks the chunks for digit b
        uint32_t run = 0;
        int64_t c = 0;
        for (; c + kScanAhead <= chunks; c += kScanAhead) {
            uint32_t v[kScanAhead];
#pragma unroll
            for (int q = 0; q < kScanAhead; ++q) v[q] = chunk_sums[(c + q) * bins + b];
#pragma unroll
            for (int q = 0; q < kScanAhead; ++q) { chunk_sums[(c + q) * bins + b] = run; run += v[q]; }
        }
        for (; c < chunks; ++c) { const uint32_t v = chunk_sums[c * bins + b]; chunk_sums[c * bins + b] = run; run += v; }
        totals[b] = run;
    }
}

// Level 2 as a launch of its own, for sorts with many chunks: there the one workgroup that would run it
// inside sort_scan_kernel reads every other workgroup's sums from memory, alone on the chip, and takes
// longer than a launch costs (72 M pairs, 275 chunks: 230 µs against 11 µs).
__global__ __launch_bounds__(kBlock) void sort_scan_chunks_kernel(
    uint32_t* __restrict__ chunk_sums, int bins, int64_t m_max, const int64_t* __restrict__ m_dev,
    uint32_t* __restrict__ totals)
{
    const int64_t m = sort_count_of(m_dev, m_max);
    const int64_t used = (m + kSortTile - 1) / kSortTile;
    const int64_t chunks = (used + kSortChunkTiles - 1) / kSortChunkTiles;
    const int b = blockIdx.x * kBlock + threadIdx.x;
    if (b >= bins) return;
    uint32_t run = 0;
    int64_t c = 0;
    for (; c + kScanAhead <= chunks; c += kScanAhead) {
        uint32_t v[kScanAhead];
#pragma unroll
        for (int q = 0; q < kScanAhead; ++q) v[q] = chunk_sums[(c + q) * bins + b];
#pragma unroll
        for (int q = 0; q < kScanAhead; ++q) { chunk_sums[(c + q) * bins + b] = run; run += v[q]; }
    }
    for (; c < chunks; ++c) { const uint32_t v = chunk_sums[c * bins + b]; chunk_sums[c * bins + b] = run; run += v; }
    totals[b] = run;
}

template <typename Reader, int NBITS>
__global__ __launch_bounds__(kBlock) void sort_scatter_kernel(
    Reader in, int64_t m_max, const int64_t* __restrict__ m_dev, int shift,
    const uint32_t* __restrict__ tile_hist /* scanned */, const uint32_t* __restrict__ chunk_sums /* scanned */,
    const uint32_t* __restrict__ totals, uint32_t* __restrict__ keys_out, uint32_t* __restrict__ vals_out, int32_t* status)
{
    constexpr int bins = 1 << NBITS;
    __shared__ uint32_t out_base[bins];                         // global index of the tile's first pair of a digit,
                                                                // minus the digit's first index inside the tile
    __shared__ uint16_t wave_hist[kWavesPerBlock][bins];
    __shared__ uint32_t s_key[kSortTile];
    __shared__ uint32_t s_val[kSortTile];
    __shared__ uint32_t wave_sums[16];
    const int64_t m = sort_count_of(m_dev, m_max);
    const int64_t used = (m + kSortTile - 1) / kSortTile;
    constexpr uint32_t mask = (uint32_t)bins - 1u;
    const int w = wave_id();
    const int lane = lane_id();
    constexpr int kBinsPerThread = (bins + kBlock - 1) / kBlock;
    int32_t faults = 0;

    // Tiles in stripes per XCD (the grid is a multiple of 8, so a block stays on its XCD over the
    // grid stride): consecutive tiles write neighbouring runs of every digit's region, a few tens of
    // bytes each, and one XCD's L2 then merges what four XCDs would write into one 128-byte line
    // piece by piece (scatter 0.343 -> 0.327 ms per step on 15.7 M pairs).
    const int64_t padded = xcd_striped_grid_dev(used, kSortStripe);
    for (int64_t v = blockIdx.x; v < padded; v += gridDim.x) {
        const int64_t tile = xcd_striped_tile((unsigned)v, kSortStripe);
        if (tile >= used) continue;                              // block-uniform
        const int64_t base = tile * kSortTile;
        const int64_t wbase = base + (int64_t)w * kSortWaveSpan;
        for (int b = lane; b < bins; b += kWave) wave_hist[w][b] = 0;

        uint32_t key[kSortItems];
        uint32_t val[kSortItems];
        uint32_t rank[kSortItems];
        const bool whole = base + kSortTile <= m;
        if (whole) {
#pragma unroll
            for (int it = 0; it < kSortItems; ++it) in.pair(wbase + it * kWave + lane, &key[it], &val[it], &faults);
        } else {
#pragma unroll
            for (int it = 0; it < kSortItems; ++it) {
                const int64_t i = wbase + it * kWave + lane;
                key[it] = 0u;
                val[it] = 0u;
                if (i < m) in.pair(i, &key[it], &val[it], &faults);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // the zeroing above, seen by the wave's other lanes
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int it = 0; it < kSortItems; ++it) {
            const bool valid = whole || wbase + it * kWave + lane < m;
            const uint32_t digit = (key[it] >> shift) & mask;
            const uint64_t same = match_bits_n<NBITS>(digit, valid);
            const uint32_t before = popc_below(same);
            uint32_t seen = 0;
            if (valid) seen = wave_hist[w][digit];
            __builtin_amdgcn_wave_barrier();
            rank[it] = seen + before;
            if (valid && before == 0) wave_hist[w][digit] = (uint16_t)(seen + __popcll(same));
            __builtin_amdgcn_wave_barrier();
        }
        __syncthreads();

        // per digit: waves' counts -> waves' offsets inside the digit; the tile's count of the digit
        uint32_t count[kBinsPerThread];
        uint32_t tot[kBinsPerThread];
        uint32_t sum = 0, tsum = 0;
#pragma unroll
        for (int q = 0; q < kBinsPerThread; ++q) {
            const int b = threadIdx.x * kBinsPerThread + q;
            uint32_t run = 0;
            if (b < bins) {
#pragma unroll
                for (int k = 0; k < kWavesPerBlock; ++k) {
                    const uint32_t v = wave_hist[k][b];
                    wave_hist[k][b] = (uint16_t)run;
                    run += v;
                }
            }
            count[q] = run;
            sum += run;
            tot[q] = b < bins ? totals[b] : 0u;
            tsum += tot[q];
        }
        // exclusive scans over the digits: inside the tile (sum) and over the whole input (totals)
        uint32_t unused;
        uint32_t in_tile = block_exclusive_scan(sum, wave_sums, &unused);
        uint32_t in_all = block_exclusive_scan(tsum, wave_sums, &unused);
#pragma unroll
        for (int q = 0; q < kBinsPerThread; ++q) {
            const int b = threadIdx.x * kBinsPerThread + q;
            if (b < bins) {
                out_base[b] = in_all + chunk_sums[(tile / kSortChunkTiles) * bins + b] + tile_hist[tile * bins + b] - in_tile;
#pragma unroll
                for (int k = 0; k < kWavesPerBlock; ++k) wave_hist[k][b] = (uint16_t)(wave_hist[k][b] + in_tile);
            }
            in_tile += count[q];
            in_all += tot[q];
        }
        __syncthreads();
        // the tile in digit order, in LDS
#pragma unroll
        for (int it = 0; it < kSortItems; ++it) {
            const bool valid = whole || wbase + it * kWave + lane < m;
            if (valid) {
                const uint32_t digit = (key[it] >> shift) & mask;
                const uint32_t at = (uint32_t)wave_hist[w][digit] + rank[it];
                s_key[at] = key[it];
                s_val[at] = val[it];
            }
        }
        __syncthreads();
        const int valid_in_tile = (int)(m - base < kSortTile ? m - base : kSortTile);
#pragma unroll
        for (int it = 0; it < kSortItems; ++it) {
            const int at = it * kBlock + threadIdx.x;
            if (at < valid_in_tile) {
                const uint32_t k = s_key[at];
                const uint32_t j = out_base[(k >> shift) & mask] + (uint32_t)at;
                keys_out[j] = k;
                vals_out[j] = s_val[at];
            }
        }
        __syncthreads();
    }
    if (ballot(faults != 0) != 0) {
        for (int off = 32; off > 0; off >>= 1) faults |= __shfl_down(faults, off);
        if (lane == 0) report(status, faults);
    }
}

static int64_t sort_tiles(int64_t m_max) { return (m_max + kSortTile - 1) / kSortTile; }

size_t radix_sort_scratch_bytes(int64_t m_max)
{
    Carver c(nullptr);
    c.take<uint32_t>((size_t)kSortMaxBins);
    c.take<uint32_t>(1);
    c.take<uint32_t>((size_t)kSortMaxBins * (size_t)sort_tiles(m_max));
    c.take<uint32_t>((size_t)kSortMaxBins * (size_t)((sort_tiles(m_max) + kSortChunkTiles - 1) / kSortChunkTiles));
    return c.used;
}

fs_status radix_sort_pairs(uint32_t* keys_a, uint32_t* vals_a, uint32_t* keys_b, uint32_t* vals_b,
                           int64_t m_max, const int64_t* m_dev, int key_bits, void* scratch,
                           hipStream_t stream, uint32_t** keys_out, uint32_t** vals_out, const SortSource& src)
{
    *keys_out = keys_a;
    *vals_out = vals_a;
    if (m_max <= 0) return FS_OK;
    if (key_bits < 1) key_bits = 1;
    if (key_bits > 32) key_bits = 32;
    const int64_t tiles = sort_tiles(m_max);
    if (tiles > 0x7FFFFFFF) return FS_ERR_SIZE;
    Carver c(scratch);
    uint32_t* totals = c.take<uint32_t>((size_t)kSortMaxBins);
    uint32_t* scan_done = c.take<uint32_t>(1);
    uint32_t* tile_hist = c.take<uint32_t>((size_t)kSortMaxBins * (size_t)tiles);
    const int64_t chunks = (tiles + kSortChunkTiles - 1) / kSortChunkTiles;
    uint32_t* chunk_sums = c.take<uint32_t>((size_t)kSortMaxBins * (size_t)chunks);

    // blocks walk the tiles with a grid stride: when the pair count lives on the device the grid
    // is sized for m_max, and idle blocks would otherwise dominate a small sort
    const int64_t padded_tiles = xcd_striped_grid(tiles, kSortStripe);       // a multiple of 8
    const unsigned grid = (unsigned)(padded_tiles < kSortMaxGrid ? padded_tiles : kSortMaxGrid);
    const int passes = radix_sort_passes(key_bits);
    // The second scan level runs inside the first level's launch for small sorts.  When the pair count lives on
    // the device (the plan's candidates: a few per cent of the rows the buffers are sized for), "small" cannot be
    // known here; the launch is then fused up to a size at which the lone workgroup costs at most a tenth of a pass.
    const bool fused_scan = chunks <= kSortFusedScanChunks || (m_dev != nullptr && chunks <= kSortFusedScanChunksDev);
    int shift = 0;
    const bool from_rows = src.rows != nullptr;
    // from_rows: source -> A -> B -> A ...; else A -> B -> A ...
    uint32_t* src_k = keys_a; uint32_t* src_v = vals_a;
    uint32_t* dst_k = from_rows ? keys_a : keys_b;
    uint32_t* dst_v = from_rows ? vals_a : vals_b;
    for (int p = 0; p < passes; ++p) {
        // spread the bits evenly over the passes: 27 bits -> 9, 9, 9; 32 bits -> 8, 8, 8, 8
        const int left = key_bits - shift;
        const int nbits = (left + (passes - p) - 1) / (passes - p);
        const unsigned scan_threads = (1u << nbits) < (unsigned)kWave ? (unsigned)kWave : (1u << nbits);   // <= 1024
        if (p == 0 && from_rows) {
            const RowPosReader in{src.rows, src.pos, src.R, src.n};
#define FS_COUNT_ROWS(NB)                                                                                     \
    FS_LAUNCH("sort_count", (sort_count_kernel<RowPosReader, NB>), dim3(grid), dim3(kBlock), stream, in, m_max,     \
              m_dev, shift, tile_hist, scan_done)
            FS_DISPATCH_BITS(nbits, FS_COUNT_ROWS)
#undef FS_COUNT_ROWS
            FS_LAUNCH("sort_scan", sort_scan_kernel, dim3((unsigned)chunks), dim3(scan_threads), stream,
                      tile_hist, 1 << nbits, m_max, m_dev, chunk_sums, totals, scan_done, fused_scan ? 1 : 0);
            if (!fused_scan)
                FS_LAUNCH("sort_scan_chunks", sort_scan_chunks_kernel, dim3(((1u << nbits) + kBlock - 1) / kBlock),
                          dim3(kBlock), stream, chunk_sums, 1 << nbits, m_max, m_dev, totals);
#define FS_SCATTER_ROWS(NB)                                                                                   \
    FS_LAUNCH("sort_scatter", (sort_scatter_kernel<RowPosReader, NB>), dim3(grid), dim3(kBlock), stream, in, m_max, \
              m_dev, shift, tile_hist, chunk_sums, totals, dst_k, dst_v, src.status)
            FS_DISPATCH_BITS(nbits, FS_SCATTER_ROWS)
#undef FS_SCATTER_ROWS
        } else {
            const PairReader in{src_k, src_v};
#define FS_COUNT_PAIRS(NB)                                                                                    \
    FS_LAUNCH("sort_count", (sort_count_kernel<PairReader, NB>), dim3(grid), dim3(kBlock), stream, in, m_max,       \
              m_dev, shift, tile_hist, scan_done)
            FS_DISPATCH_BITS(nbits, FS_COUNT_PAIRS)
#undef FS_COUNT_PAIRS
            FS_LAUNCH("sort_scan", sort_scan_kernel, dim3((unsigned)chunks), dim3(scan_threads), stream,
                      tile_hist, 1 << nbits, m_max, m_dev, chunk_sums, totals, scan_done, fused_scan ? 1 : 0);
            if (!fused_scan)
                FS_LAUNCH("sort_scan_chunks", sort_scan_chunks_kernel, dim3(((1u << nbits) + kBlock - 1) / kBlock),
                          dim3(kBlock), stream, chunk_sums, 1 << nbits, m_max, m_dev, totals);
#define FS_SCATTER_PAIRS(NB)                                                                                  \
    FS_LAUNCH("sort_scatter", (sort_scatter_kernel<PairReader, NB>), dim3(grid), dim3(kBlock), stream, in, m_max,   \
              m_dev, shift, tile_hist, chunk_sums, totals, dst_k, dst_v, (int32_t*)nullptr)
            FS_DISPATCH_BITS(nbits, FS_SCATTER_PAIRS)
#undef FS_SCATTER_PAIRS
        }
        shift += nbits;
        src_k = dst_k; src_v = dst_v;
        dst_k = (src_k == keys_a) ? keys_b : keys_a;
        dst_v = (src_v == vals_a) ? vals_b : vals_a;
    }
    *keys_out = src_k;
    *vals_out = src_v;
    return FS_OK;
}

}  // namespace fs
