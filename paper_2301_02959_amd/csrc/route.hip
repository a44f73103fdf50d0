// fs_route_bucketize: jagged ids -> (tier, owner) -> stable bucketize by owner.
//
// A stable counting sort of the n lookups by destination bucket, in four steps
// that touch each lookup twice:
//   route_remap     one 2048-lookup tile per block: table of each lookup, global
//                   row g, placement entry, destination; per-tile bucket
//                   histogram (wave-aggregated LDS adds) plus the tile's three tier
//                   counts; dest (u16) and g (u32) go to the workspace; each block also
//                   validates its share of the offsets
//   route_scan      one block per bucket (and per tier): exclusive scan of its per-tile
//                   counts over the tiles, and its total
//   route_scatter   same tiles: each wave ranks its 512 consecutive lookups by
//                   ballot matching against a wave-private running histogram in
//                   LDS, adds the tile's and the bucket's base, writes
//                   out_rows / out_pos
//                   (its first block also writes bucket_offsets and tier_counts)
//   route_prepare / route_finalize   only for an empty batch: the offsets check and the
//                   zero outputs
// No spin-waits anywhere: the only cross-block communication is between launches.
#include <atomic>

#include "fs_common.h"

namespace fs {

constexpr int kRouteItems = 8;                        // lookups per thread
constexpr int kRouteTile = kBlock * kRouteItems;      // lookups per block
constexpr int kRouteWaveSpan = kWave * kRouteItems;   // consecutive lookups per wave
constexpr int kRouteStripe = 32;                      // tiles per XCD stripe in the scatter

__global__ __launch_bounds__(kBlock) void route_prepare_kernel(
    const int64_t* __restrict__ offsets, int64_t S, int64_t n, int32_t* status)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool bad = false;
    for (int64_t s = tid; s < S; s += stride) bad |= offsets[s] > offsets[s + 1];
    if (tid == 0) bad |= offsets[0] != 0 || offsets[S] != n;
    if (ballot(bad) != 0 && lane_id() == 0) report(status, FS_DEV_BAD_OFFSETS);
}

// Table of lookup i: the largest t in [0, T) with offsets[t * B] <= i.  Clamped, so bad
// offsets cannot take it out of range.
__device__ __forceinline__ int table_of(const int64_t* __restrict__ offsets, int T, int64_t B, int64_t i)
{
    int lo = 0, hi = T - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (offsets[(int64_t)mid * B] <= i) lo = mid; else hi = mid - 1;
    }
    return lo;
}

__global__ __launch_bounds__(kBlock) void route_remap_kernel(
    const int64_t* __restrict__ ids, const int64_t* __restrict__ offsets, int T, int64_t B,
    const int64_t* __restrict__ row_base, const uint32_t* __restrict__ placement,
    int64_t n, int U, int W, int self, int dest_bits,
    uint16_t* __restrict__ dest_out, uint32_t* __restrict__ g_out, int32_t* __restrict__ slot_out /* or null */,
    uint32_t* __restrict__ tile_hist /* [U + 3][tiles]: buckets, then the three tiers */, int64_t tiles,
    int32_t* status)
{
    // this block's share of the offsets check (S = T * B segments over `tiles` blocks)
    {
        const int64_t S = (int64_t)T * B;
        const int64_t per = (S + tiles - 1) / tiles;
        const int64_t lo = (int64_t)blockIdx.x * per;
        const int64_t hi = lo + per < S ? lo + per : S;
        bool bad = false;
        for (int64_t sg = lo + threadIdx.x; sg < hi; sg += kBlock) bad |= offsets[sg] > offsets[sg + 1];
        if (blockIdx.x == 0 && threadIdx.x == 0) bad |= offsets[0] != 0 || offsets[S] != n;
        if (ballot(bad) != 0 && lane_id() == 0) report(status, FS_DEV_BAD_OFFSETS);
    }
    extern __shared__ uint32_t lds_hist[];            // [U]
    __shared__ int tile_tables[2];
    __shared__ unsigned int wave_tiers[kWavesPerBlock][3];
    const int64_t tile = blockIdx.x;
    const int64_t base = tile * kRouteTile;
    for (int b = threadIdx.x; b < U; b += kBlock) lds_hist[b] = 0;
    if (threadIdx.x == 0) {
        const int64_t last = (base + kRouteTile < n ? base + kRouteTile : n) - 1;
        tile_tables[0] = table_of(offsets, T, B, base);
        tile_tables[1] = table_of(offsets, T, B, last);
    }
    __syncthreads();
    const int t_lo = __builtin_amdgcn_readfirstlane(tile_tables[0]);
    const int t_hi = __builtin_amdgcn_readfirstlane(tile_tables[1]);
    const int group_base = (self / W) * W;
    const int64_t R_all = row_base[T];                // rows of all tables; g must stay below it (and below 2^32 - 1)
    const bool rows_ok = R_all >= 1 && R_all < 4294967295LL;
    int32_t faults = rows_ok ? 0 : FS_DEV_BAD_ID;
    unsigned int tiers[3] = {0, 0, 0};

    // Three rounds of loads for the thread's 8 lookups, each round's loads all in flight together: the
    // ids, then (only in a tile that spans tables) the offsets and row_base of each lookup's table,
    // then the placement entries.  Item by item the kernel's time was a chain of 8 x 3 dependent loads.
    int64_t id[kRouteItems];
#pragma unroll
    for (int it = 0; it < kRouteItems; ++it) {
        const int64_t i = base + (int64_t)it * kBlock + threadIdx.x;
        id[it] = load_stream(ids + (i < n ? i : n - 1));             // past the end: the last id again, unused
    }
    const int64_t first_lo = row_base[t_lo];
    const int64_t rows_lo = row_base[t_lo + 1] - first_lo;
    int64_t g[kRouteItems];
#pragma unroll
    for (int it = 0; it < kRouteItems; ++it) {
        const int64_t i = base + (int64_t)it * kBlock + threadIdx.x;
        int64_t first = first_lo, rows_t = rows_lo;
        if (t_lo != t_hi) {                                          // block-uniform
            int t = t_lo;
            while (t < t_hi && offsets[(int64_t)(t + 1) * B] <= i) ++t;
            first = row_base[t];
            rows_t = row_base[t + 1] - first;
        }
        int64_t x = id[it];
        const bool valid = i < n;
        if (x < 0 || x >= rows_t) { if (valid) faults |= FS_DEV_BAD_ID; x = 0; }
        int64_t row = first + x;
        if ((uint64_t)row >= (uint64_t)R_all) { if (valid) faults |= FS_DEV_BAD_ID; row = 0; }   // row_base not ascending
        g[it] = row;
    }
    uint32_t e[kRouteItems];
#pragma unroll
    for (int it = 0; it < kRouteItems; ++it) e[it] = rows_ok ? placement[g[it]] : 0u;
#pragma unroll
    for (int it = 0; it < kRouteItems; ++it) {
        const int64_t i = base + (int64_t)it * kBlock + threadIdx.x;
        const bool valid = i < n;
        uint32_t dest = 0;
        if (valid) {
            const uint32_t tier = e[it] >> FS_TIER_SHIFT;
            const uint32_t owner = e[it] & FS_OWNER_MASK;
            if (tier == FS_TIER_GLOBAL) {
                dest = self; tiers[0]++;
            } else if (tier == FS_TIER_GROUP) {
                tiers[1]++;
                if (owner < (uint32_t)W) dest = group_base + owner;
                else { dest = self; faults |= FS_DEV_BAD_PLACEMENT; }
            } else if (tier == FS_TIER_SHARDED) {
                tiers[2]++;
                if (owner < (uint32_t)U) dest = owner;
                else { dest = self; faults |= FS_DEV_BAD_PLACEMENT; }
            } else {
                dest = self; tiers[0]++; faults |= FS_DEV_BAD_PLACEMENT;
            }
            dest_out[i] = (uint16_t)dest;
            g_out[i] = (uint32_t)g[it];
            // a replicated row's entry names no owner: its owner bits carry the row's replica slot, if it has one
            if (slot_out != nullptr)
                slot_out[i] = (tier == FS_TIER_GLOBAL && owner != FS_OWNER_MASK) ? (int32_t)owner : -1;
        }
        // one LDS add per distinct bucket per wave
        const uint64_t same = match_bits(dest, dest_bits, valid);
        if (valid && popc_below(same) == 0) atomicAdd(&lds_hist[dest], (uint32_t)__popcll(same));
    }
    // tier counts travel as three more histogram rows (no global atomics: 3 hot addresses
    // shared by every wave of the grid serialise in L2)
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        unsigned int v = tiers[k];
        for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off);
        if (lane_id() == 0) wave_tiers[wave_id()][k] = v;
    }
    __syncthreads();
    for (int b = threadIdx.x; b < U; b += kBlock) tile_hist[(int64_t)b * tiles + tile] = lds_hist[b];
    if (threadIdx.x < 3) {
        unsigned int v = 0;
        for (int k = 0; k < kWavesPerBlock; ++k) v += wave_tiers[k][threadIdx.x];
        tile_hist[(int64_t)(U + threadIdx.x) * tiles + tile] = v;
    }
    for (int off = 32; off > 0; off >>= 1) faults |= __shfl_down(faults, off);
    if (lane_id() == 0) report(status, faults);
}

// One block per bucket b: tile_hist[b][0..tiles) -> exclusive prefix in place, total[b].
constexpr int kRouteScanBlock = 1024;                 // U + 3 blocks only: as many threads each as a block can have

__global__ __launch_bounds__(kRouteScanBlock) void route_scan_kernel(uint32_t* __restrict__ tile_hist, int64_t tiles,
                                                                     uint32_t* __restrict__ totals)
{
    __shared__ uint32_t wave_sums[16];
    uint32_t* h = tile_hist + (int64_t)blockIdx.x * tiles;
    const int64_t per = (tiles + kRouteScanBlock - 1) / kRouteScanBlock;
    const int64_t lo = (int64_t)threadIdx.x * per < tiles ? (int64_t)threadIdx.x * per : tiles;
    const int64_t hi = lo + per < tiles ? lo + per : tiles;
    uint32_t sum = 0;
    for (int64_t k = lo; k < hi; ++k) sum += h[k];
    uint32_t total;
    uint32_t run = block_exclusive_scan(sum, wave_sums, &total);
    if (threadIdx.x == 0) totals[blockIdx.x] = total;
    for (int64_t k = lo; k < hi; ++k) { const uint32_t v = h[k]; h[k] = run; run += v; }
}

__global__ __launch_bounds__(kBlock) void route_scatter_kernel(
    const uint16_t* __restrict__ dest_in, const uint32_t* __restrict__ g_in, int64_t n, int U, int dest_bits,
    const uint32_t* __restrict__ tile_hist /* scanned */, int64_t tiles, const uint32_t* __restrict__ totals,
    int64_t* __restrict__ out_rows, int32_t* __restrict__ out_pos,
    int64_t* __restrict__ bucket_offsets, int64_t* __restrict__ tier_counts,
    const int32_t* __restrict__ slot_in /* or null */, int32_t* __restrict__ out_slots)
{
    extern __shared__ uint32_t lds[];
    uint32_t* bucket_base = lds;                                        // [U] first output index of the tile in bucket b
    uint16_t* wave_hist = reinterpret_cast<uint16_t*>(lds + U);         // [waves][U]
    __shared__ uint32_t scan_part[kBlock];
    // tiles in stripes per XCD: consecutive tiles write neighbouring pieces of every bucket's range,
    // which one XCD's L2 merges into whole lines (0.082 -> 0.073 ms on 15.7 M lookups)
    const int64_t tile = xcd_striped_tile(blockIdx.x, kRouteStripe);
    if (tile >= tiles) return;                                          // block-uniform, before any barrier
    const int64_t base = tile * kRouteTile;
    const int w = wave_id();
    const int lane = lane_id();

    // exclusive scan of the bucket totals (every block repeats it: U is small)
    {
        const int per = (U + kBlock - 1) / kBlock;
        const int lo = threadIdx.x * per;
        const int hi = lo + per < U ? lo + per : U;
        uint32_t sum = 0;
        for (int b = lo; b < hi; ++b) sum += totals[b];
        scan_part[threadIdx.x] = sum;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t run = 0;
            for (int k = 0; k < kBlock; ++k) { const uint32_t v = scan_part[k]; scan_part[k] = run; run += v; }
        }
        __syncthreads();
        uint32_t run = scan_part[threadIdx.x];
        const bool writes_offsets = blockIdx.x == 0;                    // tile 0 exists whenever this kernel runs
        for (int b = lo; b < hi; ++b) {
            bucket_base[b] = run + tile_hist[(int64_t)b * tiles + tile];
            if (writes_offsets) bucket_offsets[b] = (int64_t)run;
            run += totals[b];
        }
        if (writes_offsets && threadIdx.x == 0) {
            bucket_offsets[U] = n;                                      // every lookup has a bucket
            if (tier_counts != nullptr)
                for (int k = 0; k < 3; ++k) tier_counts[k] = (int64_t)totals[U + k];
        }
    }
    for (int b = threadIdx.x; b < kWavesPerBlock * U; b += kBlock) wave_hist[b] = 0;
    __syncthreads();

    uint16_t* my_hist = wave_hist + w * U;
    uint32_t dest[kRouteItems];
    uint32_t rank[kRouteItems];
    uint32_t g[kRouteItems];
    int32_t slot[kRouteItems];
#pragma unroll
    for (int it = 0; it < kRouteItems; ++it) {
        const int64_t i = base + (int64_t)w * kRouteWaveSpan + it * kWave + lane;
        const bool valid = i < n;
        dest[it] = valid ? dest_in[i] : 0;
        g[it] = valid ? g_in[i] : 0;
        slot[it] = (valid && slot_in != nullptr) ? slot_in[i] : -1;
    }
#pragma unroll
    for (int it = 0; it < kRouteItems; ++it) {
        const int64_t i = base + (int64_t)w * kRouteWaveSpan + it * kWave + lane;
        const bool valid = i < n;
        const uint64_t same = match_bits(dest[it], dest_bits, valid);
        const uint32_t before = popc_below(same);
        uint32_t seen = 0;
        if (valid) seen = my_hist[dest[it]];
        __builtin_amdgcn_wave_barrier();
        rank[it] = seen + before;
        if (valid && before == 0) my_hist[dest[it]] = (uint16_t)(seen + __popcll(same));
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    // per bucket: turn the waves' counts into the waves' first output index
    for (int b = threadIdx.x; b < U; b += kBlock) {
        uint32_t run = 0;
#pragma unroll
        for (int k = 0; k < kWavesPerBlock; ++k) {
            const uint32_t v = wave_hist[k * U + b];
            wave_hist[k * U + b] = (uint16_t)run;
            run += v;
        }
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < kRouteItems; ++it) {
        const int64_t i = base + (int64_t)w * kRouteWaveSpan + it * kWave + lane;
        if (i < n) {
            const uint32_t j = bucket_base[dest[it]] + my_hist[dest[it]] + rank[it];
            out_rows[j] = (int64_t)g[it];
            out_pos[j] = (int32_t)i;
            if (slot_in != nullptr) out_slots[j] = slot[it];
        }
    }
}

__global__ __launch_bounds__(kBlock) void route_finalize_kernel(
    const uint32_t* __restrict__ totals /* [U + 3] */, int U, int64_t n,
    int64_t* __restrict__ bucket_offsets, int64_t* __restrict__ tier_counts)
{
    if (threadIdx.x == 0) {
        int64_t run = 0;
        for (int b = 0; b < U; ++b) { bucket_offsets[b] = run; run += (n > 0 ? totals[b] : 0u); }
        bucket_offsets[U] = run;
        if (tier_counts != nullptr)
            for (int k = 0; k < 3; ++k) tier_counts[k] = n > 0 ? (int64_t)totals[U + k] : 0;
    }
}

// Both entry points: host checks, workspace carving, the five launches.
static fs_status route_run(
    const int64_t* ids, const int64_t* offsets, int32_t T, int32_t B,
    const int64_t* row_base, const uint32_t* placement,
    int64_t n, int32_t U, int32_t W, int32_t self,
    int64_t* bucket_offsets, int64_t* out_rows, int32_t* out_pos,
    int64_t* tier_counts,
    void* workspace, size_t* workspace_bytes, void* stream, int32_t* dev_status,
    bool with_slots = false, int32_t* out_slots = nullptr)
{
    if (!workspace_bytes) return FS_ERR_NULL;
    if (n < 0 || n >= (1LL << 31) || T < 1 || B < 1 || (int64_t)T * B >= (1LL << 31)) return FS_ERR_SIZE;
    if (U < 1 || U > FS_MAX_BUCKETS || W < 1 || U % W != 0 || self < 0 || self >= U) return FS_ERR_CONFIG;

    const int64_t tiles = (n + kRouteTile - 1) / kRouteTile;
    Carver ws(workspace);
    uint32_t* totals = ws.take<uint32_t>((size_t)U + 3);
    uint32_t* tile_hist = ws.take<uint32_t>(((size_t)U + 3) * (size_t)tiles);
    uint32_t* g_tmp = ws.take<uint32_t>((size_t)n);
    uint16_t* dest_tmp = ws.take<uint16_t>((size_t)n);
    int32_t* slot_tmp = with_slots ? ws.take<int32_t>((size_t)n) : nullptr;
    if (!workspace) { *workspace_bytes = ws.used; return FS_OK; }
    if (*workspace_bytes < ws.used || (reinterpret_cast<uintptr_t>(workspace) & 255)) return FS_ERR_WORKSPACE;
    if (!offsets || !row_base || !placement || !bucket_offsets) return FS_ERR_NULL;
    if (n > 0 && (!ids || !out_rows || !out_pos || (with_slots && !out_slots))) return FS_ERR_NULL;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t S = (int64_t)T * B;
    const int dest_bits = bits_for((uint64_t)(U - 1));
    if (n == 0) {
        const unsigned prep_grid = (unsigned)((S + kBlock - 1) / kBlock < 1024 ? (S + kBlock - 1) / kBlock : 1024);
        FS_LAUNCH("route_prepare", route_prepare_kernel, dim3(prep_grid), dim3(kBlock), s,
                  offsets, S, n, dev_status);
        FS_LAUNCH("route_finalize", route_finalize_kernel, dim3(1), dim3(kBlock), s,
                  totals, (int)U, n, bucket_offsets, tier_counts);
        return FS_OK;
    }
    {
        FS_LAUNCH_SMEM("route_remap", route_remap_kernel, dim3((unsigned)tiles), dim3(kBlock),
                       (size_t)U * sizeof(uint32_t), s,
                       ids, offsets, (int)T, (int64_t)B, row_base, placement, n, (int)U, (int)W, (int)self,
                       dest_bits, dest_tmp, g_tmp, slot_tmp, tile_hist, tiles, dev_status);
        FS_LAUNCH("route_scan", route_scan_kernel, dim3((unsigned)U + 3), dim3(kRouteScanBlock), s, tile_hist, tiles, totals);
        const unsigned scatter_grid = (unsigned)xcd_striped_grid(tiles, kRouteStripe);
        FS_LAUNCH_SMEM("route_scatter", route_scatter_kernel, dim3(scatter_grid), dim3(kBlock),
                       (size_t)U * sizeof(uint32_t) + (size_t)kWavesPerBlock * U * sizeof(uint16_t), s,
                       dest_tmp, g_tmp, n, (int)U, dest_bits, tile_hist, tiles, totals, out_rows, out_pos,
                       bucket_offsets, tier_counts, (const int32_t*)slot_tmp, out_slots);
    }
    return FS_OK;
}

// ---- the variant that allocates nothing ----------------------------------------
// Its workspace is this array: one copy per GPU, held until the process ends.  The name below is a
// host-side stand-in; the device address of each GPU's copy comes from hipGetSymbolAddress and is
// what every launch receives.
static __device__ __align__(256) unsigned char scratch[FS_ROUTE_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

static fs_status scratch_of_current_device(void** ptr)
{
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return FS_ERR_DEVICE;
    void* p = g_scratch_ptr[device].load(std::memory_order_acquire);
    if (p == nullptr) {                                   // first call on this GPU (two racing threads find the same address)
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return FS_ERR_DEVICE;
        g_scratch_ptr[device].store(p, std::memory_order_release);
    }
    *ptr = p;
    return FS_OK;
}

}  // namespace fs

extern "C" fs_status fs_route_bucketize(
    const int64_t* ids, const int64_t* offsets, int32_t T, int32_t B,
    const int64_t* row_base, const uint32_t* placement,
    int64_t n, int32_t U, int32_t W, int32_t self,
    int64_t* bucket_offsets, int64_t* out_rows, int32_t* out_pos,
    int64_t* tier_counts,
    void* workspace, size_t* workspace_bytes, void* stream, int32_t* dev_status)
{
    return fs::route_run(ids, offsets, T, B, row_base, placement, n, U, W, self, bucket_offsets, out_rows, out_pos,
                         tier_counts, workspace, workspace_bytes, stream, dev_status);
}

extern "C" fs_status fs_route_bucketize_slots(
    const int64_t* ids, const int64_t* offsets, int32_t T, int32_t B,
    const int64_t* row_base, const uint32_t* placement,
    int64_t n, int32_t U, int32_t W, int32_t self,
    int64_t* bucket_offsets, int64_t* out_rows, int32_t* out_pos, int32_t* out_slots,
    int64_t* tier_counts,
    void* workspace, size_t* workspace_bytes, void* stream, int32_t* dev_status)
{
    return fs::route_run(ids, offsets, T, B, row_base, placement, n, U, W, self, bucket_offsets, out_rows, out_pos,
                         tier_counts, workspace, workspace_bytes, stream, dev_status, true, out_slots);
}

extern "C" fs_status fs_route_bucketize_noalloc(
    const int64_t* ids, const int64_t* offsets, int32_t T, int32_t B,
    const int64_t* row_base, const uint32_t* placement,
    int64_t n, int32_t U, int32_t W, int32_t self,
    int64_t* bucket_offsets, int64_t* out_rows, int32_t* out_pos,
    int64_t* tier_counts, void* stream, int32_t* dev_status)
{
    using namespace fs;
    size_t need = 0;                                      // size query: host checks only, nothing launched
    fs_status rc = route_run(ids, offsets, T, B, row_base, placement, n, U, W, self, bucket_offsets, out_rows, out_pos,
                             tier_counts, nullptr, &need, stream, dev_status);
    if (rc != FS_OK) return rc;
    if (need > (size_t)FS_ROUTE_NOALLOC_SCRATCH_BYTES) return FS_ERR_WORKSPACE;
    void* ws = nullptr;
    rc = scratch_of_current_device(&ws);
    if (rc != FS_OK) return rc;
    size_t have = (size_t)FS_ROUTE_NOALLOC_SCRATCH_BYTES;
    return route_run(ids, offsets, T, B, row_base, placement, n, U, W, self, bucket_offsets, out_rows, out_pos,
                     tier_counts, ws, &have, stream, dev_status);
}
