// fs_plan_replication: row-frequency histogram and top-k rows under a byte budget.
//
// ACCUMULATE  plan_histogram: each block walks a span of 32768 sampled ids.  Zipf samples hit
//             a few rows most of the time, so a block keeps a 4096-entry direct-mapped cache of
//             (row, count) in LDS (first row to claim a slot keeps it); only misses and the final
//             flush reach the global counters, as saturating 32-bit atomic adds.
// SELECT      plan_mark / plan_scan / plan_move: stable compaction of the candidate rows (count > 0,
//             or all) in ascending row order into (key = ~count, value = row), reading counts once;
//             a stable radix sort by key then yields (count desc, row asc); plan_emit writes the
//             first k = min(budget / bytes_per_row, #candidates) rows, k, and the tier-0 tags.
// The candidate count lives in device memory; the sort kernels read it there.
//
// fs_plan_tiers (further down) reuses the compaction and the sort and cuts the sorted rows into
// tiers at the breakpoints of the per-row cost model.
#include "fs_common.h"
#include "radix_sort.h"

namespace fs {

constexpr int kSelTile = kBlock * 32;     // rows per block in the compaction (fewer, larger tiles: the one-block
                                          // scan of the tile counts is what they cost)

__device__ __forceinline__ void add_saturating(uint32_t* p, uint32_t v, int32_t* faults)
{
    const uint32_t old = atomicAdd(p, v);
    if (old > 0xFFFFFFFFu - v) {          // wrapped: pin the counter at the maximum
        atomicExch(p, 0xFFFFFFFFu);
        *faults |= FS_DEV_COUNT_OVERFLOW;
    }
}

__device__ __forceinline__ int plan_table_of(const int64_t* __restrict__ offsets, int T, int64_t B, int64_t i)
{
    int lo = 0, hi = T - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (offsets[(int64_t)mid * B] <= i) lo = mid; else hi = mid - 1;
    }
    return lo;
}

__global__ __launch_bounds__(kBlock) void plan_check_offsets_kernel(
    const int64_t* __restrict__ offsets, int64_t S, int64_t n, int32_t* ok_flag, int32_t* status)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool bad = false;
    for (int64_t s = tid; s < S; s += stride) bad |= offsets[s] > offsets[s + 1];
    if (tid == 0) bad |= offsets[0] != 0 || offsets[S] != n;
    if (ballot(bad) != 0 && lane_id() == 0) { report(status, FS_DEV_BAD_OFFSETS); atomicExch(ok_flag, 0); }
}

constexpr int kHistSlotBits = 14;
constexpr uint32_t kHistMul1 = 2654435761u, kHistMul1Inv = 0x0e8b2f51u;    // odd multipliers: bijections of 32-bit words,
constexpr uint32_t kHistMul2 = 2246822519u, kHistMul2Inv = 0xb6c92f47u;    // undone by their inverses mod 2^32
constexpr int kHistBlock = 1024;          // 16 waves per span: a span per 256 threads leaves the chip idle

// One block counts the ids of [blockIdx.x * span, + span) into an LDS table of 2^14 entries of 32 bits
// (64 KB: two blocks per CU, so that one block's flush, a stretch of nothing but global adds, runs beside
// the other's counting).  A row takes the first of its two slots (two hashes of the row) that is free or
// already its own; a row that finds both taken by other rows is added to the global counter at once.  An
// entry does not hold the row: the slot is the top 14 bits of a hash that is a bijection of 32-bit words,
// so the other 18 bits (plus one, so that a used entry is never zero, and one bit for which hash it was)
// name the row, and the 12 bits above them count it; a count that wraps sends its 4096 to the global
// counter at once.  At the end the table is flushed with one saturating add per used slot.  The first row
// to claim a slot keeps it, so the counts stay exact.
// What the kernel costs is its global adds: the chip retires about 27 G of them a second wherever they land
// (one table of 64 KB or 1 GB of counters, one XCD's or all, returning or not), and a span cannot need fewer
// than it has distinct rows.  Measured: (row, count) pairs of 64 bits, half as many entries in the same LDS:
// 7 % slower on 10^9 ids of Zipf(1.3), 6 to 8 % on batches of 16 M and 72 M ids, 7 % FASTER on 67 M ids of
// Zipf(1.3) in one round of 512 blocks (fewer entries to flush when all blocks flush together); a quarter
// as many entries 3 to 13 % slower again; 2^14 pairs and one block per CU 0.49 ms instead of 0.39 ms on
// those 67 M ids; counting the most popular rows in registers changed nothing (the LDS is not the limit).
typedef int64_t Id2 __attribute__((ext_vector_type(2)));

__global__ __launch_bounds__(kHistBlock) void plan_histogram_kernel(
    const int64_t* __restrict__ ids, const int64_t* __restrict__ offsets, int T, int64_t B,
    const int64_t* __restrict__ row_base, int64_t n, int64_t R, int64_t span, uint32_t* __restrict__ counts,
    const int32_t* __restrict__ ok_flag, int32_t* status)
{
    constexpr int kSlots = 1 << kHistSlotBits;
    constexpr int kRestBits = 32 - kHistSlotBits;                   // bits of a row's hash that its slot does not give
    constexpr int kCountShift = kRestBits + 2;                      // entry: [count | which hash | rest + 1]
    constexpr uint32_t kTagMask = (1u << kCountShift) - 1u;
    constexpr uint32_t kCountMax = (1u << (32 - kCountShift)) - 1u;
    __shared__ uint32_t table[kSlots];         // 0 = free
    __shared__ int span_tables[2];
    if (*ok_flag == 0) return;                 // bad offsets: count nothing
    const int64_t base = (int64_t)blockIdx.x * span;
    const int64_t end = base + span < n ? base + span : n;
    if (base >= end) return;
    for (int s = threadIdx.x; s < kSlots; s += kHistBlock) table[s] = 0;
    if (threadIdx.x == 0) {
        span_tables[0] = plan_table_of(offsets, T, B, base);
        span_tables[1] = plan_table_of(offsets, T, B, end - 1);
    }
    __syncthreads();
    const int t_lo = __builtin_amdgcn_readfirstlane(span_tables[0]);
    const int t_hi = __builtin_amdgcn_readfirstlane(span_tables[1]);
    int32_t faults = 0;
    // Counts one row in the LDS table.  At most one global add comes of it: of 1 for a row that finds both
    // its slots taken, of a full count field for a row whose count in the table has just wrapped to zero.  The
    // add is issued here and its old value handed back (`*went` = the row + 1, `*amount`), so that the caller
    // can look at the answers of a whole batch of ids at once instead of waiting for each on its own.
    auto count_row = [&](uint32_t g, uint32_t* went, uint32_t* amount, uint32_t* old) {
        const uint32_t h1 = g * kHistMul1;
        const uint32_t s1 = h1 >> kRestBits;
        const uint32_t tag1 = (h1 & ((1u << kRestBits) - 1u)) + 1u;
        uint32_t e = table[s1];
        if (e == 0) e = atomicCAS(&table[s1], 0u, tag1);
        uint32_t* mine = nullptr;
        if (e == 0 || (e & kTagMask) == tag1) mine = &table[s1];
        else {
            const uint32_t h2 = (g ^ (g >> 15)) * kHistMul2;
            const uint32_t s2 = h2 >> kRestBits;
            const uint32_t tag2 = ((h2 & ((1u << kRestBits) - 1u)) + 1u) | (1u << (kRestBits + 1));
            e = table[s2];
            if (e == 0) e = atomicCAS(&table[s2], 0u, tag2);
            if (e == 0 || (e & kTagMask) == tag2) mine = &table[s2];
        }
        if (mine != nullptr) {
            // the count is the entry's top field: a carry out of it is lost, the tag below it stays whole
            const uint32_t before = atomicAdd(mine, 1u << kCountShift);
            if ((before >> kCountShift) != kCountMax) return;
            *amount = kCountMax + 1u;                               // wrapped to zero: that many counts go to memory now
        }
        *went = g + 1u;
        *old = atomicAdd(counts + g, *amount);
    };
    auto settle = [&](uint32_t went, uint32_t amount, uint32_t old) {   // the add wrapped: pin the counter at the maximum
        if (went != 0 && old > 0xFFFFFFFFu - amount) {
            atomicExch(counts + (went - 1u), 0xFFFFFFFFu);
            faults |= FS_DEV_COUNT_OVERFLOW;
        }
    };
    // The span table by table (nearly always one): the table's first row and size are the same for all of
    // its ids, so the loop over the ids loads nothing but the ids, two to a lane (16 bytes) where the
    // address allows it.
    for (int t = t_lo; t <= t_hi; ++t) {
        int64_t lo = offsets[(int64_t)t * B];
        int64_t hi = offsets[(int64_t)(t + 1) * B];
        lo = lo > base ? lo : base;
        hi = hi < end ? hi : end;
        if (lo >= hi) continue;
        const int64_t first = row_base[t];
        const int64_t rows_t = row_base[t + 1] - first;
        auto count_one = [&](int64_t id, uint32_t* went, uint32_t* amount, uint32_t* old) {
            *went = 0;
            *amount = 1u;
            *old = 0;
            if (id < 0 || id >= rows_t) { faults |= FS_DEV_BAD_ID; id = 0; }
            if ((uint64_t)(first + id) >= (uint64_t)R) { faults |= FS_DEV_BAD_ID; return; }   // row_base does not fit R
            count_row((uint32_t)(first + id), went, amount, old);
        };
        if ((reinterpret_cast<uintptr_t>(ids + lo) & 15) != 0) {         // an odd first id: on its own
            if (threadIdx.x == 0) {
                uint32_t went, amount, old;
                count_one(load_stream(ids + lo), &went, &amount, &old);
                settle(went, amount, old);
            }
            ++lo;
        }
        const Id2* pairs = reinterpret_cast<const Id2*>(ids + lo);
        const int64_t num_pairs = (hi - lo) >> 1;
        constexpr int kAhead = 4;                                // pairs of ids in flight per thread
        int64_t p = threadIdx.x;
        for (; p + (int64_t)(kAhead - 1) * kHistBlock < num_pairs; p += (int64_t)kAhead * kHistBlock) {
            Id2 id[kAhead];
            uint32_t went[2 * kAhead], amount[2 * kAhead], old[2 * kAhead];
#pragma unroll
            for (int q = 0; q < kAhead; ++q) id[q] = load_stream(pairs + p + (int64_t)q * kHistBlock);
#pragma unroll
            for (int q = 0; q < kAhead; ++q) {
                count_one(id[q].x, &went[2 * q], &amount[2 * q], &old[2 * q]);
                count_one(id[q].y, &went[2 * q + 1], &amount[2 * q + 1], &old[2 * q + 1]);
            }
#pragma unroll
            for (int q = 0; q < 2 * kAhead; ++q) settle(went[q], amount[q], old[q]);
        }
        for (; p < num_pairs; p += kHistBlock) {
            const Id2 id = load_stream(pairs + p);
            uint32_t went[2], amount[2], old[2];
            count_one(id.x, &went[0], &amount[0], &old[0]);
            count_one(id.y, &went[1], &amount[1], &old[1]);
            settle(went[0], amount[0], old[0]);
            settle(went[1], amount[1], old[1]);
        }
        if (((hi - lo) & 1) != 0 && threadIdx.x == kHistBlock - 1) {     // an odd last id
            uint32_t went, amount, old;
            count_one(load_stream(ids + hi - 1), &went, &amount, &old);
            settle(went, amount, old);
        }
    }
    __syncthreads();
    // The flush: one saturating add per used slot.  A thread's adds are all issued before the first old
    // value is looked at: one after the other, each waiting for its answer, they are the longest stretch
    // of a span (nothing else runs on the CU beside the block that holds its LDS).
    constexpr int kPerThread = kSlots / kHistBlock;
    constexpr int kBatch = kPerThread < 8 ? kPerThread : 8;
#pragma unroll 1
    for (int s0 = 0; s0 < kPerThread; s0 += kBatch) {
        uint32_t tag[kBatch], add[kBatch], old[kBatch];
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
            const int s = (s0 + q) * kHistBlock + threadIdx.x;
            const uint32_t e = table[s];
            add[q] = e >> kCountShift;
            // the row back from its slot and the rest of its hash: both hashes are bijections of 32-bit words
            const uint32_t h = ((uint32_t)s << kRestBits) | ((e & ((1u << (kRestBits + 1)) - 1u)) - 1u);
            uint32_t g;
            if ((e >> (kRestBits + 1)) & 1u) {
                const uint32_t y = h * kHistMul2Inv;
                g = y ^ (y >> 15) ^ (y >> 30);
            } else {
                g = h * kHistMul1Inv;
            }
            tag[q] = e != 0 ? g + 1u : 0u;
        }
#pragma unroll
        for (int q = 0; q < kBatch; ++q)
            old[q] = (tag[q] != 0 && add[q] != 0) ? atomicAdd(counts + (tag[q] - 1u), add[q]) : 0u;
#pragma unroll
        for (int q = 0; q < kBatch; ++q) {
            if (tag[q] != 0 && add[q] != 0 && old[q] > 0xFFFFFFFFu - add[q]) {     // wrapped: pin the counter at the maximum
                atomicExch(counts + (tag[q] - 1u), 0xFFFFFFFFu);
                faults |= FS_DEV_COUNT_OVERFLOW;
            }
        }
    }
    if (ballot(faults != 0) != 0) {
        for (int off = 32; off > 0; off >>= 1) faults |= __shfl_down(faults, off);
        if (lane_id() == 0) report(status, faults);
    }
}

// Span length for n ids: batches keep 32 k spans (many blocks).  From one 64 k span for each of the two
// blocks a CU holds, spans of up to 128 k ids, shortened so that their number is a multiple of the CU count
// where that is possible.  A popular row is flushed once per span, so a planning pass over very many ids
// (from 2^27) takes spans of up to 512 k ids, all of one length and a whole number of rounds over the chip's
// 512 resident blocks: 10^9 ids of Zipf(1.3) in one call take 4.7 ms with 128 k spans, 4.1 ms with 512 k,
// 10 ms with 2 M.  A training batch of a flatter law (72 M ids of Zipf(1.1) over 16 tables) does better with
// the shorter spans (1.13 ms at 96 k, 1.25 ms at 144 k): the first rows to arrive keep the slots, and a fresh
// table serves the rows that repeat within a stretch.
constexpr int64_t kHistSpanSmall = 32768;
constexpr int64_t kHistSpanLarge = 131072;
constexpr int64_t kHistSpanHuge = 524288;
constexpr int64_t kHistHugeFrom = (int64_t)1 << 27;
constexpr int64_t kHistCus = 256;

static int64_t hist_span(int64_t n)
{
    if (n < 2 * kHistCus * (kHistSpanLarge / 2)) return kHistSpanSmall;   // under one 64 k span for every CU, twice over
    const int64_t longest = n >= kHistHugeFrom ? kHistSpanHuge : kHistSpanLarge;
    const int64_t per_round = n >= kHistHugeFrom ? 2 * kHistCus : kHistCus;
    const int64_t rounds = (n + per_round * longest - 1) / (per_round * longest);
    int64_t s = (n + per_round * rounds - 1) / (per_round * rounds);
    s = (s + 8191) / 8192 * 8192;                                // whole rounds of 8 ids per thread
    return s < longest ? s : longest;
}

// ---- selection --------------------------------------------------------------
// Reads counts once: the candidates of a 8192-row tile are packed, in row order, at the tile's
// own place in a staging buffer (keys/vals at [tile * 8192 + i]) and counted.
// VEC: a lane loads four consecutive counters at once (counts 16-byte aligned); the packed order is the same.
template <bool VEC>
__global__ __launch_bounds__(kBlock) void plan_mark_kernel(
    const uint32_t* __restrict__ counts, int64_t R, int allow_zero, uint32_t* __restrict__ tile_count,
    uint32_t* __restrict__ stage_keys, uint32_t* __restrict__ stage_vals)
{
    __shared__ uint32_t wave_sum[kWavesPerBlock];
    constexpr int kItems = kSelTile / kBlock;
    constexpr int kSpan = kWave * kItems;                 // consecutive rows per wave
    constexpr int kStep = VEC ? 4 : 1;                    // consecutive rows per lane and load
    const int w = wave_id();
    const int lane = lane_id();
    const int64_t tile_base = (int64_t)blockIdx.x * kSelTile;
    const int64_t base = tile_base + (int64_t)w * kSpan;
    // item `it` of a lane is row base + row_of(it): with VEC, load it / 4 brings rows 4 * lane .. 4 * lane + 3 of a
    // stretch of 256
    auto row_of = [&](int it) { return VEC ? (it / 4) * (kWave * 4) + lane * 4 + (it & 3) : it * kWave + lane; };
    uint32_t cnt[kItems];
    uint32_t before[kItems];
    bool cand[kItems];
    uint32_t total = 0;
    if constexpr (VEC) {
#pragma unroll
        for (int v = 0; v < kItems / 4; ++v) {
            const int64_t g = base + row_of(4 * v);
            u32x4 c = {0u, 0u, 0u, 0u};
            if (g + 3 < R) {
                c = *reinterpret_cast<const u32x4*>(counts + g);
            } else {
                if (g < R) c[0] = counts[g];
                if (g + 1 < R) c[1] = counts[g + 1];
                if (g + 2 < R) c[2] = counts[g + 2];
            }
            cnt[4 * v] = c[0]; cnt[4 * v + 1] = c[1]; cnt[4 * v + 2] = c[2]; cnt[4 * v + 3] = c[3];
        }
    } else {
#pragma unroll
        for (int it = 0; it < kItems; ++it) {
            const int64_t g = base + row_of(it);
            cnt[it] = g < R ? counts[g] : 0u;
        }
    }
    // Position of a candidate among the wave's: those of earlier stretches, those of lower lanes in its stretch
    // (one ballot per item position), and the lane's own earlier items of the stretch.
#pragma unroll
    for (int it0 = 0; it0 < kItems; it0 += kStep) {
        uint32_t lower = 0, mine = 0, all = 0;
#pragma unroll
        for (int e = 0; e < kStep; ++e) {
            const int it = it0 + e;
            const int64_t g = base + row_of(it);
            cand[it] = g < R && (allow_zero || cnt[it] != 0);
            const uint64_t bal = ballot(cand[it]);
            before[it] = mine;
            lower += (uint32_t)popc_below(bal);
            mine += cand[it] ? 1u : 0u;
            all += (uint32_t)__popcll(bal);
        }
#pragma unroll
        for (int e = 0; e < kStep; ++e) before[it0 + e] += total + lower;
        total += all;
    }
    if (lane == 0) wave_sum[w] = total;
    __syncthreads();
    uint32_t off = 0, all = 0;
    for (int k = 0; k < kWavesPerBlock; ++k) {
        if (k < w) off += wave_sum[k];
        all += wave_sum[k];
    }
    if (threadIdx.x == 0) tile_count[blockIdx.x] = all;
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        if (cand[it]) {
            const int64_t g = base + row_of(it);
            stage_keys[tile_base + off + before[it]] = ~cnt[it];
            stage_vals[tile_base + off + before[it]] = (uint32_t)g;
        }
    }
}

static fs_status launch_mark(const uint32_t* counts, int64_t R, int allow_zero, int64_t sel_tiles, uint32_t* tile_count,
                             uint32_t* stage_keys, uint32_t* stage_vals, hipStream_t s)
{
    if ((reinterpret_cast<uintptr_t>(counts) & 15) == 0)
        FS_LAUNCH("plan_mark", plan_mark_kernel<true>, dim3((unsigned)sel_tiles), dim3(kBlock), s,
                  counts, R, allow_zero, tile_count, stage_keys, stage_vals);
    else
        FS_LAUNCH("plan_mark", plan_mark_kernel<false>, dim3((unsigned)sel_tiles), dim3(kBlock), s,
                  counts, R, allow_zero, tile_count, stage_keys, stage_vals);
    return FS_OK;
}

constexpr int kScanBlock = 1024;

__global__ __launch_bounds__(kScanBlock) void plan_scan_kernel(uint32_t* __restrict__ tile_count, int64_t tiles,
                                                               int64_t* __restrict__ num_candidates)
{
    __shared__ uint32_t wave_sums[16];
    const int64_t per = (tiles + kScanBlock - 1) / kScanBlock;
    if (per <= 16) {
        // up to 16 k tiles: a thread sums a short run of consecutive tiles, ONE scan over the block's 1024
        // sums, the thread then writes its run's prefixes (0.019 -> 0.012 ms for 10 k tiles; for longer
        // runs the strided accesses cost more than the scans they save)
        const int64_t lo = (int64_t)threadIdx.x * per < tiles ? (int64_t)threadIdx.x * per : tiles;
        const int64_t hi = lo + per < tiles ? lo + per : tiles;
        uint32_t sum = 0;
        for (int64_t k = lo; k < hi; ++k) sum += tile_count[k];
        uint32_t total;
        uint32_t run = block_exclusive_scan(sum, wave_sums, &total);
        for (int64_t k = lo; k < hi; ++k) { const uint32_t v = tile_count[k]; tile_count[k] = run; run += v; }
        if (threadIdx.x == 0) *num_candidates = (int64_t)total;
        return;
    }
    uint32_t carry = 0;                                          // coalesced rounds of 1024 tiles, 8 rounds of loads in flight
    for (int64_t base = 0; base < tiles; base += 8 * kScanBlock) {
        uint32_t v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int64_t k = base + (int64_t)q * kScanBlock + threadIdx.x;
            v[q] = k < tiles ? tile_count[k] : 0u;
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int64_t k = base + (int64_t)q * kScanBlock + threadIdx.x;
            uint32_t total;
            const uint32_t before = block_exclusive_scan(v[q], wave_sums, &total);
            if (k < tiles) tile_count[k] = carry + before;
            carry += total;
        }
    }
    if (threadIdx.x == 0) *num_candidates = (int64_t)carry;
}

// Moves each tile's packed candidates to their final place (tile_base = scanned tile counts).
__global__ __launch_bounds__(kBlock) void plan_move_kernel(
    const uint32_t* __restrict__ tile_base, int64_t tiles, const int64_t* __restrict__ num_candidates,
    const uint32_t* __restrict__ stage_keys, const uint32_t* __restrict__ stage_vals,
    uint32_t* __restrict__ keys, uint32_t* __restrict__ vals)
{
    const int64_t tile = blockIdx.x;
    const uint32_t first = tile_base[tile];
    const uint32_t next = tile + 1 < tiles ? tile_base[tile + 1] : (uint32_t)*num_candidates;
    const int64_t from = tile * kSelTile;
    for (uint32_t i = threadIdx.x; i < next - first; i += kBlock) {
        keys[first + i] = stage_keys[from + i];
        vals[first + i] = stage_vals[from + i];
    }
}

__global__ __launch_bounds__(kBlock) void plan_emit_kernel(
    const uint32_t* __restrict__ vals, const int64_t* __restrict__ num_candidates, int64_t cap,
    int64_t* __restrict__ sel_rows, int64_t* __restrict__ num_selected, uint32_t* __restrict__ placement)
{
    const int64_t nc = *num_candidates;
    const int64_t k = cap < nc ? cap : nc;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < k; i += stride) {
        const uint32_t g = vals[i];
        sel_rows[i] = (int64_t)g;
        if (placement != nullptr) placement[g] &= FS_OWNER_MASK;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) *num_selected = k;
}

__global__ void plan_set_flag_kernel(int32_t* flag) { *flag = 1; }

// The same check by one block that also sets the flag itself (few segments: one launch instead of two).
constexpr int64_t kCheckOneBlockMax = 8192;
__global__ __launch_bounds__(kHistBlock) void plan_check_offsets_one_kernel(
    const int64_t* __restrict__ offsets, int64_t S, int64_t n, int32_t* ok_flag, int32_t* status)
{
    __shared__ int any_bad;
    if (threadIdx.x == 0) any_bad = 0;
    __syncthreads();
    bool bad = false;
    for (int64_t s = threadIdx.x; s < S; s += kHistBlock) bad |= offsets[s] > offsets[s + 1];
    if (threadIdx.x == 0) bad |= offsets[0] != 0 || offsets[S] != n;
    if (ballot(bad) != 0 && lane_id() == 0) any_bad = 1;
    __syncthreads();
    if (threadIdx.x == 0) {
        *ok_flag = any_bad ? 0 : 1;
        if (any_bad) report(status, FS_DEV_BAD_OFFSETS);
    }
}

// ---- tier planner -----------------------------------------------------------
// After the same compaction and sort, rows stand in descending frequency order with
// key = ~count.  The breakpoints are thresholds on the count (found on the host from the
// parameters), so points A, C and the Flex breakpoint are partition points of the sorted keys;
// point B and the Flex budget need sums of counts over prefixes, which come from one pass of
// per-tile sums plus a scan of those.  One wave then finds every cut with 64-way searches.
constexpr int kSumTile = 4096;                // sorted counts per tile sum

typedef unsigned __int128 u128;
typedef __int128 i128;

struct TierConsts {
    uint64_t thr_a, thr_c, thr_f;             // smallest count at or above the breakpoint (2^63: none)
    int64_t static_term;                      // (dp U - 1) S
    int64_t dyn_factor;                       // U B
    int64_t flex_cost;                        // (dp U / W - 1) S
    int32_t granule, W, tiers;
};

__global__ __launch_bounds__(kBlock) void tiers_tile_sums_kernel(
    const uint32_t* __restrict__ keys, const int64_t* __restrict__ num_candidates, uint64_t* __restrict__ tile_sum)
{
    __shared__ uint64_t part[kWavesPerBlock];
    const int64_t K = *num_candidates;
    const int64_t base = (int64_t)blockIdx.x * kSumTile;
    uint64_t sum = 0;
    for (int i = threadIdx.x; i < kSumTile; i += kBlock) {
        const int64_t k = base + i;
        if (k < K) sum += (uint32_t)~keys[k];
    }
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_down(sum, off);
    if (lane_id() == 0) part[wave_id()] = sum;
    __syncthreads();
    if (threadIdx.x == 0) tile_sum[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

// tile_sum[t] -> sum of the tiles before t, tile_sum[tiles] = the grand total.  One block.
__global__ __launch_bounds__(kScanBlock) void tiers_scan_sums_kernel(uint64_t* __restrict__ tile_sum, int64_t tiles)
{
    __shared__ uint64_t wave_tot[kScanBlock / kWave];
    const int lane = lane_id();
    const int w = wave_id();
    uint64_t carry = 0;
    for (int64_t base = 0; base < tiles; base += kScanBlock) {
        const int64_t k = base + threadIdx.x;
        const uint64_t v = k < tiles ? tile_sum[k] : 0;
        uint64_t incl = v;
        for (int off = 1; off < kWave; off <<= 1) {
            const uint64_t up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        __syncthreads();                       // wave_tot of the previous round has been read
        if (lane == kWave - 1) wave_tot[w] = incl;
        __syncthreads();
        uint64_t before = 0, all = 0;
        for (int q = 0; q < kScanBlock / kWave; ++q) {
            const uint64_t t = wave_tot[q];
            if (q < w) before += t;
            all += t;
        }
        if (k < tiles) tile_sum[k] = carry + before + incl - v;
        carry += all;
    }
    if (threadIdx.x == 0) tile_sum[tiles] = carry;
}

// First index in [lo, hi) at which pred turns false (pred holds on a prefix of the range); hi if it
// never does.  Every lane of the wave calls it with the same bounds; 64 probes per round.
template <typename Pred>
__device__ __forceinline__ int64_t wave_partition_point(int64_t lo, int64_t hi, Pred pred)
{
    const int lane = lane_id();
    while (lo < hi) {
        const int64_t step = (hi - lo + kWave - 1) / kWave;
        const int64_t probe = lo + (int64_t)(lane + 1) * step - 1;      // last index of this lane's piece
        const bool holds = probe < hi ? pred(probe) : false;
        int pieces = __popcll(ballot(holds));                            // whole pieces on which pred holds
        // The count is the same in every lane, and left to itself the compiler does the two bound updates
        // below in scalar registers, where (hipcc of ROCm 7.2, gfx950) the second of two back-to-back
        // 64-bit compare-and-selects reuses the first one's condition bit: lo then takes hi's branch
        // whenever the probe past new_lo lies outside the range.  Held in a vector register the count
        // makes them vector selects.
        asm volatile("" : "+v"(pieces));
        const int64_t new_lo = lo + (int64_t)pieces * step;
        const int64_t first_false_probe = new_lo + step - 1;
        hi = first_false_probe < hi ? first_false_probe : hi;
        lo = new_lo < hi ? new_lo : hi;
    }
    return lo;
}

// Sum of the first k sorted counts: the scanned tile sums plus a partial tile, summed by the wave.
__device__ __forceinline__ uint64_t prefix_count(const uint32_t* __restrict__ keys,
                                                 const uint64_t* __restrict__ tile_sum, int64_t k)
{
    const int64_t t = k / kSumTile;
    uint64_t part = 0;
    for (int64_t i = t * kSumTile + lane_id(); i < k; i += kWave) part += (uint32_t)~keys[i];
    for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
    return tile_sum[t] + part;
}

// Summed DP memory terms of the first k rows, times U * S:  k (dp U - 1) S - U B P(k).
__device__ __forceinline__ i128 cum_memory(const TierConsts& c, int64_t k, uint64_t prefix)
{
    return (i128)k * (i128)c.static_term - (i128)c.dyn_factor * (i128)prefix;
}

__global__ __launch_bounds__(kWave) void tiers_cuts_kernel(
    const uint32_t* __restrict__ keys, const int64_t* __restrict__ num_candidates,
    const uint64_t* __restrict__ tile_sum, const TierConsts c, int64_t* __restrict__ cuts)
{
    const int lane = lane_id();
    const int64_t K = *num_candidates;
    const int64_t tiles = (K + kSumTile - 1) / kSumTile;
    auto at_least = [&](uint64_t thr) {
        return wave_partition_point(0, K, [&](int64_t i) { return (uint64_t)(uint32_t)~keys[i] >= thr; });
    };
    const int64_t kA = at_least(c.thr_a);
    const int64_t kC = at_least(c.thr_c);
    const int64_t kF = at_least(c.thr_f);

    // point B: the summed terms are <= 0 on a prefix of k = 0 .. K.  Tile boundaries first
    // (k_t = min(t * tile, K), P(k_t) = tile_sum[t]), then the rows of the one tile that holds it.
    const int64_t t_false = wave_partition_point(0, tiles + 1, [&](int64_t t) {
        const int64_t k = t * kSumTile < K ? t * kSumTile : K;
        return cum_memory(c, k, tile_sum[t]) <= 0;
    });
    int64_t kB;
    if (t_false > tiles) {
        kB = K;
    } else {
        const int64_t t0 = t_false - 1;                                  // boundary t0 holds, t0 + 1 does not
        const int64_t first = t0 * kSumTile;
        constexpr int kPer = kSumTile / kWave;                           // consecutive rows per lane
        uint64_t mine = 0;
        for (int q = 0; q < kPer; ++q) {
            const int64_t i = first + (int64_t)lane * kPer + q;
            if (i < K) mine += (uint32_t)~keys[i];
        }
        uint64_t incl = mine;
        for (int off = 1; off < kWave; off <<= 1) {
            const uint64_t up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        uint64_t run = tile_sum[t0] + incl - mine;
        int64_t best = first;                                            // cum(first) <= 0 is known
        for (int q = 0; q < kPer; ++q) {
            const int64_t i = first + (int64_t)lane * kPer + q;
            if (i < K) {
                run += (uint32_t)~keys[i];
                if (cum_memory(c, i + 1, run) <= 0) best = i + 1;
            }
        }
        for (int off = 32; off > 0; off >>= 1) {
            const int64_t other = __shfl_xor(best, off);
            best = other > best ? other : best;
        }
        kB = best;
    }

    const int64_t gran = c.granule;
    int64_t n_dp, n_flex = 0;
    if (c.tiers == 2) {
        n_dp = kB / gran * gran;
    } else {
        n_dp = kA / gran * gran;
        const i128 saved = -cum_memory(c, n_dp, prefix_count(keys, tile_sum, n_dp));     // >= 0
        int64_t room = K - n_dp;
        if (kF - n_dp < room) room = kF > n_dp ? kF - n_dp : 0;
        int64_t lo = 0, hi = room;                                       // most rows j with j * flex_cost <= saved
        if (c.flex_cost > 0) {
            while (lo < hi) {
                const int64_t mid = lo + (hi - lo + 1) / 2;
                if ((i128)mid * (i128)c.flex_cost <= saved) lo = mid; else hi = mid - 1;
            }
        } else {
            lo = room;
        }
        n_flex = lo / gran * gran;
    }
    const uint64_t sum_dp = prefix_count(keys, tile_sum, n_dp);
    const uint64_t sum_both = prefix_count(keys, tile_sum, n_dp + n_flex);
    if (lane == 0) {
        cuts[0] = K; cuts[1] = kA; cuts[2] = kB; cuts[3] = kC; cuts[4] = kF;
        cuts[5] = n_dp; cuts[6] = n_flex;
        cuts[7] = (int64_t)tile_sum[tiles]; cuts[8] = (int64_t)sum_dp; cuts[9] = (int64_t)(sum_both - sum_dp);
    }
}

__global__ __launch_bounds__(kBlock) void tiers_emit_kernel(
    const uint32_t* __restrict__ vals, const int64_t* __restrict__ cuts, int64_t cap, int W,
    int64_t* __restrict__ sorted_rows, uint32_t* __restrict__ placement)
{
    const int64_t n_dp = cuts[5];
    const int64_t n_both = n_dp + cuts[6];
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_both; i += stride) {
        const uint32_t g = vals[i];
        if (i < cap) sorted_rows[i] = (int64_t)g;
        if (placement != nullptr) {
            if (i < n_dp) placement[g] &= FS_OWNER_MASK;
            else placement[g] = (1u << FS_TIER_SHIFT) | (uint32_t)((i - n_dp) % W);
        }
    }
}

}  // namespace fs

extern "C" fs_status fs_plan_replication(
    const int64_t* ids, const int64_t* offsets, int32_t T, int32_t B,
    const int64_t* row_base, int64_t n, int64_t R,
    uint32_t* counts, int32_t flags,
    int64_t budget_bytes, int64_t bytes_per_row,
    int64_t* sel_rows, int64_t* num_selected,
    uint32_t* placement,
    void* workspace, size_t* workspace_bytes, void* stream, int32_t* dev_status)
{
    using namespace fs;
    if (!workspace_bytes) return FS_ERR_NULL;
    if (flags & ~(FS_PLAN_ACCUMULATE | FS_PLAN_SELECT | FS_PLAN_TAG | FS_PLAN_ALLOW_ZERO)) return FS_ERR_CONFIG;
    if ((flags & FS_PLAN_TAG) && !(flags & FS_PLAN_SELECT)) return FS_ERR_CONFIG;
    if (R < 1 || R >= 4294967295LL) return FS_ERR_SIZE;
    const bool acc = flags & FS_PLAN_ACCUMULATE;
    const bool sel = flags & FS_PLAN_SELECT;
    if (acc && (n < 0 || n >= (1LL << 31) || T < 1 || B < 1 || (int64_t)T * B >= (1LL << 31))) return FS_ERR_SIZE;
    if (sel && (budget_bytes < 0 || bytes_per_row < 1)) return FS_ERR_SIZE;

    const int64_t sel_tiles = sel ? (R + kSelTile - 1) / kSelTile : 0;
    const int64_t m_max = sel ? R : 0;
    Carver ws(workspace);
    int32_t* ok_flag = ws.take<int32_t>(1);
    int64_t* num_cand = ws.take<int64_t>(1);
    uint32_t* tile_count = ws.take<uint32_t>((size_t)sel_tiles);
    uint32_t* keys_a = ws.take<uint32_t>((size_t)m_max);
    uint32_t* vals_a = ws.take<uint32_t>((size_t)m_max);
    uint32_t* keys_b = ws.take<uint32_t>((size_t)m_max);
    uint32_t* vals_b = ws.take<uint32_t>((size_t)m_max);
    char* sort_scratch = ws.take<char>(sel ? radix_sort_scratch_bytes(m_max) : 0);
    if (!workspace) { *workspace_bytes = ws.used; return FS_OK; }
    if (*workspace_bytes < ws.used || (reinterpret_cast<uintptr_t>(workspace) & 255)) return FS_ERR_WORKSPACE;
    if (!counts) return FS_ERR_NULL;
    if (acc && (!offsets || !row_base || (n > 0 && !ids))) return FS_ERR_NULL;
    if (acc && ((reinterpret_cast<uintptr_t>(ids) & 7) || (reinterpret_cast<uintptr_t>(counts) & 3))) return FS_ERR_ALIGN;   // natural alignment: ids are read two at a time
    if (sel && !num_selected) return FS_ERR_NULL;
    if ((flags & FS_PLAN_TAG) && !placement) return FS_ERR_NULL;
    const int64_t cap = sel ? budget_bytes / bytes_per_row : 0;
    if (sel && cap > 0 && !sel_rows) return FS_ERR_NULL;

    hipStream_t s = static_cast<hipStream_t>(stream);
    if (acc) {
        const int64_t S = (int64_t)T * B;
        if (S <= kCheckOneBlockMax) {
            FS_LAUNCH("plan_check_offsets", plan_check_offsets_one_kernel, dim3(1), dim3(kHistBlock), s,
                      offsets, S, n, ok_flag, dev_status);
        } else {
            FS_LAUNCH("plan_set_flag", plan_set_flag_kernel, dim3(1), dim3(1), s, ok_flag);
            const unsigned grid = (unsigned)((S + kBlock - 1) / kBlock < 1024 ? (S + kBlock - 1) / kBlock : 1024);
            FS_LAUNCH("plan_check_offsets", plan_check_offsets_kernel, dim3(grid), dim3(kBlock), s,
                      offsets, S, n, ok_flag, dev_status);
        }
        if (n > 0) {
            const int64_t span = hist_span(n);
            const int64_t blocks = (n + span - 1) / span;
            FS_LAUNCH("plan_histogram", plan_histogram_kernel, dim3((unsigned)blocks), dim3(kHistBlock), s,
                      ids, offsets, (int)T, (int64_t)B, row_base, n, R, span, counts, ok_flag, dev_status);
        }
    }
    if (sel) {
        const int allow_zero = (flags & FS_PLAN_ALLOW_ZERO) ? 1 : 0;
        if (fs_status rc = launch_mark(counts, R, allow_zero, sel_tiles, tile_count, keys_b, vals_b, s); rc != FS_OK) return rc;
        FS_LAUNCH("plan_scan", plan_scan_kernel, dim3(1), dim3(kScanBlock), s, tile_count, sel_tiles, num_cand);
        FS_LAUNCH("plan_move", plan_move_kernel, dim3((unsigned)sel_tiles), dim3(kBlock), s,
                  tile_count, sel_tiles, num_cand, keys_b, vals_b, keys_a, vals_a);
        uint32_t* keys = nullptr;
        uint32_t* vals = nullptr;
        fs_status rc = radix_sort_pairs(keys_a, vals_a, keys_b, vals_b, m_max, num_cand, 32, sort_scratch, s,
                                        &keys, &vals);
        if (rc != FS_OK) return rc;
        FS_LAUNCH("plan_emit", plan_emit_kernel, dim3(1024), dim3(kBlock), s,
                  vals, num_cand, cap, sel_rows, num_selected, (flags & FS_PLAN_TAG) ? placement : nullptr);
    }
    return FS_OK;
}

extern "C" fs_status fs_plan_tiers(
    const uint32_t* counts, int64_t R, const fs_tier_params* params, int32_t tiers,
    int64_t* sorted_rows, int64_t cap, int64_t* cuts, uint32_t* placement,
    void* workspace, size_t* workspace_bytes, void* stream, int32_t* dev_status)
{
    using namespace fs;
    (void)dev_status;
    if (!workspace_bytes || !params) return FS_ERR_NULL;
    if (R < 1 || R >= 4294967295LL || cap < 0) return FS_ERR_SIZE;
    if (tiers != 2 && tiers != 3) return FS_ERR_CONFIG;
    const fs_tier_params& p = *params;
    if (p.num_samples < 1 || p.num_samples >= (1LL << 40) || p.B < 1 || p.B >= (1LL << 31)) return FS_ERR_CONFIG;
    if (p.U < 1 || p.U > FS_MAX_BUCKETS || p.W < 1 || p.U % p.W != 0) return FS_ERR_CONFIG;
    if (p.dp_multiplier < 1 || p.dp_multiplier > 1024 || p.granule < 1 || p.granule > (1 << 20)) return FS_ERR_CONFIG;
    const int64_t bw_max = 1LL << 20;
    if (p.a2a_global < 1 || p.a2a_global >= bw_max || p.a2a_intra < 1 || p.a2a_intra >= bw_max ||
        p.ar_global < 1 || p.ar_global >= bw_max || p.ar_cross < 1 || p.ar_cross >= bw_max)
        return FS_ERR_CONFIG;

    const int64_t sel_tiles = (R + kSelTile - 1) / kSelTile;
    const int64_t sum_tiles = (R + kSumTile - 1) / kSumTile;
    Carver ws(workspace);
    int64_t* num_cand = ws.take<int64_t>(1);
    uint32_t* tile_count = ws.take<uint32_t>((size_t)sel_tiles);
    uint64_t* tile_sum = ws.take<uint64_t>((size_t)sum_tiles + 1);
    uint32_t* keys_a = ws.take<uint32_t>((size_t)R);
    uint32_t* vals_a = ws.take<uint32_t>((size_t)R);
    uint32_t* keys_b = ws.take<uint32_t>((size_t)R);
    uint32_t* vals_b = ws.take<uint32_t>((size_t)R);
    char* sort_scratch = ws.take<char>(radix_sort_scratch_bytes(R));
    if (!workspace) { *workspace_bytes = ws.used; return FS_OK; }
    if (*workspace_bytes < ws.used || (reinterpret_cast<uintptr_t>(workspace) & 255)) return FS_ERR_WORKSPACE;
    if (!counts || !cuts) return FS_ERR_NULL;
    if (cap > 0 && !sorted_rows) return FS_ERR_NULL;

    // Breakpoints as thresholds on the count, exact: the smallest count c with
    //   A:    U B c >= (dp U - 1) S                      (DP memory term <= 0)
    //   C:    2 B ar_global c >= a2a_global S            (DP traffic term <= 0)
    //   FLEX: 2 B (a2a_intra - a2a_global) W ar_cross c >= S a2a_global a2a_intra
    auto ceil_div = [](u128 num, u128 den) -> uint64_t {
        const u128 q = (num + den - 1) / den;
        return q > (u128)1 << 62 ? (uint64_t)1 << 62 : (uint64_t)q;
    };
    TierConsts c;
    c.static_term = ((int64_t)p.dp_multiplier * p.U - 1) * p.num_samples;
    c.dyn_factor = (int64_t)p.U * p.B;
    c.flex_cost = ((int64_t)p.dp_multiplier * (p.U / p.W) - 1) * p.num_samples;
    c.granule = p.granule;
    c.W = p.W;
    c.tiers = tiers;
    c.thr_a = ceil_div((u128)c.static_term, (u128)c.dyn_factor);
    c.thr_c = ceil_div((u128)p.a2a_global * (u128)p.num_samples, (u128)2 * p.B * p.ar_global);
    c.thr_f = p.a2a_intra > p.a2a_global
                  ? ceil_div((u128)p.num_samples * p.a2a_global * p.a2a_intra,
                             (u128)2 * p.B * (p.a2a_intra - p.a2a_global) * p.W * p.ar_cross)
                  : (uint64_t)1 << 62;

    hipStream_t s = static_cast<hipStream_t>(stream);
    if (fs_status rc = launch_mark(counts, R, 0, sel_tiles, tile_count, keys_b, vals_b, s); rc != FS_OK) return rc;
    FS_LAUNCH("plan_scan", plan_scan_kernel, dim3(1), dim3(kScanBlock), s, tile_count, sel_tiles, num_cand);
    FS_LAUNCH("plan_move", plan_move_kernel, dim3((unsigned)sel_tiles), dim3(kBlock), s,
              tile_count, sel_tiles, num_cand, keys_b, vals_b, keys_a, vals_a);
    uint32_t* keys = nullptr;
    uint32_t* vals = nullptr;
    fs_status rc = radix_sort_pairs(keys_a, vals_a, keys_b, vals_b, R, num_cand, 32, sort_scratch, s, &keys, &vals);
    if (rc != FS_OK) return rc;
    FS_LAUNCH("tiers_tile_sums", tiers_tile_sums_kernel, dim3((unsigned)sum_tiles), dim3(kBlock), s,
              keys, num_cand, tile_sum);
    FS_LAUNCH("tiers_scan_sums", tiers_scan_sums_kernel, dim3(1), dim3(kScanBlock), s, tile_sum, sum_tiles);
    FS_LAUNCH("tiers_cuts", tiers_cuts_kernel, dim3(1), dim3(kWave), s, keys, num_cand, tile_sum, c, cuts);
    FS_LAUNCH("tiers_emit", tiers_emit_kernel, dim3(1024), dim3(kBlock), s, vals, cuts, cap, (int)p.W,
              sorted_rows, placement);
    return FS_OK;
}
