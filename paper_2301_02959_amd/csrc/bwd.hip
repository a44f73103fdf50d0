// fs_seq_grad_bwd: row_grads[u(r), :] = sum of f32(grad_out[pos[j], :]) over the lookups of row r.
//
// Sort-by-row segmented reduction:
//   radix sort        stable by row, the first pass reading and validating (row, pos) itself; lookups of one row keep their j order, which is
//                     ascending pos for any fs_route_bucketize output
//   bwd_count_heads   per 256-lookup chunk of the sorted order: number of runs that
//                     start in it, with a block-local exclusive prefix
//   bwd_scan_blocks   exclusive scan of the per-block sums -> index of every run,
//                     *num_unique
//   bwd_segreduce     a group of LG lanes (one 16-byte piece of the row per lane) walks
//                     one chunk left to right with 8 gradient rows in flight; the chunk's
//                     keys and positions are staged in LDS by coalesced loads and read back
//                     as broadcasts; a run that starts in the chunk goes to row_grads, the
//                     piece that continues a run from the previous chunk goes to carry[chunk]
//   bwd_singletons    runs of one lookup (most runs: the cold tail) are skipped by the walk and
//                     converted here, fully parallel
//   bwd_fold          for every run that spills over a chunk end: row_grads += carry of
//                     the following chunks, left to right
// which is exactly the summation order stated in flexshard.h (chunk = FS_BWD_TILE).
// variant 1 replaces carry + fold by fp32 atomic adds into pre-zeroed rows.
// HBM-bound: grad_out is read once (random 16*units-byte rows), row_grads written once.
// (fs_seq_grad_bwd's variant 1 still reads and writes row_grads with atomics in L2.)
#include "fs_common.h"
#include "radix_sort.h"
#include "update_rules.h"

namespace fs {

constexpr int kChunk = FS_BWD_TILE;
constexpr int kChunksPerBlock = 64;          // bwd_count_heads: chunks per block
constexpr int kSinglesSplit = 4;             // bwd_singletons: waves per chunk (divides kChunk / 64)
constexpr int kBwdUnroll = 8;               // rows a group keeps in flight
constexpr uint32_t kNoKey = 0xFFFFFFFFu;     // never a row: R < 2^32 - 1

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// Block b covers chunks [64 b, 64 b + 64): 16 waves, each walks 4 of them (with 4 waves of 16 chunks
// each the kernel's time was the chain of 16 dependent rounds of loads per wave).  chunk_local[c] = runs
// that start in the block's chunks before c; block_sum[b] = runs that start in the block.
constexpr int kHeadsBlock = 1024;
__global__ __launch_bounds__(kHeadsBlock) void bwd_count_heads_kernel(
    const uint32_t* __restrict__ keys, const uint32_t* __restrict__ vals, int64_t m, int64_t chunks,
    uint32_t n, uint32_t R,
    uint32_t* __restrict__ chunk_local, uint32_t* __restrict__ block_sum, int32_t* status)
{
    __shared__ uint32_t heads[kChunksPerBlock];
    const int w = wave_id();
    const int lane = lane_id();
    constexpr int kPerWave = kChunksPerBlock / (kHeadsBlock / kWave);
    bool disorder = false, bad = false, unsorted = false;
    for (int q = 0; q < kPerWave; ++q) {
        const int slot = w * kPerWave + q;
        const int64_t chunk = (int64_t)blockIdx.x * kChunksPerBlock + slot;
        uint32_t count = 0;
        if (chunk < chunks) {
            const int64_t k0 = chunk * kChunk;
#pragma unroll
            for (int s = 0; s < kChunk / kWave; ++s) {
                const int64_t k = k0 + s * kWave + lane;
                bool head = false;
                if (k < m) {                                         // the four loads in one round, none behind a compare
                    const int64_t kp = k > 0 ? k - 1 : 0;
                    const uint32_t key = keys[k], prev = keys[kp];
                    const uint32_t val = vals[k], pval = vals[kp];
                    head = k == 0 || key != prev;
                    if (!head && val < pval) disorder = true;
                    // pairs a caller sorted (the library's own sort has validated its input): the kernels
                    // below clamp a position outside the batch, here it is reported
                    if (key >= R || val >= n) bad = true;
                    if (k > 0 && key < prev) unsorted = true;
                }
                count += (uint32_t)__popcll(ballot(head));
            }
        }
        if (lane == 0) heads[slot] = count;
    }
    if (ballot(disorder) != 0 && lane == 0) report(status, FS_DEV_POS_ORDER);
    if (ballot(bad) != 0 && lane == 0) report(status, FS_DEV_BAD_ID);
    if (ballot(unsorted) != 0 && lane == 0) report(status, FS_DEV_NOT_SORTED);
    __syncthreads();
    if (w == 0) {
        const uint32_t mine = heads[lane];
        uint32_t incl = mine;
        for (int off = 1; off < kWave; off <<= 1) {
            const uint32_t up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        const int64_t chunk = (int64_t)blockIdx.x * kChunksPerBlock + lane;
        if (chunk < chunks) chunk_local[chunk] = incl - mine;
        if (lane == kWave - 1) block_sum[blockIdx.x] = incl;
    }
}

// One block: block_sum[0..blocks) -> exclusive prefix in place, block_sum[blocks] = total.
constexpr int kScanBlock = 1024;

__global__ __launch_bounds__(kScanBlock) void bwd_scan_blocks_kernel(
    uint32_t* __restrict__ block_sum, int64_t blocks, int64_t cap, int64_t* __restrict__ num_unique,
    int32_t* status)
{
    __shared__ uint32_t wave_sums[16];
    uint32_t carry = 0;                                          // coalesced rounds of 1024 entries
    for (int64_t base = 0; base < blocks; base += kScanBlock) {
        const int64_t k = base + threadIdx.x;
        const uint32_t v = k < blocks ? block_sum[k] : 0u;
        uint32_t total;
        const uint32_t before = block_exclusive_scan(v, wave_sums, &total);
        if (k < blocks) block_sum[k] = carry + before;
        carry += total;
    }
    if (threadIdx.x == 0) {
        block_sum[blocks] = carry;
        *num_unique = (int64_t)carry;
        if ((int64_t)carry > cap) report(status, FS_DEV_UNIQUE_OVERFLOW);
    }
}

__device__ __forceinline__ uint32_t runs_before(const uint32_t* __restrict__ block_base,
                                                const uint32_t* __restrict__ chunk_local, int64_t chunk, int64_t chunks)
{
    if (chunk >= chunks) return block_base[(chunks + kChunksPerBlock - 1) / kChunksPerBlock];
    return block_base[chunk / kChunksPerBlock] + chunk_local[chunk];
}

template <int DT>
struct Vec;
template <>
struct Vec<FS_F32> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void load(const u32x4& x, float* f)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = __uint_as_float(x[i]);   // (a bit_cast of a vector element miscompiles)
    }
};
template <>
struct Vec<FS_F16> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void load(const u32x4& x, float* f)
    {
        const f16x8 h = __builtin_bit_cast(f16x8, x);
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = (float)h[i];
    }
};
template <>
struct Vec<FS_BF16> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void load(const u32x4& x, float* f)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(x[i] << 16);
            f[2 * i + 1] = __uint_as_float(x[i] & 0xFFFF0000u);
        }
    }
};

// A group of LG lanes (LG >= 16) walks one chunk of 256 sorted lookups left to right.  The
// group first stages the chunk's keys and positions in LDS with coalesced loads (a per-step
// index load in front of every gradient row would stall the row loads); bit 31 of a staged
// position says "the run's piece ends here" (next key differs, or last lookup of the chunk).
// They are read back as LDS broadcasts, 8 lookups per batch, the next batch's 8 gradient
// rows already in flight while the current batch is summed.
constexpr uint32_t kEndBit = 0x80000000u;        // positions are < 2^31
constexpr uint32_t kSkip = 0xFFFFFFFFu;          // a run of one lookup: bwd_singletons writes it (not a position + flag:
                                                 // positions stop at 2^31 - 2)


template <int LG, int DT, bool EXACT>            // EXACT: units == LG, the row stride is a compile-time constant
__global__ __launch_bounds__(kBlock) void bwd_segreduce_kernel(
    const u32x4* __restrict__ grad, int units, int D,
    const uint32_t* __restrict__ keys, const uint32_t* __restrict__ vals, int64_t m, int64_t chunks, uint32_t n,
    const uint32_t* __restrict__ block_base, const uint32_t* __restrict__ chunk_local,
    int64_t* __restrict__ uniq_rows, float* __restrict__ row_grads, int64_t cap,
    float* __restrict__ carry, int atomic, uint8_t* __restrict__ applied)
{
    static_assert(LG >= 16 && LG <= kWave, "groups of 16..64 lanes (smaller groups would need > 64 KB of LDS)");
    constexpr int N = Vec<DT>::N;
    constexpr int GPB = kBlock / LG;
    constexpr int U8 = kBwdUnroll;
    constexpr int kPad = 2 * U8;                 // batches issued past the end read position 0
    __shared__ __attribute__((aligned(16))) uint32_t s_val[GPB][kChunk + kPad];
    __shared__ uint32_t s_key[GPB][kChunk + 1];  // [kChunk]: the key that follows the chunk
    __shared__ __attribute__((aligned(16))) float s_stage[N == 8 ? GPB : 1][N == 8 ? LG * 8 : 4];
    const int lig = threadIdx.x % LG;
    const int gi = threadIdx.x / LG;
    int64_t chunk = (int64_t)blockIdx.x * GPB + gi;
    const bool group_on = chunk < chunks;                        // idle groups walk the last chunk, writing nothing
    if (!group_on) chunk = chunks - 1;
    const int c = blockIdx.y * LG + lig;                         // 16-byte piece of the row
    const bool lane_on = group_on && c < units;
    const int cc = c < units ? c : 0;
    const int64_t k0 = chunk * kChunk;
    const int64_t k1 = k0 + kChunk < m ? k0 + kChunk : m;
    const int cnt = (int)(k1 - k0);
    const int col = cc * N;

    {
        constexpr int PER = kChunk / LG;
        uint32_t key[PER], prev[PER], next[PER], val[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) {                          // all loads first, then the LDS writes
            const int64_t k = k0 + i * LG + lig;
            key[i] = k < k1 ? keys[k] : kNoKey;
            prev[i] = k > 0 ? keys[k - 1] : kNoKey;
            next[i] = k + 1 < m ? keys[k + 1] : kNoKey;
            val[i] = k < k1 ? vals[k] : 0u;                      // past the end: position 0, loaded but unused
        }
#pragma unroll
        for (int i = 0; i < PER; ++i) val[i] = val[i] < n ? val[i] : 0u;   // a position outside the batch reads row 0
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int e = i * LG + lig;
            const bool end = k0 + e + 1 >= k1 || next[i] != key[i];
            const bool single = k0 + e < k1 && prev[i] != key[i] && next[i] != key[i];
            s_key[gi][e] = key[i];
            s_val[gi][e] = single ? kSkip : (val[i] | (end ? kEndBit : 0u));
            if (e == kChunk - 1) s_key[gi][kChunk] = next[i];
        }
        if (lig < kPad) s_val[gi][kChunk + lig] = 0u;
    }
    bool piece_cont = k0 > 0 && keys[k0 - 1] == keys[k0];    // first piece continues the previous chunk's run
    int64_t u = (int64_t)runs_before(block_base, chunk_local, chunk, chunks) - 1;
    bool fresh = true;
    float acc[N];
    __syncthreads();

    const uint32_t* my_val = s_val[gi];
    const uint32_t* my_key = s_key[gi];
    const u32x4* my_grad = grad + cc;

    // 8 row loads, never predicated (a predicated load makes the compiler serialise the batch)
#define FS_ISSUE(X, PV, E0)                                                                  \
    _Pragma("unroll") for (int j = 0; j < U8; ++j) {                                         \
        PV[j] = my_val[(E0) + j];                                                            \
        X[j] = load_stream(my_grad + (int64_t)(PV[j] == kSkip ? 0u : PV[j] & ~kEndBit) * (EXACT ? LG : units)); \
    }
#define FS_CONSUME(X, PV, E0)                                                                \
    _Pragma("unroll") for (int j = 0; j < U8; ++j) {                                         \
        if ((E0) + j < cnt && PV[j] == kSkip) {                                              \
            ++u;                       /* a run of one: counted here, written elsewhere */   \
        } else if ((E0) + j < cnt) {                                                         \
            float f[N];                                                                      \
            Vec<DT>::load(X[j], f);                                                          \
            if (fresh) {                                                                     \
                if (!piece_cont) ++u;                                                        \
                _Pragma("unroll") for (int q = 0; q < N; ++q) acc[q] = f[q];                 \
            } else {                                                                         \
                _Pragma("unroll") for (int q = 0; q < N; ++q) acc[q] = acc[q] + f[q];        \
            }                                                                                \
            fresh = false;                                                                   \
            if (PV[j] & kEndBit) {                                                           \
                flush((E0) + j);                                                             \
                fresh = true;                                                                \
                piece_cont = false;                                                          \
            }                                                                                \
        }                                                                                    \
    }

    // The piece that ends at chunk-local index e goes out.  A lane holds N consecutive floats;
    // with N = 8 a direct store would be two instructions that each fill every other 16 bytes
    // of the row, so the group first transposes through LDS: afterwards lane i owns floats
    // [4i, 4i+4) of each half of the group's slab and both stores are fully coalesced.
    // The stores are non-temporal: the rows are not read again by this kernel (1.99 -> 1.74 ms
    // on 15.7M lookups of 512-byte rows).
    auto store_row = [&](float* row) {           // row = first float of the destination row
        if constexpr (N == 4) {
            if (lane_on) store_stream(reinterpret_cast<f32x4*>(row + col), f32x4{acc[0], acc[1], acc[2], acc[3]});
        } else {
            float* stage = s_stage[gi];
            *reinterpret_cast<f32x4*>(stage + lig * 8) = f32x4{acc[0], acc[1], acc[2], acc[3]};
            *reinterpret_cast<f32x4*>(stage + lig * 8 + 4) = f32x4{acc[4], acc[5], acc[6], acc[7]};
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const f32x4 lo = *reinterpret_cast<const f32x4*>(stage + lig * 4);
            const f32x4 hi = *reinterpret_cast<const f32x4*>(stage + LG * 4 + lig * 4);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            const int slab = blockIdx.y * LG * 8;
            const int col_lo = slab + lig * 4;
            const int col_hi = slab + LG * 4 + lig * 4;
            if (group_on && col_lo < D) store_stream(reinterpret_cast<f32x4*>(row + col_lo), lo);
            if (group_on && col_hi < D) store_stream(reinterpret_cast<f32x4*>(row + col_hi), hi);
        }
    };
    auto flush = [&](int e) {
        if (piece_cont && !atomic) {
            store_row(carry + chunk * D);
        } else if (u < cap) {
            float* dst = row_grads + u * D;
            const uint32_t key = my_key[e];
            const bool run_goes_on = my_key[e + 1] == key;       // also across the chunk end
            if (atomic && (piece_cont || run_goes_on)) {
                if (lane_on) {
#pragma unroll
                    for (int q = 0; q < N; ++q) unsafeAtomicAdd(dst + col + q, acc[q]);
                }
            } else {
                store_row(dst);
            }
            if (lane_on && !piece_cont && c == 0) {
                uniq_rows[u] = (int64_t)key;
                if (applied != nullptr) applied[u] = 0;          // this row's gradient is in row_grads
            }
        }
    };

    u32x4 xa[U8], xb[U8];
    uint32_t pa[U8], pb[U8];
    FS_ISSUE(xa, pa, 0)
#pragma unroll 1
    for (int e0 = 0; e0 < cnt; e0 += 2 * U8) {
        FS_ISSUE(xb, pb, e0 + U8)
        FS_CONSUME(xa, pa, e0)
        FS_ISSUE(xa, pa, e0 + 2 * U8)
        FS_CONSUME(xb, pb, e0 + U8)
    }
#undef FS_ISSUE
#undef FS_CONSUME
}

// Moves CNT * 64/LG listed singletons: the rows' loads first, then conversion and stores.  An index
// past the list repeats the last entry (same bytes to the same place), so nothing is predicated.
template <int CNT, int LG, int DT, bool EXACT>
__device__ __forceinline__ void singles_batch(
    const u32x4* __restrict__ grad, int units, int D, const uint32_t* s_pos, const uint32_t* s_run,
    const uint32_t* s_key, float* stage, uint32_t s, uint32_t singles, int c, bool all_fit, int64_t cap,
    int64_t* __restrict__ uniq_rows, float* __restrict__ row_grads)
{
    constexpr int N = Vec<DT>::N;
    constexpr int RPI = kWave / LG;
    const int g = lane_id() / LG;
    const bool lane_on = c < units;
    const int cc = lane_on ? c : 0;
    u32x4 x[CNT];
    uint32_t run[CNT];
    uint32_t at[CNT];
#pragma unroll
    for (int j = 0; j < CNT; ++j) {
        const uint32_t want = s + j * RPI + g;
        at[j] = want < singles ? want : singles - 1;
        run[j] = s_run[at[j]];
        x[j] = load_stream(grad + (int64_t)s_pos[at[j]] * (EXACT ? LG : units) + cc);
    }
    const int lig = lane_id() % LG;
#pragma unroll
    for (int j = 0; j < CNT; ++j) {
        const bool fits = all_fit || (int64_t)run[j] < cap;          // the same for the whole group
        float f[N];
        Vec<DT>::load(x[j], f);
        float* row = row_grads + (int64_t)run[j] * D;
        if constexpr (N == 4) {
            if (lane_on && fits) store_stream(reinterpret_cast<f32x4*>(row + cc * 4), f32x4{f[0], f[1], f[2], f[3]});
        } else {
            // 8 floats per lane: stored as they are, each 16-byte store would cover half of every
            // 32 bytes.  Through the wave's LDS slab lane i takes floats [4i, 4i+4) of each half of
            // the group's columns instead, and both stores are fully coalesced.
            float* gs = stage + g * LG * 8;
            *reinterpret_cast<f32x4*>(gs + lig * 8) = f32x4{f[0], f[1], f[2], f[3]};
            *reinterpret_cast<f32x4*>(gs + lig * 8 + 4) = f32x4{f[4], f[5], f[6], f[7]};
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const f32x4 lo = *reinterpret_cast<const f32x4*>(gs + lig * 4);
            const f32x4 hi = *reinterpret_cast<const f32x4*>(gs + LG * 4 + lig * 4);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            const int slab = (c - lig) * 8;                          // first column of the group's slab
            const int col_lo = slab + lig * 4;
            const int col_hi = slab + LG * 4 + lig * 4;
            if (fits && col_lo < D) store_stream(reinterpret_cast<f32x4*>(row + col_lo), lo);
            if (fits && col_hi < D) store_stream(reinterpret_cast<f32x4*>(row + col_hi), hi);
        }
        if (fits && c == 0) uniq_rows[run[j]] = (int64_t)s_key[at[j]];
    }
}

// The singletons of a wave's share of one chunk, listed in LDS (position, run index, row), in order.
// kSinglesSplit waves share a chunk: each reads all of its keys (run indices need the heads before
// it) but lists only the singletons of its own quarter.  Shorter-lived waves with less to move each
// are faster here, as for a plain copy: 1, 2, 4, 8 waves per chunk take 0.366, 0.340, 0.340, 0.389 ms
// on 15.7 M lookups and 2.63, 2.54, 2.50, 2.72 ms on 72 M.  Returns false (wave-uniform) if the wave
// has nothing to do; *runs_end = index after the last run that starts in the part of the chunk read so far.
__device__ __forceinline__ bool list_singletons(
    const uint32_t* __restrict__ keys, const uint32_t* __restrict__ vals, int64_t m, int64_t chunks, uint32_t n,
    const uint32_t* __restrict__ block_base, const uint32_t* __restrict__ chunk_local,
    uint32_t* s_pos, uint32_t* s_run, uint32_t* s_key, uint32_t* singles_out, uint32_t* runs_end)
{
    const int lane = lane_id();
    const int64_t wave_global = (int64_t)blockIdx.x * kWavesPerBlock + wave_id();
    const int64_t chunk = wave_global / kSinglesSplit;
    const int part = (int)(wave_global % kSinglesSplit);
    if (chunk >= chunks) return false;
    const int64_t k0 = chunk * kChunk;
    const int64_t k1 = k0 + kChunk < m ? k0 + kChunk : m;
    const uint32_t first_run = runs_before(block_base, chunk_local, chunk, chunks);

    uint32_t heads_before = 0, singles = 0;
#pragma unroll
    for (int q = 0; q < kChunk / kWave; ++q) {
        const int64_t k = k0 + q * kWave + lane;
        const bool valid = k < k1;
        const uint32_t key = valid ? keys[k] : kNoKey;
        const uint32_t prev = (valid && k > 0) ? keys[k - 1] : kNoKey;
        const uint32_t next = (valid && k + 1 < m) ? keys[k + 1] : kNoKey;
        const bool head = valid && key != prev;
        const bool single = head && key != next && q * kSinglesSplit / (kChunk / kWave) == part;
        const uint64_t hb = ballot(head);
        const uint64_t sb = ballot(single);
        if (single) {
            const uint32_t at = singles + (uint32_t)popc_below(sb);
            const uint32_t p = vals[k];
            s_pos[at] = p < n ? p : 0u;                          // a position outside the batch reads row 0
            s_run[at] = first_run + heads_before + (uint32_t)popc_below(hb);
            s_key[at] = key;
        }
        heads_before += (uint32_t)__popcll(hb);
        singles += (uint32_t)__popcll(sb);
    }
    *singles_out = singles;
    *runs_end = first_run + heads_before;
    if (singles == 0) return false;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    return true;
}

// The backward that applies the optimizer step itself, for rows looked up once: their gradient is the
// one converted row, so instead of writing it to row_grads (and an optimizer step reading it back) the
// wave updates the table row in place: gradient row in, table row in and out, 1.5 KB of traffic per
// 512-byte row where gradient-out-and-back-in costs 3.5 KB.  The arithmetic and the lane layout are those
// of fs_sparse_update's kernel (RowUpdate: lane i of a group holds quads i and LG + i of the row), which
// the gradient reaches through the same LDS transposition that the plain kernel uses for its stores; the
// new rows are therefore bit for bit what fs_seq_grad_bwd followed by fs_sparse_update writes.
// applied[u] = 1 tells the optimizer step that follows (for the rows summed from several lookups) to
// leave entry u alone.  Rows of up to 64 pieces.
template <int CNT, int LG, int DT, int OPT, bool EXACT>
__device__ __forceinline__ void singles_update_batch(
    const u32x4* __restrict__ grad, const UpdateArgs& a, const uint32_t* s_pos, const uint32_t* s_run,
    const uint32_t* s_key, float* stage, uint32_t s, uint32_t singles, int64_t cap,
    int64_t* __restrict__ uniq_rows, uint8_t* __restrict__ applied)
{
    constexpr int N = Vec<DT>::N;
    constexpr int P = N / 4;
    constexpr int RPI = kWave / LG;
    typedef typename Quad<DT>::type quad_t;
    const int g = lane_id() / LG;
    const int lig = lane_id() % LG;
    const int units = EXACT ? LG : a.units;
    const int64_t D = EXACT ? LG * N : a.D;
    const bool piece_on = lig < units;                               // the lane's 16-byte piece of the gradient row exists
    int col[P];
    bool on[P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int c = (p * LG + lig) * 4;
        on[p] = c < D;
        col[p] = on[p] ? c : 0;
    }
    const quad_t* wq = reinterpret_cast<const quad_t*>(a.weights);
    quad_t* wq_out = reinterpret_cast<quad_t*>(a.weights);
    quad_t* store_out = reinterpret_cast<quad_t*>(a.store);

    u32x4 x[CNT];
    quad_t wx[CNT][P];
    f32x4 sx[CNT][P];
    float srow[CNT];
    int64_t row[CNT];
    uint32_t run[CNT];
    bool ok[CNT];
    int slot[CNT];
#pragma unroll
    for (int j = 0; j < CNT; ++j) {
        const uint32_t want = s + j * RPI + g;
        const uint32_t at = want < singles ? want : singles - 1;     // past the list: the last entry again, not stored
        run[j] = s_run[at];
        const uint32_t key = s_key[at];
        ok[j] = want < singles && (int64_t)run[j] < cap && (int64_t)key < a.R;
        row[j] = (int64_t)key < a.R ? (int64_t)key : 0;
        x[j] = load_stream(grad + (int64_t)s_pos[at] * units + (piece_on ? lig : 0));
#pragma unroll
        for (int p = 0; p < P; ++p) {
            wx[j][p] = load_stream(wq + ((row[j] * D + col[p]) >> 2));
            if constexpr (OPT == FS_OPT_ADAGRAD)
                sx[j][p] = load_stream(reinterpret_cast<const f32x4*>(a.state + row[j] * D + col[p]));
        }
        if constexpr (OPT == FS_OPT_ADAGRAD_ROWWISE) srow[j] = a.state[row[j]];
        slot[j] = -1;
        if (a.store != nullptr) slot[j] = a.slot_of_row[row[j]];     // (wave-uniform branch: the load itself is not predicated)
    }
#pragma unroll
    for (int j = 0; j < CNT; ++j) {
        if (!ok[j]) slot[j] = -1;
        if (slot[j] >= a.k) { if (lig == 0) report(a.status, FS_DEV_BAD_ID); slot[j] = -1; }
    }
#pragma unroll
    for (int j = 0; j < CNT; ++j) {
        float f[N];
        Vec<DT>::load(x[j], f);
        f32x4 gx[P];
        if constexpr (N == 4) {
            gx[0] = f32x4{f[0], f[1], f[2], f[3]};                   // lane i holds quad i already
        } else {
            // 8 consecutive floats per lane -> quads i and LG + i, through the wave's LDS slab
            float* gs = stage + g * LG * 8;
            *reinterpret_cast<f32x4*>(gs + lig * 8) = f32x4{f[0], f[1], f[2], f[3]};
            *reinterpret_cast<f32x4*>(gs + lig * 8 + 4) = f32x4{f[4], f[5], f[6], f[7]};
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            gx[0] = *reinterpret_cast<const f32x4*>(gs + lig * 4);
            gx[1] = *reinterpret_cast<const f32x4*>(gs + LG * 4 + lig * 4);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        RowUpdate<LG, DT, OPT>::apply(wx[j], gx, sx[j], srow[j], on, col, row[j], D, lig, ok[j], slot[j], a.lr, a.eps,
                                      wq_out, store_out, a.state);
        const uint32_t want = s + j * RPI + g;
        if (want < singles && (int64_t)run[j] < cap && lig == 0) {
            uniq_rows[run[j]] = (int64_t)s_key[want];
            applied[run[j]] = 1;
        }
    }
}

template <int LG, int DT, int OPT, bool EXACT>
__global__ __launch_bounds__(kBlock) void bwd_singletons_update_kernel(
    const u32x4* __restrict__ grad, const UpdateArgs a,
    const uint32_t* __restrict__ keys, const uint32_t* __restrict__ vals, int64_t m, int64_t chunks, uint32_t n,
    const uint32_t* __restrict__ block_base, const uint32_t* __restrict__ chunk_local,
    int64_t* __restrict__ uniq_rows, int64_t cap, uint8_t* __restrict__ applied)
{
    constexpr int RPI = kWave / LG;
    constexpr int CNT = 2;                                           // rows a group keeps in flight (each brings a gradient row, a table
                                                                     // row and its state): 1 and 2 measure the same, 4 is 5 % and 8 is
                                                                     // 25 % slower on 15.7 M lookups of 512-byte rows
    __shared__ uint32_t s_pos[kWavesPerBlock][kChunk / kSinglesSplit];
    __shared__ uint32_t s_run[kWavesPerBlock][kChunk / kSinglesSplit];
    __shared__ uint32_t s_key[kWavesPerBlock][kChunk / kSinglesSplit];
    __shared__ __attribute__((aligned(16))) float s_stage[kWavesPerBlock][kWave * 8];
    const int w = wave_id();
    uint32_t singles, runs_end;
    if (!list_singletons(keys, vals, m, chunks, n, block_base, chunk_local, s_pos[w], s_run[w], s_key[w], &singles,
                         &runs_end))
        return;                                                      // wave-uniform; no block barrier below
    for (uint32_t s = 0; s < singles; s += CNT * RPI)
        singles_update_batch<CNT, LG, DT, OPT, EXACT>(grad, a, s_pos[w], s_run[w], s_key[w], s_stage[w], s, singles, cap,
                                                       uniq_rows, applied);
}

// Runs of one lookup need no sum: row_grads[u] = f32(grad_out[pos]).  They are most of the runs
// (the cold tail of the popularity distribution) and a store in the sequential walk above stalls
// the wave's later loads (loads and stores share one in-order counter), so this kernel converts
// them instead, fully parallel: a wave takes a quarter of a chunk, finds its singletons and their
// run indices with ballots, lists them in LDS and moves 64/LG rows per instruction, 8 in flight.
template <int LG, int DT, bool EXACT>
__global__ __launch_bounds__(kBlock) void bwd_singletons_kernel(
    const u32x4* __restrict__ grad, int units, int D,
    const uint32_t* __restrict__ keys, const uint32_t* __restrict__ vals, int64_t m, int64_t chunks, uint32_t n,
    const uint32_t* __restrict__ block_base, const uint32_t* __restrict__ chunk_local,
    int64_t* __restrict__ uniq_rows, float* __restrict__ row_grads, int64_t cap)
{
    constexpr int RPI = kWave / LG;
    constexpr int UNR = 8;
    __shared__ uint32_t s_pos[kWavesPerBlock][kChunk / kSinglesSplit];
    __shared__ uint32_t s_run[kWavesPerBlock][kChunk / kSinglesSplit];
    __shared__ uint32_t s_key[kWavesPerBlock][kChunk / kSinglesSplit];
    __shared__ __attribute__((aligned(16))) float s_stage[kWavesPerBlock][kWave * 8];   // store transposition, per wave
    const int w = wave_id();
    const int lane = lane_id();
    uint32_t singles, runs_end;
    if (!list_singletons(keys, vals, m, chunks, n, block_base, chunk_local, s_pos[w], s_run[w], s_key[w], &singles,
                         &runs_end))
        return;                                                  // wave-uniform; no block barrier below
    const int c = blockIdx.y * LG + lane % LG;
    const bool all_fit = (int64_t)runs_end <= cap;
    // Full batches of UNR instructions, then ONE batch of exactly as many instructions as the rest
    // needs: padding the last batch with repeats of the last row would write that row again and
    // again, and with ~18 singletons per chunk that is a third of the kernel's traffic.
    uint32_t s = 0;
    for (; s + UNR * RPI <= singles; s += UNR * RPI)
        singles_batch<UNR, LG, DT, EXACT>(grad, units, D, s_pos[w], s_run[w], s_key[w], s_stage[w], s, singles, c, all_fit,
                                          cap, uniq_rows, row_grads);
    if (s < singles) {
#define FS_TAIL(CNT) case CNT: singles_batch<CNT, LG, DT, EXACT>(grad, units, D, s_pos[w], s_run[w], s_key[w],    \
                                                                 s_stage[w], s, singles, c, all_fit, cap, uniq_rows, \
                                                                 row_grads); break
        switch ((singles - s + RPI - 1) / RPI) {
            FS_TAIL(1); FS_TAIL(2); FS_TAIL(3); FS_TAIL(4); FS_TAIL(5); FS_TAIL(6); FS_TAIL(7);
            default: singles_batch<UNR, LG, DT, EXACT>(grad, units, D, s_pos[w], s_run[w], s_key[w], s_stage[w], s,
                                                       singles, c, all_fit, cap, uniq_rows, row_grads);
        }
#undef FS_TAIL
    }
}

// One wave per chunk; a wave whose chunk starts a spilling run (one that goes on into the next
// chunk) adds the carries of the chunks the run goes on into, left to right.
__global__ __launch_bounds__(kBlock) void bwd_fold_kernel(
    const uint32_t* __restrict__ keys, int64_t m, int64_t chunks,
    const uint32_t* __restrict__ block_base, const uint32_t* __restrict__ chunk_local,
    float* __restrict__ row_grads, int D, int64_t cap, const float* __restrict__ carry)
{
    const int64_t chunk = (int64_t)blockIdx.x * kWavesPerBlock + wave_id();
    const int64_t k0 = chunk * kChunk;
    const int64_t k1 = k0 + kChunk;
    if (k1 >= m) return;                                             // nothing follows this chunk
    // Every index the decision needs, loaded in one round: a wave's time here is a chain of
    // dependent loads, and there are as many waves as chunks.
    const uint32_t key = keys[k1 - 1];
    const uint32_t next = keys[k1];
    const uint32_t head = keys[k0];
    const uint32_t before = k0 > 0 ? keys[k0 - 1] : kNoKey;
    const bool has_far = chunk + 2 < chunks;                         // then (chunk + 2) * kChunk < m
    const uint32_t far = keys[has_far ? k1 + kChunk : k1];
    const int64_t u = (int64_t)runs_before(block_base, chunk_local, chunk + 1, chunks) - 1;
    if (next != key) return;                                         // the chunk's last run ends with it
    if (head == key && before == key) return;                        // the run started in an earlier chunk
    if (u >= cap) return;
    // The last chunk whose first lookup still belongs to the run.  Most spilling runs end in the
    // very next chunk, so the search gallops from there (1, 2, 4 .. chunks ahead) and then bisects:
    // no further load for a short run instead of log2(m) dependent ones.
    int64_t lo = chunk + 1, step = 1;                                // chunk lo starts inside the run
    bool go_on = has_far && far == key;
    while (go_on) {
        lo += step;
        step <<= 1;
        go_on = lo + step < chunks && keys[(lo + step) * kChunk] == key;
    }
    int64_t hi = lo + step < chunks ? lo + step : chunks;            // chunk hi does not (or does not exist)
    while (hi - lo > 1) {
        const int64_t mid = lo + ((hi - lo) >> 1);
        if (keys[mid * kChunk] == key) lo = mid; else hi = mid;
    }
    const int64_t last_chunk = lo;
    constexpr int kAhead = 32;                   // carries in flight: the longest run's chain is latency-bound
    for (int col = lane_id() * 4; col < D; col += kWave * 4) {
        f32x4 acc = *reinterpret_cast<const f32x4*>(row_grads + u * D + col);
        int64_t cc = chunk + 1;
        for (; cc + kAhead <= last_chunk + 1; cc += kAhead) {
            f32x4 part[kAhead];
#pragma unroll
            for (int j = 0; j < kAhead; ++j)
                part[j] = *reinterpret_cast<const f32x4*>(carry + (cc + j) * D + col);
#pragma unroll
            for (int j = 0; j < kAhead; ++j) acc = acc + part[j];
        }
        for (; cc <= last_chunk; ++cc) acc = acc + *reinterpret_cast<const f32x4*>(carry + cc * D + col);
        *reinterpret_cast<f32x4*>(row_grads + u * D + col) = acc;
    }
}

// variant 1: rows that receive atomic adds start at zero.
__global__ __launch_bounds__(kBlock) void bwd_zero_spilled_kernel(
    const uint32_t* __restrict__ keys, int64_t m, int64_t chunks,
    const uint32_t* __restrict__ block_base, const uint32_t* __restrict__ chunk_local,
    float* __restrict__ row_grads, int D, int64_t cap)
{
    const int64_t chunk = (int64_t)blockIdx.x * kWavesPerBlock + wave_id();
    if (chunk >= chunks || chunk == 0) return;
    const int64_t k0 = chunk * kChunk;
    if (keys[k0 - 1] != keys[k0]) return;
    const int64_t u = (int64_t)runs_before(block_base, chunk_local, chunk, chunks) - 1;
    if (u >= cap) return;
    for (int col = lane_id() * 4; col < D; col += kWave * 4)
        *reinterpret_cast<f32x4*>(row_grads + u * D + col) = f32x4{0.f, 0.f, 0.f, 0.f};
}

__global__ void bwd_empty_kernel(int64_t* num_unique) { *num_unique = 0; }

template <int LG>
static fs_status launch_segreduce(fs_dtype dtype, const void* grad, int units, int D, const uint32_t* keys,
                                  const uint32_t* vals, int64_t m, int64_t chunks, uint32_t n, const uint32_t* block_base,
                                  const uint32_t* chunk_local, int64_t* uniq_rows, float* row_grads, int64_t cap,
                                  float* carry, int atomic, uint8_t* applied, hipStream_t stream)
{
    constexpr int GPB = kBlock / LG;
    const dim3 grid((unsigned)((chunks + GPB - 1) / GPB), (unsigned)((units + LG - 1) / LG));
    const u32x4* g = static_cast<const u32x4*>(grad);
#define FS_SEG_LAUNCH(DT, EX)                                                                                      \
    FS_LAUNCH("bwd_segreduce", (bwd_segreduce_kernel<LG, DT, EX>), grid, dim3(kBlock), stream, g, units, D, keys, vals, \
              m, chunks, n, block_base, chunk_local, uniq_rows, row_grads, cap, carry, atomic, applied)
    const bool exact = units == LG;
    if (dtype == FS_F32) { if (exact) FS_SEG_LAUNCH(FS_F32, true); else FS_SEG_LAUNCH(FS_F32, false); }
    else if (dtype == FS_F16) { if (exact) FS_SEG_LAUNCH(FS_F16, true); else FS_SEG_LAUNCH(FS_F16, false); }
    else { if (exact) FS_SEG_LAUNCH(FS_BF16, true); else FS_SEG_LAUNCH(FS_BF16, false); }
#undef FS_SEG_LAUNCH
    return FS_OK;
}

template <int LG>
static fs_status launch_singletons(fs_dtype dtype, const void* grad, int units, int D, const uint32_t* keys,
                                   const uint32_t* vals, int64_t m, int64_t chunks, uint32_t n, const uint32_t* block_base,
                                   const uint32_t* chunk_local, int64_t* uniq_rows, float* row_grads, int64_t cap,
                                   hipStream_t stream)
{
    const int64_t waves = chunks * kSinglesSplit;
    if ((waves + kWavesPerBlock - 1) / kWavesPerBlock > 0x7FFFFFFF) return FS_ERR_SIZE;
    const dim3 grid((unsigned)((waves + kWavesPerBlock - 1) / kWavesPerBlock), (unsigned)((units + LG - 1) / LG));
    const u32x4* g = static_cast<const u32x4*>(grad);
#define FS_SINGLE_LAUNCH(DT, EX)                                                                                   \
    FS_LAUNCH("bwd_singletons", (bwd_singletons_kernel<LG, DT, EX>), grid, dim3(kBlock), stream, g, units, D, keys,     \
              vals, m, chunks, n, block_base, chunk_local, uniq_rows, row_grads, cap)
    const bool exact = units == LG && LG >= 16;
    if (dtype == FS_F32) { if (exact) FS_SINGLE_LAUNCH(FS_F32, (LG >= 16)); else FS_SINGLE_LAUNCH(FS_F32, false); }
    else if (dtype == FS_F16) { if (exact) FS_SINGLE_LAUNCH(FS_F16, (LG >= 16)); else FS_SINGLE_LAUNCH(FS_F16, false); }
    else { if (exact) FS_SINGLE_LAUNCH(FS_BF16, (LG >= 16)); else FS_SINGLE_LAUNCH(FS_BF16, false); }
#undef FS_SINGLE_LAUNCH
    return FS_OK;
}

// fs_seq_grad_bwd_update's kernel for the rows looked up once (rows of up to 64 pieces).
template <int LG, int DT>
static fs_status launch_singletons_update_opt(int optimizer, const void* grad, const UpdateArgs& a, const uint32_t* keys,
                                              const uint32_t* vals, int64_t m, int64_t chunks, uint32_t n,
                                              const uint32_t* block_base, const uint32_t* chunk_local, int64_t* uniq_rows,
                                              int64_t cap, uint8_t* applied, hipStream_t stream)
{
    const int64_t waves = chunks * kSinglesSplit;
    if ((waves + kWavesPerBlock - 1) / kWavesPerBlock > 0x7FFFFFFF) return FS_ERR_SIZE;
    const dim3 grid((unsigned)((waves + kWavesPerBlock - 1) / kWavesPerBlock));
    const u32x4* g = static_cast<const u32x4*>(grad);
#define FS_SU_LAUNCH(OPT, EX)                                                                                      \
    FS_LAUNCH("bwd_singletons_update", (bwd_singletons_update_kernel<LG, DT, OPT, EX>), grid, dim3(kBlock), stream, g, a, \
              keys, vals, m, chunks, n, block_base, chunk_local, uniq_rows, cap, applied)
    const bool exact = a.units == LG;
    if (optimizer == FS_OPT_SGD) { if (exact) FS_SU_LAUNCH(FS_OPT_SGD, true); else FS_SU_LAUNCH(FS_OPT_SGD, false); }
    else if (optimizer == FS_OPT_ADAGRAD) { if (exact) FS_SU_LAUNCH(FS_OPT_ADAGRAD, true); else FS_SU_LAUNCH(FS_OPT_ADAGRAD, false); }
    else { if (exact) FS_SU_LAUNCH(FS_OPT_ADAGRAD_ROWWISE, true); else FS_SU_LAUNCH(FS_OPT_ADAGRAD_ROWWISE, false); }
#undef FS_SU_LAUNCH
    return FS_OK;
}

template <int LG>
static fs_status launch_singletons_update(fs_dtype dtype, int optimizer, const void* grad, const UpdateArgs& a,
                                          const uint32_t* keys, const uint32_t* vals, int64_t m, int64_t chunks, uint32_t n,
                                          const uint32_t* block_base, const uint32_t* chunk_local, int64_t* uniq_rows,
                                          int64_t cap, uint8_t* applied, hipStream_t stream)
{
    if (dtype == FS_F32)
        return launch_singletons_update_opt<LG, FS_F32>(optimizer, grad, a, keys, vals, m, chunks, n, block_base, chunk_local,
                                                        uniq_rows, cap, applied, stream);
    if (dtype == FS_F16)
        return launch_singletons_update_opt<LG, FS_F16>(optimizer, grad, a, keys, vals, m, chunks, n, block_base, chunk_local,
                                                        uniq_rows, cap, applied, stream);
    return launch_singletons_update_opt<LG, FS_BF16>(optimizer, grad, a, keys, vals, m, chunks, n, block_base, chunk_local,
                                                     uniq_rows, cap, applied, stream);
}

// Everything after the sort: (keys, vals) are the lookups in (row, position) order.
struct BwdScratch {
    uint32_t* chunk_local;
    uint32_t* block_base;
    float* carry;
};

static fs_status bwd_after_sort(const void* grad_out, int64_t n, int D, fs_dtype dtype, int units,
                                const uint32_t* keys, const uint32_t* vals, int64_t m, int64_t R, int variant,
                                int64_t* uniq_rows, float* row_grads, int64_t cap_unique, int64_t* num_unique,
                                const BwdScratch& w, hipStream_t s, int32_t* dev_status,
                                const UpdateArgs* update = nullptr, int optimizer = 0, uint8_t* applied = nullptr)
{
    const int64_t chunks = (m + kChunk - 1) / kChunk;
    const int64_t blocks = (chunks + kChunksPerBlock - 1) / kChunksPerBlock;
    FS_LAUNCH("bwd_count_heads", bwd_count_heads_kernel, dim3((unsigned)blocks), dim3(kHeadsBlock), s,
              keys, vals, m, chunks, (uint32_t)n, (uint32_t)R, w.chunk_local, w.block_base, dev_status);
    FS_LAUNCH("bwd_scan_blocks", bwd_scan_blocks_kernel, dim3(1), dim3(kScanBlock), s,
              w.block_base, blocks, cap_unique, num_unique, dev_status);
    const unsigned wave_grid = (unsigned)((chunks + kWavesPerBlock - 1) / kWavesPerBlock);
    if (variant == 1)
        FS_LAUNCH("bwd_zero_spilled", bwd_zero_spilled_kernel, dim3(wave_grid), dim3(kBlock), s,
                  keys, m, chunks, w.block_base, w.chunk_local, row_grads, D, cap_unique);
    fs_status rc;
#define FS_SEG(LG)                                                                                              \
    rc = launch_segreduce<LG>(dtype, grad_out, units, D, keys, vals, m, chunks, (uint32_t)n, w.block_base,        \
                              w.chunk_local, uniq_rows, row_grads, cap_unique, w.carry, variant, applied, s)
    if (units <= 16) FS_SEG(16);            // rows under 256 bytes leave lanes of the group idle
    else if (units <= 32) FS_SEG(32);
    else FS_SEG(64);
#undef FS_SEG
    if (rc != FS_OK) return rc;
    if (update != nullptr) {                     // rows looked up once are updated in place, the others flagged for the step below
#define FS_SINGLE_UPDATE(LG)                                                                                    \
    rc = launch_singletons_update<LG>(dtype, optimizer, grad_out, *update, keys, vals, m, chunks, (uint32_t)n,    \
                                      w.block_base, w.chunk_local, uniq_rows, cap_unique, applied, s)
        if (units <= 1) FS_SINGLE_UPDATE(1);         // the group sizes of fs_sparse_update: the row-wise rule's sum of
        else if (units <= 2) FS_SINGLE_UPDATE(2);    // squares is taken over the group, and both must round alike
        else if (units <= 4) FS_SINGLE_UPDATE(4);
        else if (units <= 8) FS_SINGLE_UPDATE(8);
        else if (units <= 16) FS_SINGLE_UPDATE(16);
        else if (units <= 32) FS_SINGLE_UPDATE(32);
        else FS_SINGLE_UPDATE(64);
#undef FS_SINGLE_UPDATE
        if (rc != FS_OK) return rc;
        FS_LAUNCH("bwd_fold", bwd_fold_kernel, dim3(wave_grid), dim3(kBlock), s,
                  keys, m, chunks, w.block_base, w.chunk_local, row_grads, D, cap_unique, w.carry);
        UpdateArgs rest = *update;               // the optimizer step on the rows whose gradient is in row_grads
        rest.uniq_rows = uniq_rows; rest.row_grads = row_grads; rest.cap = cap_unique; rest.num_unique = num_unique;
        rest.skip = applied;
        return sparse_update_launch(rest, dtype, optimizer, s);
    }
#define FS_SINGLE(LG)                                                                                           \
    rc = launch_singletons<LG>(dtype, grad_out, units, D, keys, vals, m, chunks, (uint32_t)n, w.block_base,       \
                               w.chunk_local, uniq_rows, row_grads, cap_unique, s)
    if (units <= 1) FS_SINGLE(1);
    else if (units <= 2) FS_SINGLE(2);
    else if (units <= 4) FS_SINGLE(4);
    else if (units <= 8) FS_SINGLE(8);
    else if (units <= 16) FS_SINGLE(16);
    else if (units <= 32) FS_SINGLE(32);
    else FS_SINGLE(64);
#undef FS_SINGLE
    if (rc != FS_OK) return rc;
    if (variant == 0)
        FS_LAUNCH("bwd_fold", bwd_fold_kernel, dim3(wave_grid), dim3(kBlock), s,
                  keys, m, chunks, w.block_base, w.chunk_local, row_grads, D, cap_unique, w.carry);
    return FS_OK;
}

static BwdScratch take_bwd_scratch(Carver& ws, int64_t m, int D, int variant)
{
    const int64_t chunks = (m + kChunk - 1) / kChunk;
    const int64_t blocks = (chunks + kChunksPerBlock - 1) / kChunksPerBlock;
    BwdScratch w;
    w.chunk_local = ws.take<uint32_t>((size_t)chunks);
    w.block_base = ws.take<uint32_t>((size_t)blocks + 1);
    w.carry = ws.take<float>(variant == 0 ? (size_t)chunks * (size_t)D : 0);
    return w;
}

}  // namespace fs

extern "C" fs_status fs_seq_grad_bwd(
    const void* grad_out, int64_t n, int32_t D, fs_dtype dtype,
    const int64_t* rows, const int32_t* pos, int64_t j0, int64_t j1, int64_t R,
    int32_t variant,
    int64_t* uniq_rows, float* row_grads, int64_t cap_unique, int64_t* num_unique,
    void* workspace, size_t* workspace_bytes, void* stream, int32_t* dev_status)
{
    using namespace fs;
    if (!workspace_bytes) return FS_ERR_NULL;
    const int es = dtype_bytes(dtype);
    if (es == 0) return FS_ERR_DTYPE;
    if (R < 1 || R >= 4294967295LL || n < 0 || n >= (1LL << 31) || D < 1 || j0 < 0 || j0 > j1 || cap_unique < 0)
        return FS_ERR_SIZE;
    if (variant != 0 && variant != 1) return FS_ERR_CONFIG;
    const int64_t row_bytes = (int64_t)D * es;
    if (row_bytes % 16 != 0) return FS_ERR_ALIGN;
    const int64_t m = j1 - j0;
    if (m >= (1LL << 31)) return FS_ERR_SIZE;
    const int units = (int)(row_bytes / 16);

    Carver ws(workspace);
    uint32_t* keys_a = ws.take<uint32_t>((size_t)m);
    uint32_t* vals_a = ws.take<uint32_t>((size_t)m);
    uint32_t* keys_b = ws.take<uint32_t>((size_t)m);
    uint32_t* vals_b = ws.take<uint32_t>((size_t)m);
    char* sort_scratch = ws.take<char>(radix_sort_scratch_bytes(m));
    const BwdScratch scratch = take_bwd_scratch(ws, m, (int)D, (int)variant);
    if (!workspace) { *workspace_bytes = ws.used; return FS_OK; }
    if (*workspace_bytes < ws.used || (reinterpret_cast<uintptr_t>(workspace) & 255)) return FS_ERR_WORKSPACE;
    if (!num_unique) return FS_ERR_NULL;

    hipStream_t s = static_cast<hipStream_t>(stream);
    if (m == 0) {
        FS_LAUNCH("bwd_empty", bwd_empty_kernel, dim3(1), dim3(1), s, num_unique);
        return FS_OK;
    }
    if (!grad_out || !rows || !pos) return FS_ERR_NULL;
    if (cap_unique > 0 && (!uniq_rows || !row_grads)) return FS_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(grad_out) | reinterpret_cast<uintptr_t>(row_grads)) & 15) return FS_ERR_ALIGN;

    uint32_t* keys = nullptr;
    uint32_t* vals = nullptr;
    SortSource source;                           // the sort's first pass reads (row, pos) itself
    source.rows = rows + j0;
    source.pos = pos + j0;
    source.R = R;
    source.n = n;
    source.status = dev_status;
    fs_status rc = radix_sort_pairs(keys_a, vals_a, keys_b, vals_b, m, nullptr, bits_for((uint64_t)(R - 1)),
                                    sort_scratch, s, &keys, &vals, source);
    if (rc != FS_OK) return rc;
    return bwd_after_sort(grad_out, n, (int)D, dtype, units, keys, vals, m, R, (int)variant, uniq_rows, row_grads,
                          cap_unique, num_unique, scratch, s, dev_status);
}

extern "C" fs_status fs_sort_lookups(
    const int64_t* rows, const int32_t* pos, int64_t j0, int64_t j1, int64_t R, int64_t n,
    uint32_t* sorted_rows, uint32_t* sorted_pos,
    void* workspace, size_t* workspace_bytes, void* stream, int32_t* dev_status)
{
    using namespace fs;
    if (!workspace_bytes) return FS_ERR_NULL;
    if (R < 1 || R >= 4294967295LL || n < 0 || n >= (1LL << 31) || j0 < 0 || j0 > j1) return FS_ERR_SIZE;
    const int64_t m = j1 - j0;
    if (m >= (1LL << 31)) return FS_ERR_SIZE;
    Carver ws(workspace);
    uint32_t* keys_w = ws.take<uint32_t>((size_t)m);
    uint32_t* vals_w = ws.take<uint32_t>((size_t)m);
    char* sort_scratch = ws.take<char>(radix_sort_scratch_bytes(m));
    if (!workspace) { *workspace_bytes = ws.used; return FS_OK; }
    if (*workspace_bytes < ws.used || (reinterpret_cast<uintptr_t>(workspace) & 255)) return FS_ERR_WORKSPACE;
    if (m == 0) return FS_OK;
    if (!rows || !pos || !sorted_rows || !sorted_pos) return FS_ERR_NULL;
    // The first pass reads (rows, pos) and writes buffer A, later passes alternate A -> B -> A: with an odd
    // number of passes the result lands in A, with an even number in B.  The caller's arrays take that role.
    const int key_bits = bits_for((uint64_t)(R - 1));
    const int passes = radix_sort_passes(key_bits);
    uint32_t* keys_a = (passes & 1) ? sorted_rows : keys_w;
    uint32_t* vals_a = (passes & 1) ? sorted_pos : vals_w;
    uint32_t* keys_b = (passes & 1) ? keys_w : sorted_rows;
    uint32_t* vals_b = (passes & 1) ? vals_w : sorted_pos;
    SortSource source;
    source.rows = rows + j0;
    source.pos = pos + j0;
    source.R = R;
    source.n = n;
    source.status = dev_status;
    uint32_t* keys = nullptr;
    uint32_t* vals = nullptr;
    const fs_status rc = radix_sort_pairs(keys_a, vals_a, keys_b, vals_b, m, nullptr, key_bits, sort_scratch,
                                          static_cast<hipStream_t>(stream), &keys, &vals, source);
    if (rc != FS_OK) return rc;
    if (keys != sorted_rows || vals != sorted_pos) return FS_ERR_DEVICE;     // cannot happen: see above
    return FS_OK;
}

extern "C" fs_status fs_seq_grad_bwd_sorted(
    const void* grad_out, int64_t n, int32_t D, fs_dtype dtype,
    const uint32_t* sorted_rows, const uint32_t* sorted_pos, int64_t m, int64_t R,
    int32_t variant,
    int64_t* uniq_rows, float* row_grads, int64_t cap_unique, int64_t* num_unique,
    void* workspace, size_t* workspace_bytes, void* stream, int32_t* dev_status)
{
    using namespace fs;
    if (!workspace_bytes) return FS_ERR_NULL;
    const int es = dtype_bytes(dtype);
    if (es == 0) return FS_ERR_DTYPE;
    if (R < 1 || R >= 4294967295LL || n < 0 || n >= (1LL << 31) || D < 1 || m < 0 || m >= (1LL << 31) || cap_unique < 0)
        return FS_ERR_SIZE;
    if (variant != 0 && variant != 1) return FS_ERR_CONFIG;
    const int64_t row_bytes = (int64_t)D * es;
    if (row_bytes % 16 != 0) return FS_ERR_ALIGN;
    const int units = (int)(row_bytes / 16);
    Carver ws(workspace);
    const BwdScratch scratch = take_bwd_scratch(ws, m, (int)D, (int)variant);
    if (!workspace) { *workspace_bytes = ws.used; return FS_OK; }
    if (*workspace_bytes < ws.used || (reinterpret_cast<uintptr_t>(workspace) & 255)) return FS_ERR_WORKSPACE;
    if (!num_unique) return FS_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (m == 0) {
        FS_LAUNCH("bwd_empty", bwd_empty_kernel, dim3(1), dim3(1), s, num_unique);
        return FS_OK;
    }
    if (!grad_out || !sorted_rows || !sorted_pos) return FS_ERR_NULL;
    if (cap_unique > 0 && (!uniq_rows || !row_grads)) return FS_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(grad_out) | reinterpret_cast<uintptr_t>(row_grads)) & 15) return FS_ERR_ALIGN;
    return bwd_after_sort(grad_out, n, (int)D, dtype, units, sorted_rows, sorted_pos, m, R, (int)variant, uniq_rows,
                          row_grads, cap_unique, num_unique, scratch, s, dev_status);
}

extern "C" fs_status fs_seq_grad_bwd_update(
    const void* grad_out, int64_t n, int32_t D, fs_dtype dtype,
    const uint32_t* sorted_rows, const uint32_t* sorted_pos, int64_t m, int64_t R,
    void* weights, int32_t optimizer, float lr, float eps, float* state,
    void* store, const int32_t* slot_of_row, int64_t k,
    int64_t* uniq_rows, float* row_grads, int64_t cap_unique, int64_t* num_unique,
    void* workspace, size_t* workspace_bytes, void* stream, int32_t* dev_status)
{
    using namespace fs;
    if (!workspace_bytes) return FS_ERR_NULL;
    const int es = dtype_bytes(dtype);
    if (es == 0) return FS_ERR_DTYPE;
    if (R < 1 || R >= 4294967295LL || n < 0 || n >= (1LL << 31) || D < 1 || m < 0 || m >= (1LL << 31) || cap_unique < 0 ||
        k < 0 || k >= (1LL << 31))
        return FS_ERR_SIZE;
    if (optimizer != FS_OPT_SGD && optimizer != FS_OPT_ADAGRAD && optimizer != FS_OPT_ADAGRAD_ROWWISE) return FS_ERR_CONFIG;
    const int64_t row_bytes = (int64_t)D * es;
    if (row_bytes % 16 != 0) return FS_ERR_ALIGN;
    const int units = (int)(row_bytes / 16);
    Carver ws(workspace);
    const BwdScratch scratch = take_bwd_scratch(ws, m, (int)D, 0);
    uint8_t* applied = ws.take<uint8_t>((size_t)cap_unique);
    if (!workspace) { *workspace_bytes = ws.used; return FS_OK; }
    if (*workspace_bytes < ws.used || (reinterpret_cast<uintptr_t>(workspace) & 255)) return FS_ERR_WORKSPACE;
    if (!num_unique || !weights) return FS_ERR_NULL;
    if (optimizer != FS_OPT_SGD && !state) return FS_ERR_NULL;
    if ((store != nullptr) != (slot_of_row != nullptr)) return FS_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (m == 0) {
        FS_LAUNCH("bwd_empty", bwd_empty_kernel, dim3(1), dim3(1), s, num_unique);
        return FS_OK;
    }
    if (!grad_out || !sorted_rows || !sorted_pos) return FS_ERR_NULL;
    if (cap_unique > 0 && (!uniq_rows || !row_grads)) return FS_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(grad_out) | reinterpret_cast<uintptr_t>(row_grads) | reinterpret_cast<uintptr_t>(weights) |
         reinterpret_cast<uintptr_t>(store) | reinterpret_cast<uintptr_t>(state)) & 15)
        return FS_ERR_ALIGN;
    UpdateArgs a;
    a.weights = static_cast<u32x4*>(weights); a.R = R; a.units = units; a.D = D;
    a.uniq_rows = uniq_rows; a.row_grads = row_grads; a.cap = cap_unique; a.num_unique = num_unique;
    a.lr = lr; a.eps = eps; a.state = state;
    a.store = static_cast<u32x4*>(store); a.slot_of_row = slot_of_row; a.k = k; a.status = dev_status;
    a.skip = nullptr;
    if (units > kWave || cap_unique == 0) {
        // rows of more than 64 pieces (or no room for any row): the two steps one after the other
        const fs_status rc = bwd_after_sort(grad_out, n, (int)D, dtype, units, sorted_rows, sorted_pos, m, R, 0, uniq_rows,
                                            row_grads, cap_unique, num_unique, scratch, s, dev_status);
        if (rc != FS_OK || cap_unique == 0) return rc;
        return sparse_update_launch(a, dtype, optimizer, s);
    }
    return bwd_after_sort(grad_out, n, (int)D, dtype, units, sorted_rows, sorted_pos, m, R, 0, uniq_rows, row_grads,
                          cap_unique, num_unique, scratch, s, dev_status, &a, optimizer, applied);
}
