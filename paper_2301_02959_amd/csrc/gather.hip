// fs_seq_gather_fwd: out[pos[j], :] = weights[rows[j], :] for j in [j0, j1), and its relatives
// fs_seq_gather_send, fs_replica_build and fs_seq_gather_fwd_replica, which run the same kernel
// with the position replaced by j itself or with a second row source; fs_seq_unbucketize, whose row
// loads do not wait for an index, has a kernel of its own.
//
// HBM-bound bit copy.  A wave owns 64 consecutive lookups: it fetches their 64 row
// indices and 64 positions with ONE coalesced load each (a per-row index load in
// front of every row costs a third of the bandwidth: the store cannot issue before
// its index has come back from HBM), then hands them to the lanes with
// ds_bpermute.  A row of `units` 16-byte pieces is moved by a group of LG lanes
// (LG = the power of two >= units, at most 64), one 128-bit load and one 128-bit
// non-temporal store per lane, so a wave moves 64/LG rows per instruction and keeps
// UNR instructions in flight.  Table reads stay cacheable (popular rows are re-read
// from L2 / Infinity Cache), the output is streamed past the caches.
// Blocks take tiles in stripes per XCD (see xcd_striped_tile): an XCD's consecutive
// blocks write consecutive pieces of the output, and the cold, other-bucket tail of the
// j range is still spread over all XCDs (one contiguous eighth of j per XCD would leave
// the last XCD with all the cache misses).
#include "fs_common.h"

namespace fs {

constexpr int kGatherRowsPerWave = kWave;
constexpr int kGatherRowsPerBlock = kGatherRowsPerWave * kWavesPerBlock;

template <int LG>
struct GatherShape {
    static constexpr int RPI = kWave / LG;                                   // rows per instruction
    static constexpr int UNR = RPI >= 8 ? kWave / RPI : (LG == 16 ? 8 : 16); // instructions in flight (256-byte rows with 16:
                                                                             // 9 % slower on 4 M lookups, 5 % faster on 8 M)
};

// Moves the wave's 64 rows.  GUARD = false: every lookup of the wave is valid, loads and
// stores carry no per-lane predicate (a predicated load makes the compiler wait for each
// load before it issues the next, which serialises the 16 loads of a batch).
// EXACT: the row is exactly LG pieces long (power-of-two row sizes), so there is no loop over
// pieces and no idle lane.
template <int LG, bool GUARD, bool EXACT>
__device__ __forceinline__ void gather_wave(int units, u32x4* __restrict__ out,
                                            const u32x4* my_src, int32_t my_pos, int my_ok)
{
    constexpr int RPI = GatherShape<LG>::RPI;
    constexpr int UNR = GatherShape<LG>::UNR;
    const int lane = lane_id();
    const int g = lane / LG;
    const int lig = lane % LG;
#pragma unroll 1
    for (int s = 0; s < kGatherRowsPerWave; s += UNR * RPI) {
        const u32x4* src[UNR];
        int64_t dst[UNR];
        bool ok[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int from = s + u * RPI + g;            // lane that holds this row's indices
            src[u] = reinterpret_cast<const u32x4*>(__shfl((int64_t) reinterpret_cast<uintptr_t>(my_src), from));
            const int32_t p = __shfl(my_pos, from);
            ok[u] = GUARD ? __shfl(my_ok, from) != 0 : true;
            dst[u] = EXACT ? (int64_t)p * LG : (int64_t)p * units;
        }
        if (EXACT) {
            u32x4 v[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) v[u] = src[u][lig];               // invalid lookups read row 0
#pragma unroll
            for (int u = 0; u < UNR; ++u)
                if (!GUARD || ok[u]) store_stream(out + dst[u] + lig, v[u]);
        } else {
            for (int c = lig; c < units; c += LG) {
                u32x4 v[UNR];
#pragma unroll
                for (int u = 0; u < UNR; ++u) v[u] = src[u][c];
#pragma unroll
                for (int u = 0; u < UNR; ++u)
                    if (!GUARD || ok[u]) store_stream(out + dst[u] + c, v[u]);
            }
        }
    }
}

// Which of the two index arrays a launch reads.
//   kBoth:     out[pos[j]]  = weights[rows[j]]     (fs_seq_gather_fwd)
//   kToSend:   out[j]       = weights[rows[j]]     (fs_seq_gather_send, fs_replica_build)
//   (fs_seq_unbucketize, out[pos[j]] = recv[j], has a kernel of its own further down)
//   kReplica:  as kBoth, but a row with slot_of_row[row] >= 0 is read from store[slot]
//   kSorted:   as kBoth with the lookups as 32-bit (row, position) pairs (fs_seq_gather_fwd_sorted)
//   kSlots:    as kReplica with the slot of lookup j given in slots[j], read beside its row and position
//              (fs_seq_gather_fwd_slots): no load of the slot map in front of the row's
enum GatherMode { kBoth = 0, kToSend = 1, kReplica = 3, kSorted = 4, kSlots = 5 };

struct GatherArgs {
    const u32x4* weights;
    int64_t R;
    int units;
    const int64_t* rows;
    const uint32_t* rows32;          // kSorted only (then rows is unused)
    const int32_t* pos;
    int64_t m;
    const int64_t* m_dev;            // if set, only the first min(m, *m_dev) lookups are moved
    u32x4* out;
    int64_t n;
    int32_t* status;
    int stripe;                      // workgroups per XCD stripe (1: tiles in launch order)
    const u32x4* store;              // kReplica and kSlots
    const int32_t* slot_of_row;      // kReplica: [R]
    const int32_t* slots;            // kSlots: [m], one per lookup
    int64_t k;
};

// Workgroups are dealt to the 8 XCDs round-robin (workgroup b runs on XCD b % 8).  Taking tile b in
// that order makes every XCD write every eighth 128 KB piece of the output; letting an XCD's
// consecutive workgroups take consecutive tiles instead, in stripes of kXcdStripe tiles (4 MB of
// 512-byte rows), raises the write rate of this store pattern from 5.65 to 6.45 TB/s (a fill in the
// gather's shape; stripes of 8 or 16 tiles gain half of that, one contiguous eighth per XCD as much
// as the stripes).  The gather itself gains 5 % on 15.7 M lookups of 512-byte rows that are mostly
// cache hits (1.62 -> 1.54 ms, stripes of 32 or 64 tiles; 128: 2 %), 3-5 % on 256-byte rows under
// heavier skew, nothing on a mid-size batch, and loses 1 % where cold reads dominate (72 M lookups
// over 164 GB).  Stripes rather than eighths, because the j order is bucket-major: its tail, the other
// buckets' cold rows, would otherwise all land on the last XCD.
constexpr int kXcdStripe = 32;

template <int LG, bool EXACT, int MODE>
__global__ __launch_bounds__(kBlock) void gather_rows_kernel(const GatherArgs a)
{
    const int lane = lane_id();
    const int64_t wbase = (xcd_striped_tile(blockIdx.x, a.stripe) * kWavesPerBlock + wave_id()) * kGatherRowsPerWave;
    int64_t m = a.m;
    if (a.m_dev) { const int64_t md = *a.m_dev; m = md < m ? (md < 0 ? 0 : md) : m; }
    if (wbase >= m) return;                              // wave-uniform

    // one coalesced load of the wave's 64 (row, position) pairs
    const int64_t jj = wbase + lane;
    int64_t my_row = 0;
    int32_t my_pos = 0;
    int my_ok = 0;
    if (jj < m) {
        my_row = MODE == kSorted ? (int64_t)load_stream(a.rows32 + jj) : load_stream(a.rows + jj);
        my_pos = MODE == kToSend ? (int32_t)jj : load_stream(a.pos + jj);
        // unsigned compares: one test each also catches the negative values (n < 2^31)
        my_ok = ((uint64_t)my_row < (uint64_t)a.R && (uint32_t)my_pos < (uint32_t)a.n) ? 1 : 0;
        if (!my_ok) { report(a.status, FS_DEV_BAD_ID); my_row = 0; my_pos = 0; }
    }
    int32_t my_slot = -1;
    if (MODE == kSlots && jj < m) my_slot = load_stream(a.slots + jj);
    const int64_t stride = EXACT ? LG : a.units;
    const u32x4* my_src = a.weights + my_row * stride;
    if (MODE == kSlots && my_ok && my_slot >= 0) {
        if (my_slot < a.k) my_src = a.store + (int64_t)my_slot * stride;
        else { report(a.status, FS_DEV_BAD_ID); my_ok = 0; my_src = a.weights; my_pos = 0; }
    }
    if (MODE == kReplica && my_ok) {
        const int32_t slot = a.slot_of_row[my_row];      // cacheable: popular rows repeat
        if (slot >= 0) {
            if (slot < a.k) my_src = a.store + (int64_t)slot * stride;
            else { report(a.status, FS_DEV_BAD_ID); my_ok = 0; my_src = a.weights; my_pos = 0; }
        }
    }
    if (ballot(my_ok != 0) == ~0ull) gather_wave<LG, false, EXACT>(a.units, a.out, my_src, my_pos, my_ok);
    else gather_wave<LG, true, EXACT>(a.units, a.out, my_src, my_pos, my_ok);   // ragged tail or a bad index
}

// fs_seq_unbucketize has no index in front of its row loads (row j of recv is row j), only in front
// of its stores, so it can take the shape of the fastest plain copy: one 16-byte piece per lane and
// instruction, waves that live for one instruction's worth of rows (64/LG of them), the position
// load in flight together with the row load.
constexpr int kUnbucketizeStripe = 1024;

template <int LG>
__global__ __launch_bounds__(kBlock) void unbucketize_rows_kernel(const GatherArgs a)
{
    // workgroups in stripes per XCD, as in the gather: 1024 of them write 4 MB of 512-byte rows (2.64 -> 2.53 ms)
    const int64_t j = (xcd_striped_tile(blockIdx.x, a.stripe) * kBlock + threadIdx.x) / LG;   // this group's lookup
    const int lig = threadIdx.x % LG;
    if (j >= a.m) return;
    const int32_t p = load_stream(a.pos + j);
    for (int c = lig; c < a.units; c += LG) {
        const u32x4 v = load_stream(a.weights + j * a.units + c);
        if ((uint32_t)p < (uint32_t)a.n) store_stream(a.out + (int64_t)p * a.units + c, v);
    }
    if ((uint32_t)p >= (uint32_t)a.n && lig == 0) report(a.status, FS_DEV_BAD_ID);
}

template <int LG>
static fs_status launch_unbucketize_lg(const GatherArgs& a_in, hipStream_t stream)
{
    GatherArgs a = a_in;
    const int64_t tiles = (a.m * LG + kBlock - 1) / kBlock;
    a.stripe = tiles >= (int64_t)kXcds * kUnbucketizeStripe ? kUnbucketizeStripe : 1;
    const int64_t grid = xcd_striped_grid(tiles, a.stripe);
    if (grid > 0x7FFFFFFF) return FS_ERR_SIZE;
    FS_LAUNCH("unbucketize", unbucketize_rows_kernel<LG>, dim3((unsigned)grid), dim3(kBlock), stream, a);
    return FS_OK;
}

static fs_status launch_unbucketize(const GatherArgs& a, hipStream_t s)
{
    if (a.units <= 1) return launch_unbucketize_lg<1>(a, s);
    if (a.units <= 2) return launch_unbucketize_lg<2>(a, s);
    if (a.units <= 4) return launch_unbucketize_lg<4>(a, s);
    if (a.units <= 8) return launch_unbucketize_lg<8>(a, s);
    if (a.units <= 16) return launch_unbucketize_lg<16>(a, s);
    if (a.units <= 32) return launch_unbucketize_lg<32>(a, s);
    return launch_unbucketize_lg<64>(a, s);
}

template <int LG, int MODE>
static fs_status launch_gather_lg(const GatherArgs& a_in, const char* name, hipStream_t stream)
{
    GatherArgs a = a_in;
    const int64_t tiles = (a.m + kGatherRowsPerBlock - 1) / kGatherRowsPerBlock;
    a.stripe = tiles >= (int64_t)kXcds * kXcdStripe ? kXcdStripe : 1;        // small launches are not padded
    const int64_t grid = xcd_striped_grid(tiles, a.stripe);
    if (grid > 0x7FFFFFFF) return FS_ERR_SIZE;
    if (a.units == LG)
        FS_LAUNCH(name, (gather_rows_kernel<LG, true, MODE>), dim3((unsigned)grid), dim3(kBlock), stream, a);
    else
        FS_LAUNCH(name, (gather_rows_kernel<LG, false, MODE>), dim3((unsigned)grid), dim3(kBlock), stream, a);
    return FS_OK;
}

template <int MODE>
static fs_status launch_gather(const GatherArgs& a, const char* name, hipStream_t s)
{
    if (a.units <= 1) return launch_gather_lg<1, MODE>(a, name, s);
    if (a.units <= 2) return launch_gather_lg<2, MODE>(a, name, s);
    if (a.units <= 4) return launch_gather_lg<4, MODE>(a, name, s);
    if (a.units <= 8) return launch_gather_lg<8, MODE>(a, name, s);
    if (a.units <= 16) return launch_gather_lg<16, MODE>(a, name, s);
    if (a.units <= 32) return launch_gather_lg<32, MODE>(a, name, s);
    return launch_gather_lg<64, MODE>(a, name, s);
}

// Host checks shared by the entry points; fills a.units.
static fs_status check_rows(const void* src, const void* dst, int32_t D, fs_dtype dtype, GatherArgs* a)
{
    const int es = dtype_bytes(dtype);
    if (es == 0) return FS_ERR_DTYPE;
    if (D < 1) return FS_ERR_SIZE;
    const int64_t row_bytes = (int64_t)D * es;
    if (row_bytes % 16 != 0) return FS_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) return FS_ERR_ALIGN;
    a->units = (int)(row_bytes / 16);
    return FS_OK;
}

// slot_of_row[r] = -1 for every row
__global__ __launch_bounds__(kBlock) void replica_clear_kernel(int32_t* __restrict__ slot_of_row, int64_t R)
{
    const int64_t step = (int64_t)gridDim.x * kBlock;
    for (int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x; r < R; r += step) slot_of_row[r] = -1;
}

// The owner bits of every tier-0 placement entry = the row's slot, FS_OWNER_MASK if it has none.
__global__ __launch_bounds__(kBlock) void replica_tag_slots_kernel(
    uint32_t* __restrict__ placement, int64_t R, const int32_t* __restrict__ slot_of_row, int32_t* status)
{
    const int64_t step = (int64_t)gridDim.x * kBlock;
    int32_t faults = 0;
    for (int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x; r < R; r += step) {
        if ((placement[r] >> FS_TIER_SHIFT) != FS_TIER_GLOBAL) continue;
        int32_t slot = slot_of_row[r];
        if (slot >= 0 && (uint32_t)slot >= FS_OWNER_MASK) { faults |= FS_DEV_BAD_ID; slot = -1; }   // no such slot number
        placement[r] = slot >= 0 ? (uint32_t)slot : FS_OWNER_MASK;
    }
    if (ballot(faults != 0) != 0 && lane_id() == 0) report(status, FS_DEV_BAD_ID);
}

// slot_of_row[sel_rows[s]] = the smallest s that names the row (as unsigned, -1 is the largest value)
__global__ __launch_bounds__(kBlock) void replica_slots_kernel(
    const int64_t* __restrict__ sel_rows, int64_t k, const int64_t* __restrict__ k_dev, int64_t R,
    int32_t* __restrict__ slot_of_row, int32_t* status)
{
    if (k_dev) { const int64_t kd = *k_dev; k = kd < k ? (kd < 0 ? 0 : kd) : k; }
    const int64_t step = (int64_t)gridDim.x * kBlock;
    for (int64_t s = (int64_t)blockIdx.x * kBlock + threadIdx.x; s < k; s += step) {
        const int64_t r = sel_rows[s];
        if ((uint64_t)r < (uint64_t)R) atomicMin(reinterpret_cast<uint32_t*>(slot_of_row) + r, (uint32_t)s);
        else report(status, FS_DEV_BAD_ID);
    }
}

}  // namespace fs

extern "C" fs_status fs_seq_gather_fwd(
    const void* weights, int64_t R, int32_t D, fs_dtype dtype,
    const int64_t* rows, const int32_t* pos, int64_t j0, int64_t j1,
    void* out, int64_t n, void* stream, int32_t* dev_status)
{
    using namespace fs;
    GatherArgs a = {};
    const fs_status st = check_rows(weights, out, D, dtype, &a);
    if (st == FS_ERR_DTYPE) return st;
    if (R < 1 || n < 0 || n >= (1LL << 31) || D < 1 || j0 < 0 || j0 > j1) return FS_ERR_SIZE;
    if (j1 == j0) return FS_OK;
    if (!weights || !rows || !pos || !out) return FS_ERR_NULL;
    if (st != FS_OK) return st;
    a.weights = static_cast<const u32x4*>(weights); a.R = R;
    a.rows = rows + j0; a.pos = pos + j0; a.m = j1 - j0;
    a.out = static_cast<u32x4*>(out); a.n = n; a.status = dev_status;
    return launch_gather<kBoth>(a, "gather_rows", static_cast<hipStream_t>(stream));
}

extern "C" fs_status fs_seq_gather_send(
    const void* weights, int64_t R, int32_t D, fs_dtype dtype,
    const int64_t* rows, int64_t j0, int64_t j1, void* send, void* stream, int32_t* dev_status)
{
    using namespace fs;
    GatherArgs a = {};
    const fs_status st = check_rows(weights, send, D, dtype, &a);
    if (st == FS_ERR_DTYPE) return st;
    if (R < 1 || D < 1 || j0 < 0 || j0 > j1 || j1 - j0 >= (1LL << 31)) return FS_ERR_SIZE;
    if (j1 == j0) return FS_OK;
    if (!weights || !rows || !send) return FS_ERR_NULL;
    if (st != FS_OK) return st;
    a.weights = static_cast<const u32x4*>(weights); a.R = R;
    a.rows = rows + j0; a.m = j1 - j0;
    a.out = static_cast<u32x4*>(send); a.n = a.m; a.status = dev_status;
    return launch_gather<kToSend>(a, "gather_send", static_cast<hipStream_t>(stream));
}

extern "C" fs_status fs_seq_unbucketize(
    const void* recv, int32_t D, fs_dtype dtype, const int32_t* pos, int64_t j0, int64_t j1,
    void* out, int64_t n, void* stream, int32_t* dev_status)
{
    using namespace fs;
    GatherArgs a = {};
    const fs_status st = check_rows(recv, out, D, dtype, &a);
    if (st == FS_ERR_DTYPE) return st;
    if (n < 0 || n >= (1LL << 31) || D < 1 || j0 < 0 || j0 > j1) return FS_ERR_SIZE;
    if (j1 == j0) return FS_OK;
    if (!recv || !pos || !out) return FS_ERR_NULL;
    if (st != FS_OK) return st;
    a.weights = static_cast<const u32x4*>(recv); a.R = j1 - j0;
    a.pos = pos + j0; a.m = j1 - j0;
    a.out = static_cast<u32x4*>(out); a.n = n; a.status = dev_status;
    return launch_unbucketize(a, static_cast<hipStream_t>(stream));
}

extern "C" fs_status fs_replica_build(
    const void* weights, int64_t R, int32_t D, fs_dtype dtype,
    const int64_t* sel_rows, int64_t k, const int64_t* num_selected,
    void* store, int32_t* slot_of_row, void* stream, int32_t* dev_status)
{
    using namespace fs;
    GatherArgs a = {};
    const fs_status st = check_rows(weights, store, D, dtype, &a);
    if (st == FS_ERR_DTYPE) return st;
    if (R < 1 || D < 1 || k < 0 || k >= (1LL << 31)) return FS_ERR_SIZE;
    if (!weights || !slot_of_row || (k > 0 && (!sel_rows || !store))) return FS_ERR_NULL;
    if (st != FS_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t clear_grid = (R + kBlock - 1) / kBlock;
    FS_LAUNCH("replica_clear", replica_clear_kernel, dim3((unsigned)(clear_grid < 8192 ? clear_grid : 8192)),
              dim3(kBlock), s, slot_of_row, R);
    if (k == 0) return FS_OK;
    const int64_t slot_grid = (k + kBlock - 1) / kBlock;
    FS_LAUNCH("replica_slots", replica_slots_kernel, dim3((unsigned)(slot_grid < 8192 ? slot_grid : 8192)),
              dim3(kBlock), s, sel_rows, k, num_selected, R, slot_of_row, dev_status);
    a.weights = static_cast<const u32x4*>(weights); a.R = R;
    a.rows = sel_rows; a.m = k; a.m_dev = num_selected;
    a.out = static_cast<u32x4*>(store); a.n = k; a.status = dev_status;
    return launch_gather<kToSend>(a, "replica_fill", s);
}

extern "C" fs_status fs_seq_gather_fwd_replica(
    const void* weights, int64_t R, int32_t D, fs_dtype dtype,
    const void* store, int64_t k, const int32_t* slot_of_row,
    const int64_t* rows, const int32_t* pos, int64_t j0, int64_t j1,
    void* out, int64_t n, void* stream, int32_t* dev_status)
{
    using namespace fs;
    GatherArgs a = {};
    const fs_status st = check_rows(weights, out, D, dtype, &a);
    if (st == FS_ERR_DTYPE) return st;
    if (R < 1 || n < 0 || n >= (1LL << 31) || D < 1 || j0 < 0 || j0 > j1 || k < 0 || k >= (1LL << 31))
        return FS_ERR_SIZE;
    if (j1 == j0) return FS_OK;
    if (!weights || !rows || !pos || !out || !slot_of_row || (k > 0 && !store)) return FS_ERR_NULL;
    if (st != FS_OK) return st;
    if (reinterpret_cast<uintptr_t>(store) & 15) return FS_ERR_ALIGN;
    a.weights = static_cast<const u32x4*>(weights); a.R = R;
    a.rows = rows + j0; a.pos = pos + j0; a.m = j1 - j0;
    a.out = static_cast<u32x4*>(out); a.n = n; a.status = dev_status;
    a.store = static_cast<const u32x4*>(store); a.slot_of_row = slot_of_row; a.k = k;
    return launch_gather<kReplica>(a, "gather_replica", static_cast<hipStream_t>(stream));
}

extern "C" fs_status fs_seq_gather_fwd_slots(
    const void* weights, int64_t R, int32_t D, fs_dtype dtype,
    const void* store, int64_t k, const int64_t* rows, const int32_t* slots, const int32_t* pos,
    int64_t j0, int64_t j1, void* out, int64_t n, void* stream, int32_t* dev_status)
{
    using namespace fs;
    GatherArgs a = {};
    const fs_status st = check_rows(weights, out, D, dtype, &a);
    if (st == FS_ERR_DTYPE) return st;
    if (R < 1 || n < 0 || n >= (1LL << 31) || D < 1 || j0 < 0 || j0 > j1 || k < 0 || k >= (1LL << 31))
        return FS_ERR_SIZE;
    if (j1 == j0) return FS_OK;
    if (!weights || !rows || !pos || !out || !slots || (k > 0 && !store)) return FS_ERR_NULL;
    if (st != FS_OK) return st;
    if (reinterpret_cast<uintptr_t>(store) & 15) return FS_ERR_ALIGN;
    a.weights = static_cast<const u32x4*>(weights); a.R = R;
    a.rows = rows + j0; a.pos = pos + j0; a.slots = slots + j0; a.m = j1 - j0;
    a.out = static_cast<u32x4*>(out); a.n = n; a.status = dev_status;
    a.store = static_cast<const u32x4*>(store); a.k = k;
    return launch_gather<kSlots>(a, "gather_slots", static_cast<hipStream_t>(stream));
}

extern "C" fs_status fs_replica_tag_slots(
    uint32_t* placement, int64_t R, const int32_t* slot_of_row, void* stream, int32_t* dev_status)
{
    using namespace fs;
    if (!placement || !slot_of_row) return FS_ERR_NULL;
    if (R < 1) return FS_ERR_SIZE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t grid = (R + kBlock - 1) / kBlock;
    FS_LAUNCH("replica_tag_slots", replica_tag_slots_kernel, dim3((unsigned)(grid < 16384 ? grid : 16384)), dim3(kBlock), s,
              placement, R, slot_of_row, dev_status);
    return FS_OK;
}

extern "C" fs_status fs_seq_gather_fwd_sorted(
    const void* weights, int64_t R, int32_t D, fs_dtype dtype,
    const uint32_t* sorted_rows, const uint32_t* sorted_pos, int64_t m,
    void* out, int64_t n, void* stream, int32_t* dev_status)
{
    using namespace fs;
    GatherArgs a = {};
    const fs_status st = check_rows(weights, out, D, dtype, &a);
    if (st == FS_ERR_DTYPE) return st;
    if (R < 1 || n < 0 || n >= (1LL << 31) || D < 1 || m < 0 || m >= (1LL << 31)) return FS_ERR_SIZE;
    if (m == 0) return FS_OK;
    if (!weights || !sorted_rows || !sorted_pos || !out) return FS_ERR_NULL;
    if (st != FS_OK) return st;
    a.weights = static_cast<const u32x4*>(weights); a.R = R;
    a.rows32 = sorted_rows; a.pos = reinterpret_cast<const int32_t*>(sorted_pos); a.m = m;   // a position >= 2^31 fails the range check
    a.out = static_cast<u32x4*>(out); a.n = n; a.status = dev_status;
    return launch_gather<kSorted>(a, "gather_sorted", static_cast<hipStream_t>(stream));
}
