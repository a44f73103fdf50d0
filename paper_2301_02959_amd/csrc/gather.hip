// fs_seq_gather_fwd: out[pos[j], :] = weights[rows[j], :] for j in [j0, j1).
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
// Blocks take tiles in launch order: the round-robin deal of blocks to the 8 XCDs
// then spreads the cold, other-bucket tail of the j range over all of them (giving
// each XCD one contiguous eighth of j leaves the last XCD with all the cache misses).
#include "fs_common.h"

namespace fs {

constexpr int kGatherRowsPerWave = kWave;
constexpr int kGatherRowsPerBlock = kGatherRowsPerWave * kWavesPerBlock;

template <int LG>
struct GatherShape {
    static constexpr int RPI = kWave / LG;                                   // rows per instruction
    static constexpr int UNR = RPI >= 8 ? kWave / RPI : (LG == 16 ? 8 : 16); // instructions in flight
};

// Moves the wave's 64 rows.  GUARD = false: every lookup of the wave is valid, loads and
// stores carry no per-lane predicate (a predicated load makes the compiler wait for each
// load before it issues the next, which serialises the 16 loads of a batch).
// EXACT: the row is exactly LG pieces long (power-of-two row sizes), so there is no loop over
// pieces and no idle lane.
template <int LG, bool GUARD, bool EXACT>
__device__ __forceinline__ void gather_wave(const u32x4* __restrict__ weights, int units, u32x4* __restrict__ out,
                                            int64_t my_row, int32_t my_pos, int my_ok)
{
    constexpr int RPI = GatherShape<LG>::RPI;
    constexpr int UNR = GatherShape<LG>::UNR;
    const int lane = lane_id();
    const int g = lane / LG;
    const int lig = lane % LG;
#pragma unroll 1
    for (int s = 0; s < kGatherRowsPerWave; s += UNR * RPI) {
        int64_t src[UNR];
        int64_t dst[UNR];
        bool ok[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int from = s + u * RPI + g;            // lane that holds this row's indices
            const int64_t r = __shfl(my_row, from);
            const int32_t p = __shfl(my_pos, from);
            ok[u] = GUARD ? __shfl(my_ok, from) != 0 : true;
            src[u] = EXACT ? r * LG : r * units;             // a compile-time stride folds into shifts
            dst[u] = EXACT ? (int64_t)p * LG : (int64_t)p * units;
        }
        if (EXACT) {
            u32x4 v[UNR];
#pragma unroll
            for (int u = 0; u < UNR; ++u) v[u] = weights[src[u] + lig];     // invalid lookups read row 0
#pragma unroll
            for (int u = 0; u < UNR; ++u)
                if (!GUARD || ok[u]) store_stream(out + dst[u] + lig, v[u]);
        } else {
            for (int c = lig; c < units; c += LG) {
                u32x4 v[UNR];
#pragma unroll
                for (int u = 0; u < UNR; ++u) v[u] = weights[src[u] + c];
#pragma unroll
                for (int u = 0; u < UNR; ++u)
                    if (!GUARD || ok[u]) store_stream(out + dst[u] + c, v[u]);
            }
        }
    }
}

template <int LG, bool EXACT>
__global__ __launch_bounds__(kBlock) void gather_rows_kernel(
    const u32x4* __restrict__ weights, int64_t R, int units,
    const int64_t* __restrict__ rows, const int32_t* __restrict__ pos, int64_t m,
    u32x4* __restrict__ out, int64_t n, int32_t* status)
{
    const int lane = lane_id();
    const int64_t wbase = ((int64_t)blockIdx.x * kWavesPerBlock + wave_id()) * kGatherRowsPerWave;
    if (wbase >= m) return;                              // wave-uniform

    // one coalesced load of the wave's 64 (row, position) pairs
    const int64_t jj = wbase + lane;
    int64_t my_row = 0;
    int32_t my_pos = 0;
    int my_ok = 0;
    if (jj < m) {
        my_row = load_stream(rows + jj);
        my_pos = load_stream(pos + jj);
        // unsigned compares: one test each also catches the negative values (n < 2^31)
        my_ok = ((uint64_t)my_row < (uint64_t)R && (uint32_t)my_pos < (uint32_t)n) ? 1 : 0;
        if (!my_ok) { report(status, FS_DEV_BAD_ID); my_row = 0; my_pos = 0; }
    }
    if (ballot(my_ok != 0) == ~0ull) gather_wave<LG, false, EXACT>(weights, units, out, my_row, my_pos, my_ok);
    else gather_wave<LG, true, EXACT>(weights, units, out, my_row, my_pos, my_ok);   // ragged tail or a bad index
}

template <int LG>
static fs_status launch_gather(const void* weights, int64_t R, int units, const int64_t* rows,
                               const int32_t* pos, int64_t m, void* out, int64_t n,
                               hipStream_t stream, int32_t* status)
{
    const int64_t grid = (m + kGatherRowsPerBlock - 1) / kGatherRowsPerBlock;
    if (grid > 0x7FFFFFFF) return FS_ERR_SIZE;
    if (units == LG)
        FS_LAUNCH("gather_rows", (gather_rows_kernel<LG, true>), dim3((unsigned)grid), dim3(kBlock), stream,
                  static_cast<const u32x4*>(weights), R, units, rows, pos, m, static_cast<u32x4*>(out), n, status);
    else
        FS_LAUNCH("gather_rows", (gather_rows_kernel<LG, false>), dim3((unsigned)grid), dim3(kBlock), stream,
                  static_cast<const u32x4*>(weights), R, units, rows, pos, m, static_cast<u32x4*>(out), n, status);
    return FS_OK;
}

}  // namespace fs

extern "C" fs_status fs_seq_gather_fwd(
    const void* weights, int64_t R, int32_t D, fs_dtype dtype,
    const int64_t* rows, const int32_t* pos, int64_t j0, int64_t j1,
    void* out, int64_t n, void* stream, int32_t* dev_status)
{
    using namespace fs;
    const int es = dtype_bytes(dtype);
    if (es == 0) return FS_ERR_DTYPE;
    if (R < 1 || n < 0 || n >= (1LL << 31) || D < 1 || j0 < 0 || j0 > j1) return FS_ERR_SIZE;
    const int64_t m = j1 - j0;
    if (m == 0) return FS_OK;
    if (!weights || !rows || !pos || !out) return FS_ERR_NULL;
    const int64_t row_bytes = (int64_t)D * es;
    if (row_bytes % 16 != 0) return FS_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(weights) | reinterpret_cast<uintptr_t>(out)) & 15) return FS_ERR_ALIGN;
    const int units = (int)(row_bytes / 16);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t* r = rows + j0;
    const int32_t* p = pos + j0;
    if (units <= 1) return launch_gather<1>(weights, R, units, r, p, m, out, n, s, dev_status);
    if (units <= 2) return launch_gather<2>(weights, R, units, r, p, m, out, n, s, dev_status);
    if (units <= 4) return launch_gather<4>(weights, R, units, r, p, m, out, n, s, dev_status);
    if (units <= 8) return launch_gather<8>(weights, R, units, r, p, m, out, n, s, dev_status);
    if (units <= 16) return launch_gather<16>(weights, R, units, r, p, m, out, n, s, dev_status);
    if (units <= 32) return launch_gather<32>(weights, R, units, r, p, m, out, n, s, dev_status);
    return launch_gather<64>(weights, R, units, r, p, m, out, n, s, dev_status);
}
