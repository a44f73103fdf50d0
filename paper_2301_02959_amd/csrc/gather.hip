// fs_seq_gather_fwd: out[pos[j], :] = weights[rows[j], :] for j in [j0, j1).
//
// HBM-bound bit copy.  A row of `units` 16-byte pieces is moved by a group of LG
// lanes (LG = the power of two >= units, at most 64), one 128-bit load and one
// 128-bit non-temporal store per lane; a wave therefore moves 64/LG rows per
// instruction and each group keeps UNR rows in flight.  Table reads stay
// cacheable (popular rows are re-read from L2 / Infinity Cache), the output is
// streamed past the caches.  Blocks are mapped so that each XCD walks one
// contiguous range of j: inside a bucket j is ascending in the flat position,
// i.e. table-major, so an XCD's L2 holds the hot rows of one or two tables.
#include "fs_common.h"

namespace fs {

constexpr int kGatherUnroll = 8;

template <int LG>
__global__ __launch_bounds__(kBlock) void gather_rows_kernel(
    const u32x4* __restrict__ weights, int64_t R, int units,
    const int64_t* __restrict__ rows, const int32_t* __restrict__ pos, int64_t m,
    u32x4* __restrict__ out, int64_t n, int64_t tiles, int64_t tiles_per_xcd,
    int32_t* status)
{
    constexpr int GPB = kBlock / LG;               // row groups per block
    constexpr int TILE = GPB * kGatherUnroll;      // rows per block
    const int64_t tile = xcd_contiguous_tile(blockIdx.x, tiles_per_xcd);
    if (tile >= tiles) return;
    const int lig = threadIdx.x % LG;
    const int gi = threadIdx.x / LG;
    const int64_t base = tile * TILE;

    int64_t src[kGatherUnroll];
    int64_t dst[kGatherUnroll];
    bool ok[kGatherUnroll];
    bool bad = false;
#pragma unroll
    for (int u = 0; u < kGatherUnroll; ++u) {
        const int64_t jj = base + (int64_t)u * GPB + gi;
        ok[u] = jj < m;
        int64_t r = 0;
        int64_t p = 0;
        if (ok[u]) {
            r = load_stream(rows + jj);
            p = load_stream(pos + jj);
            if (r < 0 || r >= R || p < 0 || p >= n) { ok[u] = false; bad = true; }
        }
        src[u] = r * units;
        dst[u] = p * units;
    }
    for (int c = lig; c < units; c += LG) {
        u32x4 v[kGatherUnroll];
#pragma unroll
        for (int u = 0; u < kGatherUnroll; ++u)
            if (ok[u]) v[u] = weights[src[u] + c];
#pragma unroll
        for (int u = 0; u < kGatherUnroll; ++u)
            if (ok[u]) store_stream(out + dst[u] + c, v[u]);
    }
    if (bad && lig == 0) report(status, FS_DEV_BAD_ID);
}

template <int LG>
static fs_status launch_gather(const void* weights, int64_t R, int units, const int64_t* rows,
                               const int32_t* pos, int64_t m, void* out, int64_t n,
                               hipStream_t stream, int32_t* status)
{
    constexpr int TILE = (kBlock / LG) * kGatherUnroll;
    const int64_t tiles = (m + TILE - 1) / TILE;
    const int64_t per_xcd = (tiles + kXcds - 1) / kXcds;
    const int64_t grid = per_xcd * kXcds;
    if (grid > 0x7FFFFFFF) return FS_ERR_SIZE;
    FS_LAUNCH("gather_rows", gather_rows_kernel<LG>, dim3((unsigned)grid), dim3(kBlock), stream,
              static_cast<const u32x4*>(weights), R, units, rows, pos, m,
              static_cast<u32x4*>(out), n, tiles, per_xcd, status);
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
