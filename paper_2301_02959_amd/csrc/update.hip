// fs_sparse_update: one optimizer step on the rows a backward pass produced gradients for.
//
//   SGD               w -= lr g
//   Adagrad           s += g^2 per element;           w -= lr g / (sqrt(s) + eps)
//   row-wise Adagrad  s_r += mean of g^2 over the row; w -= lr g / (sqrt(s_r) + eps)
//
// HBM-bound read-modify-write of scattered rows: per row one fp32 gradient row in, the table row
// in and out, the state in and out.  The layout is the gather's: a wave owns 64 consecutive
// entries of uniq_rows, reads them with one coalesced load, hands them to groups of LG lanes with
// ds_bpermute; a group moves one row per instruction (4 or 8 elements of the table row per lane and
// the matching fp32 gradients and state values, laid out so that every load is coalesced), UNR rows
// in flight.  Table rows and element-wise state are read and written in place exactly once, so
// their loads and stores are non-temporal: left cacheable, the dirty lines of 1.5 M scattered
// 512-byte rows cost a quarter of the kernel's time (0.83 -> 0.64 ms) when they are written back
// later; the mirror copy in the replica store stays cacheable, the gather reads it next.
// The row-wise rule needs the row's sum of squares: a butterfly over the group's lanes.
// Arithmetic is fp32, one IEEE operation at a time (no fused multiply-add, correctly rounded
// division and square root); the new weight is rounded once to the table's type, to nearest even.
// Rows longer than 64 pieces (1 KB) take a slower path: one wave per row, piece by piece.
#include "fs_common.h"
#include "update_rules.h"

namespace fs {


// A group of LG lanes owns a row of up to LG * N elements, in quads of 4 elements: lane i takes quad
// i of every run of LG quads (one run for fp32 tables, two for 16-bit tables), so that the fp32
// gradient and state loads of a group are one contiguous 16 * LG bytes per instruction and the table
// loads one contiguous 16 * LG (fp32) or 8 * LG (16-bit) bytes.
template <int LG, int DT, int OPT, bool EXACT>
__global__ __launch_bounds__(kBlock) void sparse_update_kernel(const UpdateArgs a)
{
    constexpr int N = Elems<DT>::N;
    constexpr int P = N / 4;                                         // quads per lane
    constexpr int RPI = kWave / LG;
    constexpr int UNR = LG >= 32 ? 4 : (LG >= 8 ? 2 : 1);          // row instructions in flight (2 and 8 are slower)
    typedef typename Quad<DT>::type quad_t;
    const int lane = lane_id();
    const int64_t wbase = ((int64_t)blockIdx.x * kWavesPerBlock + wave_id()) * kWave;
    int64_t m = a.cap;
    if (a.num_unique) { const int64_t nu = *a.num_unique; m = nu < m ? (nu < 0 ? 0 : nu) : m; }
    if (wbase >= m) return;                                          // wave-uniform

    __shared__ uint8_t s_from[kWavesPerBlock][kWave];
    const int64_t jj = wbase + lane;
    int64_t my_row = 0;
    int my_ok = 0, my_slot = -1;
    if (jj < m) {
        my_row = a.uniq_rows[jj];
        my_ok = (uint64_t)my_row < (uint64_t)a.R ? 1 : 0;
        if (!my_ok) { report(a.status, FS_DEV_BAD_ID); my_row = 0; }
        else if (a.skip != nullptr && a.skip[jj] != 0) { my_ok = 0; my_row = 0; }
        else if (a.store != nullptr) {
            my_slot = a.slot_of_row[my_row];
            if (my_slot >= a.k) { report(a.status, FS_DEV_BAD_ID); my_slot = -1; }
        }
    }
    const int g = lane / LG;
    const int lig = lane % LG;
    const int64_t D = EXACT ? LG * N : a.D;                          // elements per row
    int col[P];                                                      // first element of the lane's quads
    bool on[P];
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const int c = (p * LG + lig) * 4;
        on[p] = c < D;                                               // rows shorter than LG * N elements leave quads idle
        col[p] = on[p] ? c : 0;
    }
    const quad_t* wq = reinterpret_cast<const quad_t*>(a.weights);   // a quad is element index / 4
    quad_t* wq_out = reinterpret_cast<quad_t*>(a.weights);
    quad_t* store_out = reinterpret_cast<quad_t*>(a.store);
    // the wave's entries that have work, packed: the rounds below only walk those (with most entries
    // skipped, the rest would still cost a round of loads each)
    const uint64_t live = ballot(my_ok != 0);
    const int cnt = __popcll(live);
    if (cnt == 0) return;                                            // wave-uniform
    if (my_ok) s_from[wave_id()][popc_below(live)] = (uint8_t)lane;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int first_live = s_from[wave_id()][0];
#pragma unroll 1
    for (int s0 = 0; s0 < cnt; s0 += UNR * RPI) {
        int64_t r[UNR], u[UNR];
        int ok[UNR], sl[UNR];
#pragma unroll
        for (int j = 0; j < UNR; ++j) {
            const int at = s0 + j * RPI + g;
            ok[j] = at < cnt;
            const int from = ok[j] ? s_from[wave_id()][at] : first_live;   // past the list: the first entry again, not stored
            r[j] = __shfl(my_row, from);
            sl[j] = __shfl(my_slot, from);
            u[j] = wbase + from;
        }
        quad_t wx[UNR][P];
        f32x4 gx[UNR][P], sx[UNR][P];
        float srow[UNR];
#pragma unroll
        for (int j = 0; j < UNR; ++j) {
#pragma unroll
            for (int p = 0; p < P; ++p) {
                wx[j][p] = load_stream(wq + ((r[j] * D + col[p]) >> 2));
                gx[j][p] = load_stream(reinterpret_cast<const f32x4*>(a.row_grads + u[j] * D + col[p]));
                if constexpr (OPT == FS_OPT_ADAGRAD)
                    sx[j][p] = load_stream(reinterpret_cast<const f32x4*>(a.state + r[j] * D + col[p]));
            }
            if constexpr (OPT == FS_OPT_ADAGRAD_ROWWISE) srow[j] = a.state[r[j]];
        }
#pragma unroll
        for (int j = 0; j < UNR; ++j)
            RowUpdate<LG, DT, OPT>::apply(wx[j], gx[j], sx[j], srow[j], on, col, r[j], D, lig, ok[j] != 0, sl[j], a.lr,
                                          a.eps, wq_out, store_out, a.state);
    }
}

// Rows of more than 64 pieces: one wave per entry, the row piece by piece (64 pieces a round); the
// row-wise rule reads the gradient row twice (sum of squares first).
template <int DT, int OPT>
__global__ __launch_bounds__(kBlock) void sparse_update_long_kernel(const UpdateArgs a)
{
    constexpr int N = Elems<DT>::N;
    const int lane = lane_id();
    const int64_t u = (int64_t)blockIdx.x * kWavesPerBlock + wave_id();
    int64_t m = a.cap;
    if (a.num_unique) { const int64_t nu = *a.num_unique; m = nu < m ? (nu < 0 ? 0 : nu) : m; }
    if (u >= m) return;                                              // wave-uniform
    const int64_t r = a.uniq_rows[u];
    if ((uint64_t)r >= (uint64_t)a.R) { if (lane == 0) report(a.status, FS_DEV_BAD_ID); return; }
    if (a.skip != nullptr && a.skip[u] != 0) return;
    int slot = -1;
    if (a.store != nullptr) {
        slot = a.slot_of_row[r];
        if (slot >= a.k) { if (lane == 0) report(a.status, FS_DEV_BAD_ID); slot = -1; }
    }
    float s_row = 0.0f;
    if constexpr (OPT == FS_OPT_ADAGRAD_ROWWISE) {
        float sq = 0.0f;
        for (int c = lane; c < a.units; c += kWave) {
            const float* gp = a.row_grads + u * a.D + c * N;
#pragma unroll
            for (int i = 0; i < N; ++i) sq = sq + gp[i] * gp[i];
        }
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) sq = sq + __shfl_xor(sq, off);
        s_row = a.state[r] + sq / (float)a.D;
    }
    for (int c = lane; c < a.units; c += kWave) {
        float w[N], gf[N], sf[N];
        Elems<DT>::unpack(load_stream(a.weights + r * a.units + c), w);    // read and written once: non-temporal
        const float* gp = a.row_grads + u * a.D + c * N;
        float* sp = a.state + r * a.D + c * N;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            gf[i] = gp[i];
            if constexpr (OPT == FS_OPT_ADAGRAD) sf[i] = sp[i];
        }
        apply_rule<N, OPT>(w, gf, sf, s_row, a.lr, a.eps);
        const u32x4 out = Elems<DT>::pack(w);
        store_stream(a.weights + r * a.units + c, out);
        if (slot >= 0) a.store[(int64_t)slot * a.units + c] = out;
        if constexpr (OPT == FS_OPT_ADAGRAD) {
#pragma unroll
            for (int i = 0; i < N; ++i) sp[i] = sf[i];
        }
    }
    if constexpr (OPT == FS_OPT_ADAGRAD_ROWWISE) {
        __builtin_amdgcn_wave_barrier();                             // every lane has read state[r] above
        if (lane == 0) a.state[r] = s_row;
    }
}

template <int LG, int DT, int OPT>
static fs_status launch_update_lg(const UpdateArgs& a, hipStream_t stream)
{
    const int64_t grid = (a.cap + kBlock - 1) / kBlock;              // 64 entries per wave
    if (grid > 0x7FFFFFFF) return FS_ERR_SIZE;
    if (a.units == LG)
        FS_LAUNCH("sparse_update", (sparse_update_kernel<LG, DT, OPT, true>), dim3((unsigned)grid), dim3(kBlock), stream, a);
    else
        FS_LAUNCH("sparse_update", (sparse_update_kernel<LG, DT, OPT, false>), dim3((unsigned)grid), dim3(kBlock), stream, a);
    return FS_OK;
}

template <int DT, int OPT>
static fs_status launch_update(const UpdateArgs& a, hipStream_t stream)
{
    if (a.units > kWave) {
        const int64_t grid = (a.cap + kWavesPerBlock - 1) / kWavesPerBlock;
        if (grid > 0x7FFFFFFF) return FS_ERR_SIZE;
        FS_LAUNCH("sparse_update_long", (sparse_update_long_kernel<DT, OPT>), dim3((unsigned)grid), dim3(kBlock), stream, a);
        return FS_OK;
    }
    if (a.units <= 1) return launch_update_lg<1, DT, OPT>(a, stream);
    if (a.units <= 2) return launch_update_lg<2, DT, OPT>(a, stream);
    if (a.units <= 4) return launch_update_lg<4, DT, OPT>(a, stream);
    if (a.units <= 8) return launch_update_lg<8, DT, OPT>(a, stream);
    if (a.units <= 16) return launch_update_lg<16, DT, OPT>(a, stream);
    if (a.units <= 32) return launch_update_lg<32, DT, OPT>(a, stream);
    return launch_update_lg<64, DT, OPT>(a, stream);
}

template <int DT>
static fs_status launch_update_opt(const UpdateArgs& a, int optimizer, hipStream_t stream)
{
    if (optimizer == FS_OPT_SGD) return launch_update<DT, FS_OPT_SGD>(a, stream);
    if (optimizer == FS_OPT_ADAGRAD) return launch_update<DT, FS_OPT_ADAGRAD>(a, stream);
    return launch_update<DT, FS_OPT_ADAGRAD_ROWWISE>(a, stream);
}

fs_status sparse_update_launch(const UpdateArgs& a, fs_dtype dtype, int optimizer, hipStream_t s)
{
    if (dtype == FS_F32) return launch_update_opt<FS_F32>(a, optimizer, s);
    if (dtype == FS_F16) return launch_update_opt<FS_F16>(a, optimizer, s);
    return launch_update_opt<FS_BF16>(a, optimizer, s);
}

}  // namespace fs

extern "C" fs_status fs_sparse_update(
    void* weights, int64_t R, int32_t D, fs_dtype dtype,
    const int64_t* uniq_rows, const float* row_grads, int64_t cap_unique, const int64_t* num_unique,
    int32_t optimizer, float lr, float eps, float* state,
    void* store, const int32_t* slot_of_row, int64_t k,
    void* stream, int32_t* dev_status)
{
    using namespace fs;
    const int es = dtype_bytes(dtype);
    if (es == 0) return FS_ERR_DTYPE;
    if (R < 1 || D < 1 || cap_unique < 0 || k < 0 || k >= (1LL << 31)) return FS_ERR_SIZE;
    if (optimizer != FS_OPT_SGD && optimizer != FS_OPT_ADAGRAD && optimizer != FS_OPT_ADAGRAD_ROWWISE) return FS_ERR_CONFIG;
    if (!weights || (cap_unique > 0 && (!uniq_rows || !row_grads))) return FS_ERR_NULL;
    if (optimizer != FS_OPT_SGD && !state) return FS_ERR_NULL;
    if ((store != nullptr) != (slot_of_row != nullptr)) return FS_ERR_NULL;
    const int64_t row_bytes = (int64_t)D * es;
    if (row_bytes % 16 != 0) return FS_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(weights) | reinterpret_cast<uintptr_t>(row_grads) |
         reinterpret_cast<uintptr_t>(store) | reinterpret_cast<uintptr_t>(state)) & 15)
        return FS_ERR_ALIGN;
    if (cap_unique == 0) return FS_OK;
    UpdateArgs a;
    a.weights = static_cast<u32x4*>(weights); a.R = R; a.units = (int)(row_bytes / 16); a.D = D;
    a.uniq_rows = uniq_rows; a.row_grads = row_grads; a.cap = cap_unique; a.num_unique = num_unique;
    a.lr = lr; a.eps = eps; a.state = state;
    a.store = static_cast<u32x4*>(store); a.slot_of_row = slot_of_row; a.k = k; a.status = dev_status;
    a.skip = nullptr;
    return sparse_update_launch(a, dtype, optimizer, static_cast<hipStream_t>(stream));
}
