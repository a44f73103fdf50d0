// Shared host/device helpers of libflexshard_hip (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "flexshard.h"

namespace fs {

constexpr int kWave = 64;          // CDNA wavefront
constexpr int kBlock = 256;        // threads per workgroup used by every kernel here
constexpr int kWavesPerBlock = kBlock / kWave;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---- opt-in per-kernel timing (see fs_prof_begin in flexshard.h) -----------
void prof_pre(const char* name, hipStream_t stream);
void prof_post(hipStream_t stream);
extern bool g_prof_on;

#define FS_LAUNCH_SMEM(name, kernel, grid, block, smem, stream, ...)                    \
    do {                                                                                \
        if (fs::g_prof_on) fs::prof_pre(name, stream);                                  \
        hipLaunchKernelGGL(kernel, grid, block, smem, stream, __VA_ARGS__);             \
        if (fs::g_prof_on) fs::prof_post(stream);                                       \
        if (hipGetLastError() != hipSuccess) return FS_ERR_DEVICE;                      \
    } while (0)
#define FS_LAUNCH(name, kernel, grid, block, stream, ...)                               \
    FS_LAUNCH_SMEM(name, kernel, grid, block, 0, stream, __VA_ARGS__)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Carves 256-byte aligned pieces out of a caller-provided workspace; with a null
// base it only adds up sizes.
struct Carver {
    char* base;
    size_t used = 0;
    explicit Carver(void* p) : base(static_cast<char*>(p)) {}
    template <typename T>
    T* take(size_t count)
    {
        size_t off = used;
        used += align_up(count * sizeof(T), 256);
        return base ? reinterpret_cast<T*>(base + off) : nullptr;
    }
};

inline int dtype_bytes(fs_dtype d)
{
    return d == FS_F32 ? 4 : (d == FS_F16 || d == FS_BF16) ? 2 : 0;
}

inline int bits_for(uint64_t max_value)   // number of bits needed to write max_value
{
    int b = 1;
    while (b < 64 && (max_value >> b) != 0) ++b;
    return b;
}

// Workgroup b runs on XCD b % 8.  A kernel whose workgroup b takes tile xcd_striped_tile(b, stripe)
// gives every XCD `stripe` consecutive tiles at a time; its grid is xcd_striped_grid(tiles, stripe)
// workgroups, and those whose tile is >= tiles have nothing to do.
constexpr int kXcds = 8;

inline int64_t xcd_striped_grid(int64_t tiles, int stripe)
{
    const int64_t round = (int64_t)kXcds * stripe;
    return (tiles + round - 1) / round * round;
}

#ifdef __HIPCC__
// ---- device helpers ---------------------------------------------------------
__device__ __forceinline__ int64_t xcd_striped_grid_dev(int64_t tiles, int stripe)
{
    const int64_t round = (int64_t)kXcds * stripe;
    return (tiles + round - 1) / round * round;
}

__device__ __forceinline__ int64_t xcd_striped_tile(unsigned block, int stripe)
{
    const int64_t x = block % kXcds;
    const int64_t k = block / kXcds;
    return (k / stripe) * (int64_t)(kXcds * stripe) + x * stripe + (k % stripe);
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

// number of set bits of `mask` below this lane
__device__ __forceinline__ int popc_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
}

__device__ __forceinline__ uint64_t ballot(bool p) { return __ballot(p); }

// Lanes of the wave whose `key` has the same low `nbits` bits as this lane's,
// restricted to lanes with `valid`.  nbits ballots, no LDS.
__device__ __forceinline__ uint64_t match_bits(uint32_t key, int nbits, bool valid)
{
    const uint64_t all = ballot(valid);
    uint32_t m_lo = (uint32_t)all, m_hi = (uint32_t)(all >> 32);
#pragma unroll 1
    for (int b = 0; b < nbits; ++b) {
        uint32_t x = (uint32_t)((int32_t)(key << (31 - b)) >> 31);   // 0 or ~0: the lane's bit b
        asm volatile("" : "+v"(x));
        const uint64_t v = ballot(x != 0u);
        m_lo &= ~((uint32_t)v ^ x);                                  // lanes whose bit b agrees with this lane's
        m_hi &= ~((uint32_t)(v >> 32) ^ x);
    }
    return ((uint64_t)m_hi << 32) | m_lo;
}

// The same with the bit count known at compile time: the loop unrolls, the shifts fold.  Written on
// 32-bit halves with the lane's bit spread to a whole word: per bit one bit-field extract, one compare
// (the ballot), one exclusive-or per half, and the halves' mismatches are or-ed three at a time: a
// third fewer vector instructions than selecting between the ballot and its complement, and the sort's
// count and scatter kernels are bound by exactly these instructions.
template <int NBITS>
__device__ __forceinline__ uint64_t match_bits_n(uint32_t key, bool valid)
{
    const uint64_t all = ballot(valid);
    uint32_t m_lo = (uint32_t)all, m_hi = (uint32_t)(all >> 32);
#pragma unroll
    for (int b = 0; b < NBITS; ++b) {
        // x = 0 or ~0 as the lane's bit is clear or set; the lanes that agree with it are ~(v ^ x)
        uint32_t x = (uint32_t)((int32_t)(key << (31 - b)) >> 31);
        asm volatile("" : "+v"(x));          // one bit-field extract, and the ballot compares x itself (no second shift)
        const uint64_t v = ballot(x != 0u);
        m_lo &= ~((uint32_t)v ^ x);
        m_hi &= ~((uint32_t)(v >> 32) ^ x);
    }
    return ((uint64_t)m_hi << 32) | m_lo;
}

#define FS_DISPATCH_BITS(nbits, CALL)                                                   \
    switch (nbits) {                                                                    \
        case 1: CALL(1); break;  case 2: CALL(2); break;  case 3: CALL(3); break;       \
        case 4: CALL(4); break;  case 5: CALL(5); break;  case 6: CALL(6); break;       \
        case 7: CALL(7); break;  case 8: CALL(8); break;  case 9: CALL(9); break;       \
        default: CALL(10); break;                                                       \
    }

template <typename T>
__device__ __forceinline__ T load_stream(const T* p) { return __builtin_nontemporal_load(p); }
template <typename T>
__device__ __forceinline__ void store_stream(T* p, T v) { __builtin_nontemporal_store(v, p); }

// Exclusive prefix of `v` over the threads of the block (any multiple of 64 threads up to
// 1024); *total receives the block sum.  `wave_sums` is LDS scratch of 16 words.  Contains
// block barriers: every thread of the block must call it.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wave_sums, uint32_t* total)
{
    const int lane = lane_id();
    const int w = wave_id();
    const int waves = (int)(blockDim.x >> 6);
    uint32_t incl = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
    }
    __syncthreads();                       // wave_sums may still be read from a previous call
    if (lane == kWave - 1) wave_sums[w] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
    for (int k = 0; k < waves; ++k) {
        const uint32_t s = wave_sums[k];
        if (k < w) before += s;
        all += s;
    }
    *total = all;
    return before + incl - v;
}

__device__ __forceinline__ void report(int32_t* status, int32_t bits)
{
    if (status != nullptr && bits != 0) atomicOr(status, bits);
}
#endif  // __HIPCC__

}  // namespace fs
