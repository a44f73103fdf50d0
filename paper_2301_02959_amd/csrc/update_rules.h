// The optimizer rules of fs_sparse_update and of the backward that applies them itself
// (fs_seq_grad_bwd_update): element packing of the three table types and the update arithmetic.
// fp32, one IEEE operation at a time (no fused multiply-add, correctly rounded division and square
// root); the new weight is rounded once to the table's type, to nearest even.
#pragma once

#include "fs_common.h"

namespace fs {

typedef _Float16 h16x8 __attribute__((ext_vector_type(8)));

template <int DT>
struct Elems {
    static constexpr int N = DT == FS_F32 ? 4 : 8;
    static __device__ __forceinline__ void unpack(const u32x4& x, float* f)
    {
        if constexpr (DT == FS_F32) {
#pragma unroll
            for (int i = 0; i < 4; ++i) f[i] = __uint_as_float(x[i]);
        } else if constexpr (DT == FS_F16) {
            const h16x8 h = __builtin_bit_cast(h16x8, x);
#pragma unroll
            for (int i = 0; i < 8; ++i) f[i] = (float)h[i];
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                f[2 * i] = __uint_as_float(x[i] << 16);
                f[2 * i + 1] = __uint_as_float(x[i] & 0xFFFF0000u);
            }
        }
    }
    static __device__ __forceinline__ uint32_t bf16_bits(float v)     // round to nearest even
    {
        const uint32_t b = __float_as_uint(v);
        if ((b & 0x7FFFFFFFu) > 0x7F800000u) return (b >> 16) | 0x40u;          // NaN stays NaN
        return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
    }
    static __device__ __forceinline__ u32x4 pack(const float* f)
    {
        u32x4 x;
        if constexpr (DT == FS_F32) {
#pragma unroll
            for (int i = 0; i < 4; ++i) x[i] = __float_as_uint(f[i]);
        } else if constexpr (DT == FS_F16) {
            h16x8 h;
#pragma unroll
            for (int i = 0; i < 8; ++i) h[i] = (_Float16)f[i];                  // v_cvt_f16_f32: nearest even
            x = __builtin_bit_cast(u32x4, h);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) x[i] = bf16_bits(f[2 * i]) | (bf16_bits(f[2 * i + 1]) << 16);
        }
        return x;
    }
};

// The new values of one lane's N elements.  s_row: the row-wise state after this step.
template <int N, int OPT>
__device__ __forceinline__ void apply_rule(float* w, const float* g, float* s, float s_row, float lr, float eps)
{
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const float lg = lr * g[i];
        if constexpr (OPT == FS_OPT_SGD) {
            w[i] = w[i] - lg;
        } else if constexpr (OPT == FS_OPT_ADAGRAD) {
            s[i] = s[i] + g[i] * g[i];
            w[i] = w[i] - lg / (sqrtf(s[i]) + eps);
        } else {
            w[i] = w[i] - lg / (sqrtf(s_row) + eps);
        }
    }
}

// Four consecutive elements of a table row: 16 bytes of fp32, 8 bytes of a 16-bit type.
template <int DT>
struct Quad {
    typedef u32x4 type;
    static __device__ __forceinline__ void unpack(const type& x, float* f)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = __uint_as_float(x[i]);
    }
    static __device__ __forceinline__ type pack(const float* f)
    {
        return type{__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3])};
    }
};
template <>
struct Quad<FS_F16> {
    typedef u32x2 type;
    typedef _Float16 h16x4 __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ void unpack(const type& x, float* f)
    {
        const h16x4 h = __builtin_bit_cast(h16x4, x);
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = (float)h[i];
    }
    static __device__ __forceinline__ type pack(const float* f)
    {
        h16x4 h;
#pragma unroll
        for (int i = 0; i < 4; ++i) h[i] = (_Float16)f[i];                      // v_cvt_f16_f32: nearest even
        return __builtin_bit_cast(type, h);
    }
};
template <>
struct Quad<FS_BF16> {
    typedef u32x2 type;
    static __device__ __forceinline__ void unpack(const type& x, float* f)
    {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            f[2 * i] = __uint_as_float(x[i] << 16);
            f[2 * i + 1] = __uint_as_float(x[i] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ type pack(const float* f)
    {
        return type{Elems<FS_BF16>::bf16_bits(f[0]) | (Elems<FS_BF16>::bf16_bits(f[1]) << 16),
                    Elems<FS_BF16>::bf16_bits(f[2]) | (Elems<FS_BF16>::bf16_bits(f[3]) << 16)};
    }
};

// What one optimizer step works on (fs_sparse_update's arguments).
struct UpdateArgs {
    u32x4* weights;
    int64_t R;
    int units;                       // 16-byte pieces per table row
    int D;
    const int64_t* uniq_rows;
    const float* row_grads;
    int64_t cap;
    const int64_t* num_unique;       // device; only the first min(cap, *num_unique) entries are applied
    float lr, eps;
    float* state;
    u32x4* store;                    // replica store, or nullptr
    const int32_t* slot_of_row;
    int64_t k;
    int32_t* status;
    const uint8_t* skip;             // if set: entries u with skip[u] != 0 are left alone (another kernel updated them)
};

// Launches the optimizer step described by `a` (fs_sparse_update's kernels).
fs_status sparse_update_launch(const UpdateArgs& a, fs_dtype dtype, int optimizer, hipStream_t stream);

// One row in the quad layout: a group of LG lanes owns the row, lane `lig` holds quads lig, LG + lig, ...
// (P = 1 for fp32 tables, 2 for 16-bit tables); col[p] is the first element of the lane's quad p, on[p]
// whether the row is long enough to have it.  wx: the row's old values, gx: its fp32 gradient, sx: the
// element-wise state (Adagrad only), srow_old: the row's state (row-wise Adagrad only).  Writes the new
// row (and state, and the replica-store copy if slot >= 0) when `ok`; every lane of the group must call
// it (the row-wise rule sums over the group's lanes).
template <int LG, int DT, int OPT>
struct RowUpdate {
    static constexpr int P = Elems<DT>::N / 4;
    typedef typename Quad<DT>::type quad_t;

    static __device__ __forceinline__ void apply(
        const quad_t* wx, const f32x4* gx, const f32x4* sx, float srow_old, const bool* on, const int* col,
        int64_t r, int64_t D, int lig, bool ok, int slot, float lr, float eps,
        quad_t* wq_out, quad_t* store_out, float* state)
    {
        float s_row = 0.0f;
        if constexpr (OPT == FS_OPT_ADAGRAD_ROWWISE) {
            float sq = 0.0f;
#pragma unroll
            for (int p = 0; p < P; ++p) {
                if (on[p]) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) sq = sq + gx[p][i] * gx[p][i];
                }
            }
#pragma unroll
            for (int off = 1; off < LG; off <<= 1) sq = sq + __shfl_xor(sq, off);
            s_row = srow_old + sq / (float)D;
        }
#pragma unroll
        for (int p = 0; p < P; ++p) {
            float w[4], gf[4], sf[4];
            Quad<DT>::unpack(wx[p], w);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                gf[i] = gx[p][i];
                if constexpr (OPT == FS_OPT_ADAGRAD) sf[i] = sx[p][i];
            }
            apply_rule<4, OPT>(w, gf, sf, s_row, lr, eps);
            if (ok && on[p]) {
                const quad_t out = Quad<DT>::pack(w);
                store_stream(wq_out + ((r * D + col[p]) >> 2), out);
                if (slot >= 0) store_out[((int64_t)slot * D + col[p]) >> 2] = out;
                if constexpr (OPT == FS_OPT_ADAGRAD)
                    store_stream(reinterpret_cast<f32x4*>(state + r * D + col[p]), f32x4{sf[0], sf[1], sf[2], sf[3]});
            }
        }
        if constexpr (OPT == FS_OPT_ADAGRAD_ROWWISE) {
            if (ok && lig == 0) state[r] = s_row;
        }
    }
};

}  // namespace fs
