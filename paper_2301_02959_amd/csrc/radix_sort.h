// Stable LSD radix sort of (uint32 key, uint32 value) pairs, used by the backward
// (key = row, value = position) and by the replication plan (key = inverted count,
// value = row).  Hand-written for 64-lane waves: see radix_sort.hip.
#pragma once

#include "fs_common.h"

namespace fs {

constexpr int kSortItems = 16;                       // keys per thread
constexpr int kSortTile = kBlock * kSortItems;       // keys per block and tile
constexpr int kSortMaxDigitBits = 10;

// Where the first pass reads its pairs from.
//   rows == nullptr: (keys_a, vals_a) hold the pairs.
//   rows != nullptr: pair q is (uint32) rows[q], (uint32) pos[q], validated on the fly
//                    (row outside [0, R) -> 0, pos outside [0, n) -> 0, FS_DEV_BAD_ID into *status);
//                    keys_a / vals_a are then only used as the second buffer.
struct SortSource {
    const int64_t* rows = nullptr;
    const int32_t* pos = nullptr;
    int64_t R = 0;
    int64_t n = 0;
    int32_t* status = nullptr;
};

// Number of passes radix_sort_pairs makes over keys of key_bits bits.
inline int radix_sort_passes(int key_bits)
{
    if (key_bits < 1) key_bits = 1;
    if (key_bits > 32) key_bits = 32;
    return (key_bits + kSortMaxDigitBits - 1) / kSortMaxDigitBits;
}

// Scratch the sort needs for up to m_max pairs (beyond the two key/value buffers).
size_t radix_sort_scratch_bytes(int64_t m_max);

// Sorts pairs by the low `key_bits` bits of the key, stable.  Input in (keys_a, vals_a) or in
// `src`; (keys_b, vals_b) is the other buffer.  The number of pairs is *m_dev if m_dev != nullptr
// (device memory, read by the kernels; must be <= m_max) else m_max.  On return *keys_out /
// *vals_out name the buffer that holds the result.
fs_status radix_sort_pairs(uint32_t* keys_a, uint32_t* vals_a, uint32_t* keys_b, uint32_t* vals_b,
                           int64_t m_max, const int64_t* m_dev, int key_bits, void* scratch,
                           hipStream_t stream, uint32_t** keys_out, uint32_t** vals_out,
                           const SortSource& src = SortSource());

}  // namespace fs
