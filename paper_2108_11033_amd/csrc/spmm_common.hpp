// Definitions shared by the SpMM kernel files: vector types, the matrix-core and LDS transpose-read
// wrappers, the LDS swizzle of staged rows and the XCD-aware workgroup id map.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <type_traits>

#include "bcr_matrix.hpp"

namespace grim {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef short i16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int DT> struct Elem;
template <> struct Elem<GRIM_F32> { using type = float; };
template <> struct Elem<GRIM_F16> { using type = _Float16; };
template <> struct Elem<GRIM_BF16> { using type = unsigned short; };

template <int DT> __device__ __forceinline__ float to_f32(typename Elem<DT>::type v);
template <> __device__ __forceinline__ float to_f32<GRIM_F32>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<GRIM_F16>(_Float16 v) { return (float)v; }
template <> __device__ __forceinline__ float to_f32<GRIM_BF16>(unsigned short v) {
    return __builtin_bit_cast(float, (unsigned int)v << 16);
}

template <bool BF16>
__device__ __forceinline__ f32x4 mfma16(i16x8 a, i16x8 b, f32x4 c) {
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <bool BF16>
__device__ __forceinline__ f32x16 mfma32(i16x8 a, i16x8 b, f32x16 c) {
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// LDS transpose read: the 16 lanes of a block each name 8 bytes (4 values along n of one
// staged row); lane i of the block receives value (i % 4) of the chunks named by lanes
// i / 4, 4 + i / 4, 8 + i / 4 and 12 + i / 4 -- four rows at one column, the MFMA k order.
__device__ __forceinline__ i16x4 lds_tr_read_at(unsigned int lds_byte_address) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(uintptr_t)lds_byte_address);
}
__device__ __forceinline__ i16x4 lds_tr_read(const char *lds_addr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(lds_addr));
}

// Staged rows have no padding; the 16-byte chunks of a row are XOR-swizzled by the row
// number so that the four rows one transpose read touches fall into different bank groups
// whenever their numbers differ mod 4 (mod 8 for 128-byte rows, where consecutive rows
// already sit in opposite halves of the 256-byte bank line; measured 3-7 % faster).
template <int CPR>   // 16-byte chunks per staged row
__device__ __forceinline__ int swizzle(int row) {
    return CPR == 8 ? (((row >> 1) & 3) << 1) : CPR > 8 ? ((row & 3) << 1) : (((row >> 1) & 1) << 1);
}

// Waves that split a long strip's steps in the few-workgroups form of the row-gathering kernels.  A 36-step strip of a
// 14 x 14 layer: 8 waves of the product kernel (4 steps per batch) 7.66 us, 12 waves 7.63, 16 waves 8.56; the convolution
// kernel (3 steps per batch) 11.0 us with 8, 8.6 us with 12 -- every wave then needs one batch only --, 9.7 us with 16.
constexpr int kGatherLongWaves = 8, kConvLongWaves = 12;
static_assert(kConvLongWaves == 12, "the launcher names the instantiations");

// Workgroup id -> (tile of columns, unit of the tile's work) for the kernels whose workgroups of one
// tile fetch the same rows: ids are dealt to the 8 XCDs round-robin, each XCD has its own L2, so a
// tile's units go to one XCD.  With that alone the last ntiles % 8 tiles (all of them when there
// are fewer than 8: one tile for N <= 64) would leave XCDs idle, so each of those tiles is cut into
// 2^shift interleaved parts, enough for a multiple of 8, and the parts are dealt instead.
struct XcdMap {
    int32_t per_tile;         // units per tile
    int32_t tail_slot0;       // first slot (id / 8) of the tail tiles
    int32_t tail_tile0;       // first tail tile, a multiple of 8
    int32_t shift;            // tail tiles are cut into 1 << shift parts ...
    int32_t per_part;         // ... of this many units
};
inline XcdMap xcd_map(int32_t ntiles, int64_t per_tile, int64_t *nwg) {
    XcdMap m;
    const int32_t full = ntiles / 8, r = ntiles % 8;
    m.per_tile = (int32_t)per_tile;
    m.tail_slot0 = (int32_t)(full * per_tile);
    m.tail_tile0 = full * 8;
    m.shift = r == 0 ? 0 : r % 4 == 0 ? 1 : r % 2 == 0 ? 2 : 3;
    m.per_part = (int32_t)((per_tile + (1 << m.shift) - 1) >> m.shift);
    *nwg = 8 * (full * per_tile + (int64_t)((r << m.shift) / 8) * m.per_part);
    return m;
}
// false: the workgroup has no tile
__device__ __forceinline__ bool xcd_map_at(const XcdMap &m, int id, int ntiles, int *tile, int *unit) {
    const int xcd = id & 7, slot = id >> 3;
    if (slot < m.tail_slot0) {
        *tile = (slot / m.per_tile) * 8 + xcd;
        *unit = slot % m.per_tile;
        return true;
    }
    const int s2 = slot - m.tail_slot0;
    const int part = (s2 / m.per_part) * 8 + xcd;
    *tile = m.tail_tile0 + (part >> m.shift);
    *unit = ((s2 % m.per_part) << m.shift) + (part & ((1 << m.shift) - 1));
    return *tile < ntiles;
}


}  // namespace grim
