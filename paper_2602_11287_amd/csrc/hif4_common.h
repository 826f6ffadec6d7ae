// Shared device-side helpers of libhif4 (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/hif4.h"

namespace hif4 {

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }

// DPP controls: lane exchange inside groups of 2, 4 and 8 lanes.
constexpr int DPP_XOR1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141; // lane i <-> 7 - i inside each 8 lanes

template <int CTRL>
__device__ __forceinline__ uint32_t dpp(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}

// Packed unsigned 16-bit max of two dwords.
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
}

// Packed unsigned 16-bit min of two dwords.
__device__ __forceinline__ uint32_t pk_min_u16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
}

// Packed 16-bit saturating subtract, shift and fp16 fused multiply-add (VOP3P).
__device__ __forceinline__ uint32_t pk_sub_sat_u16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_sub_sat(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
}

__device__ __forceinline__ uint32_t pk_shl3_u16(uint32_t a)
{
    u16x2 v = __builtin_bit_cast(u16x2, a);
    v = v << (unsigned short)3;
    return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ uint32_t pk_add_f16(uint32_t a, uint32_t b)
{
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 r = __builtin_bit_cast(h2, a) + __builtin_bit_cast(h2, b);
    return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ uint32_t pk_fma_f16(uint32_t a, uint32_t b, uint32_t c)
{
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 r = __builtin_elementwise_fma(__builtin_bit_cast(h2, a), __builtin_bit_cast(h2, b), __builtin_bit_cast(h2, c));
    return __builtin_bit_cast(uint32_t, r);
}

// Three-input bit operations through v_bitop3_b32 (truth table: 0xF0 = first, 0xCC = second, 0xAA = third operand).
// On this chip it issues at the rate of a plain AND (1.3 ns per wave-instruction and SIMD with two or more waves on
// the SIMD), where v_bfi_b32 and v_and_or_b32 take 2.3 - 2.9 ns like shifts to the left, byte permutes, conversions
// and every other three-operand integer instruction (measured with loops of independent instructions).
// Bit-field insert: bits of a where mask is set, bits of b elsewhere.
__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) { return __builtin_amdgcn_bitop3_b32(a, b, mask, 0xE4); }
// x | (y & mask)
__device__ __forceinline__ uint32_t or_and(uint32_t x, uint32_t y, uint32_t mask) { return __builtin_amdgcn_bitop3_b32(x, y, mask, 0xF8); }

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }

// 16-byte and 4-byte global accesses, optionally non-temporal (streaming data that this kernel does not reuse).
template <bool NT>
__device__ __forceinline__ uint4 load16(const void *p)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 *q = static_cast<const u32x4 *>(p);
    u32x4 v = NT ? __builtin_nontemporal_load(q) : *q;
    return make_uint4(v.x, v.y, v.z, v.w);
}

template <bool NT>
__device__ __forceinline__ void store16(void *p, uint4 v)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 t = { v.x, v.y, v.z, v.w };
    if (NT) __builtin_nontemporal_store(t, static_cast<u32x4 *>(p));
    else *static_cast<u32x4 *>(p) = t;
}

template <bool NT>
__device__ __forceinline__ void store4(uint32_t *p, uint32_t v)
{
    if (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// Block -> tile of the dense tile kernels.  Workgroups are dealt to the 8 XCDs round-robin (block b runs on
// XCD b % 8) and each XCD has its own L2, so every XCD gets one contiguous run of the tile list, and the list
// walks the tiles_m x tiles_n grid in bands of 4 tile rows, each band in super-tiles of 4 x 8 tiles (fewer rows
// in the last band, fewer columns in a band's last super-tile): the ~32 workgroups an XCD runs at a time then
// share A rows 8 ways and W rows 4 ways in its L2.  The list holds the grid's tiles only, so the 8 runs are
// equal to within one tile whatever the grid's shape; the grid is tiles_m * tiles_n rounded up to 8 blocks
// (dense_tile_blocks), the surplus blocks get false.
__host__ __device__ inline int64_t dense_tile_blocks(int tiles_m, int tiles_n) { return ((int64_t)tiles_m * tiles_n + 7) / 8 * 8; }

// tile number t of that list (t < tiles_m * tiles_n)
__device__ __forceinline__ void dense_tile_of_index(int t, int tiles_m, int tiles_n, int &tile_m, int &tile_n)
{
    const int band = t / (4 * tiles_n), i = t - band * 4 * tiles_n;
    const int hb = tiles_m - 4 * band < 4 ? tiles_m - 4 * band : 4; // tile rows of this band
    const int full = tiles_n / 8;                                    // its super-tiles of 8 columns
    int sc = i / (hb * 8), wb = 8;
    if (sc >= full) sc = full, wb = tiles_n - 8 * full;
    const int r = i - sc * hb * 8;
    tile_m = 4 * band + r / wb;
    tile_n = 8 * sc + r % wb;
}

__device__ __forceinline__ bool dense_tile_of_block(int tiles_m, int tiles_n, int &tile_m, int &tile_n)
{
    const int per_xcd = (int)(gridDim.x / 8);
    const int t = (int)(blockIdx.x % 8) * per_xcd + (int)(blockIdx.x / 8);
    if (t >= tiles_m * tiles_n) return false;
    dense_tile_of_index(t, tiles_m, tiles_n, tile_m, tile_n);
    return true;
}

// The same list for a kernel whose workgroups stay and take tile after tile: the grid is 8 x `slots` blocks (slots =
// workgroups an XCD runs at a time, at most its share of the tiles), block b is slot b / 8 of XCD b % 8 and takes the
// tiles slot, slot + slots, ... of its XCD's run.  persistent_tile(k, ...) gives its k-th tile, false past the end.
__host__ __device__ inline int persistent_slots(int tiles_m, int tiles_n, int cus_per_xcd)
{
    const int64_t per_xcd = ((int64_t)tiles_m * tiles_n + 7) / 8;
    return (int)(per_xcd < cus_per_xcd ? per_xcd : cus_per_xcd);
}

__device__ __forceinline__ bool persistent_tile(int k, int tiles_m, int tiles_n, int &tile_m, int &tile_n)
{
    const int total = tiles_m * tiles_n, per_xcd = (total + 7) / 8, slots = (int)(gridDim.x / 8);
    const int in_run = (int)(blockIdx.x / 8) + k * slots;
    const int t = (int)(blockIdx.x % 8) * per_xcd + in_run;
    if (in_run >= per_xcd || t >= total) return false;
    dense_tile_of_index(t, tiles_m, tiles_n, tile_m, tile_n);
    return true;
}

} // namespace hif4
