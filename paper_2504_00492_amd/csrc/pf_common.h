// Device-side building blocks shared by the gfx950 kernels: bf16 conversion, vector types and
// the two facts about v_mfma_f32_16x16x32_bf16 that every kernel here leans on.
//
// MFMA 16x16x32 (one wavefront, lane l, r = l & 15, g = l >> 4):
//   A operand (16 x 32): lane holds A[r][8g .. 8g+7]            (8 consecutive k of row r)
//   B operand (32 x 16): lane holds B[8g .. 8g+7][r]            (8 consecutive k of column r)
//   D / C     (16 x 16): lane holds D[4g .. 4g+3][r] in acc[0..3]
// The contraction only pairs slot (g, e) of A with slot (g, e) of B, so any relabelling of k
// that is applied to both operands leaves the product unchanged.  That is what lets an
// accumulator tile (4 consecutive rows per lane) be fed back as a B operand without moving
// data between lanes: two stacked 16-row accumulator tiles fill slots e = 0..3 and e = 4..7,
// i.e. slot (g, e) carries k = 4g + e (e < 4) or 16 + 4g + (e - 4), and the matching A operand
// is read with the same relabelling.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pf {

typedef __bf16 bf16;
typedef bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b)
{
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// fp32 -> bf16, round to nearest even (v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ bf16x4 cvt4(f32x4 v)
{
    return __builtin_convertvector(v, bf16x4);
}

__device__ __forceinline__ bf16x8 join(bf16x4 lo, bf16x4 hi)
{
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

__device__ __forceinline__ bf16x8 zero8()
{
    bf16x8 z;
#pragma unroll
    for (int e = 0; e < 8; ++e) z[e] = (bf16)0.0f;
    return z;
}

// Typed 8- and 16-byte accesses.  Callers guarantee the alignment.
__device__ __forceinline__ bf16x8 ld8(const bf16 *p) { return *reinterpret_cast<const bf16x8 *>(p); }
__device__ __forceinline__ bf16x4 ld4(const bf16 *p) { return *reinterpret_cast<const bf16x4 *>(p); }
__device__ __forceinline__ void st8(bf16 *p, bf16x8 v) { *reinterpret_cast<bf16x8 *>(p) = v; }
__device__ __forceinline__ void st4(bf16 *p, bf16x4 v) { *reinterpret_cast<bf16x4 *>(p) = v; }

// LDS transposing read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane s hands in
// the address of 4 consecutive 16-bit values; lane l' of the group receives element (l' & 3)
// of the chunks handed in by lanes (l' >> 2), (l' >> 2) + 4, + 8, + 12.  With lane s pointing
// at row (s >> 2), columns 4 (s & 3) .. + 3 of a row-major 4 x 16 block, lane l' therefore
// receives rows 0..3 of column l': four consecutive rows at a fixed column, which is the
// accumulator (and, stacked twice, the B operand) layout of the 16x16x32 MFMA.
__device__ __forceinline__ bf16x4 lds_read_tr4(const bf16 *lds_ptr)
{
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4 *)(uintptr_t)(uint32_t)(uintptr_t)lds_ptr);
    return __builtin_bit_cast(bf16x4, v);
}

}  // namespace pf
