// Device-side helpers shared by the gfx950 kernels of this library (never by the CPU oracle).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace morph {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16   bf16_t;
typedef __bf16   bf16x8_t __attribute__((ext_vector_type(8)));
typedef float    f32x4   __attribute__((ext_vector_type(4)));
typedef float    f32x16  __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2   __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4   __attribute__((ext_vector_type(4)));

constexpr int kGroup = 128;   // rows of K sharing one scale / zero point

// Raw buffer descriptor over [base, base + bytes): loads that fall outside return 0 and
// stores that fall outside are dropped by the hardware range check, so ragged tiles need
// no per-lane branches.  0x00020000 = DATA_FORMAT_32 for the gfx9 family.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// AUX is the cache-policy operand: 0 = cached, kAuxStream = non-temporal (data read once: do not
// keep it in the caches at the expense of what is reused).
constexpr int kAuxStream = 2;
template <int AUX = 0>
__device__ __forceinline__ uint32_t buf_load_u32(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff)
{
    return __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, AUX);
}
template <int AUX = 0>
__device__ __forceinline__ u32x2 buf_load_u32x2(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff)
{
    return __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, AUX);
}
template <int AUX = 0>
__device__ __forceinline__ u32x4 buf_load_u32x4(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, AUX);
}

template <typename T, typename U>
__device__ __forceinline__ T bit_cast(const U& u)
{
    static_assert(sizeof(T) == sizeof(U), "size");
    return __builtin_bit_cast(T, u);
}

// Byte `y` of `lo_row` into byte 0 and byte `y` of `hi_row` into byte 2; bytes 1 and 3 zero.
// (v_perm_b32: selector 0..3 picks from the second operand, 4..7 from the first, 0x0c gives 0.)
template <int Y>
__device__ __forceinline__ uint32_t pair_bytes(uint32_t lo_row, uint32_t hi_row)
{
    return __builtin_amdgcn_perm(hi_row, lo_row, 0x0c000c00u | ((4u + Y) << 16) | (uint32_t)Y);
}

// fp16 bit tricks for 4-bit codes held in the low byte of each 16-bit half of `p`:
//   (p & 0x000F000F) | 0x6400 per half  = 1024 + low nibble          (ulp of 1024 is 1)
//   (p & 0x00F000F0) | 0x6400 per half  = 1024 + 16 * high nibble
__device__ __forceinline__ half2_t nib_lo_1024(uint32_t p)
{
    return bit_cast<half2_t>((p & 0x000F000Fu) | 0x64006400u);
}
__device__ __forceinline__ half2_t nib_hi_1024(uint32_t p)
{
    return bit_cast<half2_t>((p & 0x00F000F0u) | 0x64006400u);
}

// 16-byte store written through to memory / load served past the caches (system-scope bits sc0 sc1
// on the instruction), for data handed between workgroups inside one kernel.  wait_stores() returns
// once every store of this wave has been acknowledged.
constexpr int kAuxSystemScope = 0x11;    // cache-policy operand of the buffer builtins: sc0 | sc1
__device__ __forceinline__ void buf_store_through(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, f32x4 v)
{
    __builtin_amdgcn_raw_buffer_store_b128(bit_cast<u32x4>(v), r, byte_off, 0, kAuxSystemScope);
}
__device__ __forceinline__ f32x4 buf_load_through(__amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    return bit_cast<f32x4>(__builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, kAuxSystemScope));
}
__device__ __forceinline__ void wait_stores()
{
    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
}

__device__ __forceinline__ float h2f_bits(uint32_t bits16)
{
    return (float)bit_cast<half_t>((uint16_t)bits16);
}

// The 16-bit tensors (x, dense weights, y) are fp16 or, with BF, bfloat16 (the upper half of an
// fp32).  Widening is exact; narrowing rounds once, to nearest even.
template <bool BF>
__device__ __forceinline__ float widen16(uint32_t bits16)
{
    if constexpr (BF) return bit_cast<float>(bits16 << 16);
    else return h2f_bits(bits16);
}
template <bool BF>
__device__ __forceinline__ uint16_t narrow16(float f)
{
    if constexpr (BF) return bit_cast<uint16_t>((bf16_t)f);
    else return bit_cast<uint16_t>((half_t)f);
}

// two fp32 values rounded (to nearest even) into the two bfloat16 halves of a word
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float  f32x2_t  __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return bit_cast<uint32_t>(__builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}
// The two fp16 halves of d, each times the fp32 scale s (exact in fp32), rounded into the two bfloat16
// halves of a word.  Written as fused multiply-adds with a zero addend so that the fp16 operand is
// widened inside the instruction (v_fma_mix_f32) instead of by a conversion of its own.
__device__ __forceinline__ uint32_t scale_to_bf16x2(half2_t d, float s)
{
    return pack_bf16x2(__builtin_fmaf((float)d[0], s, 0.0f), __builtin_fmaf((float)d[1], s, 0.0f));
}

}  // namespace morph
