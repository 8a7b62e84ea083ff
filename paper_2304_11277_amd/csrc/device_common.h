// Device-side vocabulary shared by every kernel of libfsdp_flat (gfx950):
// launch constants, kernel-argument pointer tables, 16-byte vector types with
// element alignment, the bf16 / fp16 casts (Sec. 4.4) and the head-peeling helper.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "fsdp_internal.h"

namespace {

constexpr int kBlock = 256;                           // 4 wavefronts of 64 lanes
constexpr int kMaxRanks = FSDP_MAX_RANKS_PER_LAUNCH;  // rank pointers per kernarg table
constexpr int kMaxSegs = 24;                          // parameter segments per pack launch
// launch shapes of the reduce kernels (measured on MI355X)
constexpr int kReduceBlock = 256;
// the prefetch entry point shares one grid only while its smaller half moves at most this many bytes
constexpr int64_t kOneLaunchMaxBytes = 128ll << 20;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
// Same vectors with element alignment only: the compiler may still emit one
// wide access (gfx9 global memory accepts it), never assumes more than this.
typedef f32x4 f32x4_a4 __attribute__((aligned(4)));
typedef u32x4 u32x4_a2 __attribute__((aligned(2)));
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));
typedef u32x2 u32x2_a2 __attribute__((aligned(2)));

struct PtrTable {
    const void* p[kMaxRanks];
};
struct MutPtrTable {
    float* p[kMaxRanks];
};
struct SegTable {
    const float* src[kMaxSegs];   // nullptr = zero fill (the pad)
    int64_t off[kMaxSegs + 1];    // flat offsets, off[i+1] - off[i] = segment length
};

__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }

// fp32 -> bf16, round to nearest, ties to even, on the bit pattern (Sec. 4.4's
// full-to-low precision cast).  NaN keeps sign and top payload bits, forced quiet.
__device__ __forceinline__ uint32_t bf16_rne(uint32_t u)
{
    const bool is_nan = (u & 0x7FFFFFFFu) > 0x7F800000u;
    const uint32_t r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    return is_nan ? ((u >> 16) | 0x0040u) : r;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return bf16_rne(f2u(lo)) | (bf16_rne(f2u(hi)) << 16);
}

// fp32 -> fp16 (IEEE binary16), round to nearest even: the hardware conversion
// (overflow to Inf, subnormal results rounded, not flushed), except that NaN is
// mapped by rule: sign kept, top ten payload bits kept, made quiet.
__device__ __forceinline__ uint32_t f16_rne(uint32_t u)
{
    const bool is_nan = (u & 0x7FFFFFFFu) > 0x7F800000u;
    const _Float16 h = static_cast<_Float16>(u2f(u));
    const uint32_t r = static_cast<uint32_t>(__builtin_bit_cast(uint16_t, h));
    return is_nan ? (((u >> 16) & 0x8000u) | 0x7E00u | ((u >> 13) & 0x03FFu)) : r;
}
// exact fp16 -> fp32
__device__ __forceinline__ float f16_to_f32(uint32_t h16)
{
    return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(h16)));
}

// element kinds of 16-bit / 32-bit buffers (values of fsdp_dtype_t)
constexpr int kF32 = FSDP_F32, kBF16 = FSDP_BF16, kF16 = FSDP_F16;

template <int LP>   // LP = kBF16 or kF16
__device__ __forceinline__ uint32_t cast_lp(float x)
{
    if constexpr (LP == kF16) return f16_rne(f2u(x));
    else return bf16_rne(f2u(x));
}
template <int LP>
__device__ __forceinline__ uint32_t pack_lp2(float lo, float hi)
{
    return cast_lp<LP>(lo) | (cast_lp<LP>(hi) << 16);
}
// exact upcast of the low / high half of a packed pair of 16-bit values
template <int GT>
__device__ __forceinline__ float up_lo(uint32_t pair)
{
    if constexpr (GT == kF16) return f16_to_f32(pair & 0xFFFFu);
    else return u2f(pair << 16);
}
template <int GT>
__device__ __forceinline__ float up_hi(uint32_t pair)
{
    if constexpr (GT == kF16) return f16_to_f32(pair >> 16);
    else return u2f(pair & 0xFFFF0000u);
}

// number of elements (of esize bytes) from p up to the next 16-byte boundary
__device__ __forceinline__ int64_t head_elems(const void* p, int esize, int64_t n)
{
    const uint32_t mis = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(p)) & 15u;
    const int64_t h = ((16u - mis) & 15u) / esize;
    return h < n ? h : n;
}

}  // namespace
