// HIP kernels and launchers of libfsdp_flat for gfx950 (MI355X, CDNA4).
//
// Every step of the FlatParameter data path (arXiv 2304.11277, Sec. 3.2.1,
// 3.2.3, 4.4, eq. (1), Sec. 5.4) is a streaming pass over HBM, so the kernels
// share one shape: each lane moves 16-byte vectors, every load and store
// instruction covers one contiguous span across the wave, a 256-lane workgroup
// owns a contiguous tile, the destination side is always 16-byte aligned
// (ragged heads and tails are peeled off and handled element-wise) and sources
// that are only element-aligned are read through under-aligned vector types or
// realigned through LDS.  Nothing here is a contraction, so there is no MFMA.
//
// Layout of this file: device helpers (casts, vector types); unshard kernels;
// the LDS-staged pack kernel; the reduce-scatter body with its Adam epilogue
// and the kernels built from it (single, one-launch prefetch, batch); Adam;
// gradient accumulation; gradient-scaler bookkeeping; then the host side:
// argument checks, launch helpers and the extern "C" entry points.
//
// Build flags that matter for bit-exactness: -ffp-contract=off (no fused
// multiply-add), IEEE-correct fp32 divide and sqrt (hipcc's default), fp32
// denormals kept (gfx950's default).
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdint>
#include <new>
#include <vector>

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

// ---------------------------------------------------------------------------
// unshard: flat_out[w*S + k] = cast(shard_w[k])   (Sec. 3.2.1 gather, Sec. 4.4 cast)
// grid = nshards * tiles_per_shard blocks; block b serves shard b / tiles and
// tile b % tiles.  A tile is kBlock * U destination vectors of 16 bytes.
// ---------------------------------------------------------------------------
// bid = index of the workgroup among the unshard workgroups of the launch
template <int LP>
__device__ __forceinline__ void unshard_lp_body(const void* const* shards, int64_t S, uint16_t* __restrict__ out_base,
                                                int32_t tiles_per_shard, uint32_t bid)
{
    const int32_t w = bid / tiles_per_shard;
    const int32_t tile = bid - w * tiles_per_shard;
    const float* __restrict__ src = static_cast<const float*>(shards[w]);
    uint16_t* __restrict__ dst = out_base + static_cast<int64_t>(w) * S;

    // A workgroup turns 2048 consecutive floats into 256 destination vectors of
    // 8 values.  Reading them as 32 bytes per lane would make every load
    // instruction touch only every other 16 bytes of its 2 KiB span, so the
    // window goes through LDS instead: 16-byte loads that are contiguous across
    // the wave (taken from the 16-byte boundary at or below the window's start,
    // which also removes any source misalignment), then each lane reads its 8
    // floats back.  Measured 7 % faster than the direct form on MI355X.  Only
    // 16-byte blocks that hold at least one needed float are loaded, so no load
    // leaves the pages of the shard.
    __shared__ __attribute__((aligned(16))) float stage[kBlock * 8 + 8];
    const int64_t head = head_elems(dst, 2, S);
    const int64_t nvec = (S - head) >> 3;                  // full 8-element destination vectors
    const int64_t c0 = static_cast<int64_t>(tile) * kBlock;
    const int t = threadIdx.x;
    const int64_t left = nvec - c0;
    const int32_t nv_tile = left <= 0 ? 0 : (left > kBlock ? kBlock : static_cast<int32_t>(left));   // uniform
    const float* s0 = src + head + (c0 << 3);
    const int32_t shift = static_cast<int32_t>((reinterpret_cast<uintptr_t>(s0) >> 2) & 3);
    if (nv_tile > 0) {
        const f32x4* as = reinterpret_cast<const f32x4*>(s0 - shift);
        const int32_t nload = (nv_tile * 8 + shift + 3) >> 2;   // 16-byte blocks holding at least one needed float
        if (nload >= 2 * kBlock) {                              // full tile: both loads in flight together
            const f32x4 v0 = __builtin_nontemporal_load(as + t);
            const f32x4 v1 = __builtin_nontemporal_load(as + kBlock + t);
            *reinterpret_cast<f32x4*>(stage + 4 * t) = v0;
            *reinterpret_cast<f32x4*>(stage + 4 * (kBlock + t)) = v1;
            if (t == 0 && nload > 2 * kBlock)
                *reinterpret_cast<f32x4*>(stage + 8 * kBlock) = __builtin_nontemporal_load(as + 2 * kBlock);
        } else {
            if (t < nload) *reinterpret_cast<f32x4*>(stage + 4 * t) = __builtin_nontemporal_load(as + t);
            if (t + kBlock < nload)
                *reinterpret_cast<f32x4*>(stage + 4 * (kBlock + t)) = __builtin_nontemporal_load(as + kBlock + t);
        }
    }
    __syncthreads();
    if (t < nv_tile) {
        const float* l = stage + shift + 8 * t;
        u32x4 o;
        o.x = pack_lp2<LP>(l[0], l[1]);
        o.y = pack_lp2<LP>(l[2], l[3]);
        o.z = pack_lp2<LP>(l[4], l[5]);
        o.w = pack_lp2<LP>(l[6], l[7]);
        __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(dst + head + ((c0 + t) << 3)));
    }
    if (tile == 0) {   // ragged head and tail of this shard: at most 7 elements each
        const int64_t tail0 = head + (nvec << 3);
        const int64_t ntail = S - tail0;
        if (t < head) dst[t] = static_cast<uint16_t>(cast_lp<LP>(src[t]));
        if (t >= 64 && t - 64 < ntail) dst[tail0 + t - 64] = static_cast<uint16_t>(cast_lp<LP>(src[tail0 + t - 64]));
    }
}

template <int LP>
__global__ __launch_bounds__(kBlock) void unshard_lp_kernel(PtrTable shards, int64_t S,
                                                             uint16_t* __restrict__ out_base,
                                                             int32_t tiles_per_shard)
{
    unshard_lp_body<LP>(shards.p, S, out_base, tiles_per_shard, blockIdx.x);
}

__global__ __launch_bounds__(kBlock) void unshard_f32_kernel(PtrTable shards, int64_t S,
                                                              float* __restrict__ out_base,
                                                              int32_t tiles_per_shard)
{
    const int32_t w = blockIdx.x / tiles_per_shard;
    const int32_t tile = blockIdx.x - w * tiles_per_shard;
    const float* __restrict__ src = static_cast<const float*>(shards.p[w]);
    float* __restrict__ dst = out_base + static_cast<int64_t>(w) * S;

    const int64_t head = head_elems(dst, 4, S);
    const int64_t nvec = (S - head) >> 2;
    const int64_t c = static_cast<int64_t>(tile) * kBlock + threadIdx.x;
    if (c < nvec) {
        const f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4_a4*>(src + head + (c << 2)));
        __builtin_nontemporal_store(a, reinterpret_cast<f32x4*>(dst + head + (c << 2)));
    }
    if (tile == 0) {
        const int64_t tail0 = head + (nvec << 2);
        const int64_t ntail = S - tail0;
        const int t = threadIdx.x;
        if (t < head) dst[t] = src[t];
        if (t >= 64 && t - 64 < ntail) dst[tail0 + t - 64] = src[tail0 + t - 64];
    }
}

// Gather of bf16 shards (the AllGather in the low precision, Sec. 4.4):
// flat_lp[w*S + k] = lp_shard_w[k]; 16-byte destination vectors, sources only
// 2-byte aligned.
__global__ __launch_bounds__(kBlock) void gather_lp_kernel(PtrTable shards, int64_t S,
                                                            uint16_t* __restrict__ out_base,
                                                            int32_t tiles_per_shard)
{
    const int32_t w = blockIdx.x / tiles_per_shard;
    const int32_t tile = blockIdx.x - w * tiles_per_shard;
    const uint16_t* __restrict__ src = static_cast<const uint16_t*>(shards.p[w]);
    uint16_t* __restrict__ dst = out_base + static_cast<int64_t>(w) * S;

    const int64_t head = head_elems(dst, 2, S);
    const int64_t nvec = (S - head) >> 3;
    const int64_t c = static_cast<int64_t>(tile) * kBlock + threadIdx.x;
    if (c < nvec) {
        const u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const u32x4_a2*>(src + head + (c << 3)));
        __builtin_nontemporal_store(a, reinterpret_cast<u32x4*>(dst + head + (c << 3)));
    }
    if (tile == 0) {
        const int64_t tail0 = head + (nvec << 3);
        const int64_t ntail = S - tail0;
        const int t = threadIdx.x;
        if (t < head) dst[t] = src[t];
        if (t >= 64 && t - 64 < ntail) dst[tail0 + t - 64] = src[tail0 + t - 64];
    }
}

// ---------------------------------------------------------------------------
// flatten + pad + shard (Sec. 3.2.1): LDS-staged ragged pack.
// A block owns one 16-byte-aligned destination tile of kPackTile floats in one
// shard.  It walks the (prefix-summed) segment table for the parameters that
// intersect the tile, copies each piece into LDS with source-aligned 16-byte
// loads, then writes the tile out with destination-aligned 16-byte stores.  A
// segment with a null source is the zero pad.
// ---------------------------------------------------------------------------
constexpr int kPackSlots = 4;                              // 16-byte slots per lane
constexpr int kPackTile = kBlock * kPackSlots * 4;         // floats per tile (16 KiB of LDS)

__global__ __launch_bounds__(kBlock) void pack_kernel(SegTable segs, int32_t nseg, MutPtrTable dsts,
                                                      int32_t w_first, int64_t S, int64_t R0, int64_t R1,
                                                      int32_t tiles_per_shard)
{
    __shared__ __attribute__((aligned(16))) float lds[kPackTile];

    const int32_t wl = blockIdx.x / tiles_per_shard;
    const int32_t tile = blockIdx.x - wl * tiles_per_shard;
    float* __restrict__ dst = dsts.p[wl];
    const int64_t fs = static_cast<int64_t>(w_first + wl) * S;     // flat index of dst[0]
    const int64_t a = (reinterpret_cast<uintptr_t>(dst) >> 2) & 3;  // dst[k] is 16B-aligned iff (k + a) % 4 == 0
    const int64_t t0 = static_cast<int64_t>(tile) * kPackTile - a; // shard-local index of LDS slot 0

    // shard-local element range this block writes
    int64_t k_lo = t0 > 0 ? t0 : 0;
    int64_t k_hi = t0 + kPackTile < S ? t0 + kPackTile : S;
    if (R0 - fs > k_lo) k_lo = R0 - fs;
    if (R1 - fs < k_hi) k_hi = R1 - fs;
    if (k_lo >= k_hi) return;                                       // uniform: whole block leaves
    const int64_t f_lo = fs + k_lo, f_hi = fs + k_hi;
    const int tid = threadIdx.x;

    // stage [f_lo, f_hi) into lds[f - fs - t0]
    int32_t i = 0;
    while (i < nseg && segs.off[i + 1] <= f_lo) ++i;               // uniform scan over <= kMaxSegs entries
    for (; i < nseg && segs.off[i] < f_hi; ++i) {
        const int64_t lo = segs.off[i] > f_lo ? segs.off[i] : f_lo;
        const int64_t hi = segs.off[i + 1] < f_hi ? segs.off[i + 1] : f_hi;
        const int32_t n = static_cast<int32_t>(hi - lo);
        float* l = lds + (lo - fs - t0);
        const float* src = segs.src[i];
        if (src == nullptr) {
            for (int32_t j = tid; j < n; j += kBlock) l[j] = 0.0f;
            continue;
        }
        const float* __restrict__ s = src + (lo - segs.off[i]);
        const int32_t h = static_cast<int32_t>(head_elems(s, 4, n));
        const int32_t nv = (n - h) >> 2;
        if (tid < h) l[tid] = s[tid];
        const int32_t r0 = h + (nv << 2);
        if (tid >= 64 && tid - 64 < n - r0) l[r0 + tid - 64] = s[r0 + tid - 64];
        for (int32_t j0 = 0; j0 < nv; j0 += kBlock * kPackSlots) {
            f32x4 v[kPackSlots];
#pragma unroll
            for (int u = 0; u < kPackSlots; ++u) {
                const int32_t j = j0 + u * kBlock + tid;
                if (j < nv) v[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(s + h + (j << 2)));
            }
#pragma unroll
            for (int u = 0; u < kPackSlots; ++u) {
                const int32_t j = j0 + u * kBlock + tid;
                if (j < nv) {
                    float* q = l + h + (j << 2);
                    q[0] = v[u].x; q[1] = v[u].y; q[2] = v[u].z; q[3] = v[u].w;
                }
            }
        }
    }
    __syncthreads();

    // write out: slot q covers LDS floats [4q, 4q+4) = shard-local [t0 + 4q, t0 + 4q + 4)
#pragma unroll
    for (int u = 0; u < kPackSlots; ++u) {
        const int32_t q = u * kBlock + tid;
        const int64_t k0 = t0 + (q << 2);
        if (k0 >= k_lo && k0 + 4 <= k_hi) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(lds + (q << 2));
            __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(dst + k0));
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (k0 + e >= k_lo && k0 + e < k_hi) dst[k0 + e] = lds[(q << 2) + e];
        }
    }
}

// ---------------------------------------------------------------------------
// reduce-scatter rank share (Sec. 3, eq. (1)) with optional fused Adam (Sec. 5.4)
// ---------------------------------------------------------------------------
struct AdamConsts {
    float beta1, beta2, one_m_b1, one_m_b2, step_size, sqrt_bc2, eps;
};

enum PreMode { kPreNone = 0, kPreMul = 1, kPreDiv = 2 };

// x / pre, exactly: pre == 1 is the identity, a power-of-two pre is a
// multiplication by its (exact) reciprocal, anything else a true division.
template <int PRE>
__device__ __forceinline__ float pre_scale(float x, float c)
{
    if (PRE == kPreNone) return x;
    if (PRE == kPreMul) return x * c;
    return x / c;
}

__device__ __forceinline__ void adam_update(float& p, float g, float& m, float& v, const AdamConsts& c)
{
    const float mk = c.beta1 * m + c.one_m_b1 * g;
    const float vk = c.beta2 * v + c.one_m_b2 * g * g;
    const float denom = sqrtf(vk) / c.sqrt_bc2 + c.eps;
    p = p - c.step_size * (mk / denom);
    m = mk;
    v = vk;
}

// four elements at once; g holds the four gradients
__device__ __forceinline__ void adam_update4(f32x4& p, const float* g, f32x4& m, f32x4& v, const AdamConsts& c)
{
    float pp[4] = {p.x, p.y, p.z, p.w}, mm[4] = {m.x, m.y, m.z, m.w}, vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) adam_update(pp[e], g[e], mm[e], vv[e], c);
    p = f32x4{pp[0], pp[1], pp[2], pp[3]};
    m = f32x4{mm[0], mm[1], mm[2], mm[3]};
    v = f32x4{vv[0], vv[1], vv[2], vv[3]};
}

template <int GT>
__device__ __forceinline__ float load_grad(const void* base, int64_t k)
{
    if constexpr (GT == kF32) return static_cast<const float*>(base)[k];
    else return up_lo<GT>(static_cast<uint32_t>(static_cast<const uint16_t*>(base)[k]));
}

struct RsArgs {
    int32_t W;            // ranks in this launch's table
    int32_t cont;         // 1: accumulator continues from out[] (a later launch of a split W)
    int32_t last;         // 1: apply the post divide (and Adam) in this launch
    int32_t post_mul;     // 1: post is a power of two, post_c holds its exact reciprocal
    int32_t group;        // hybrid sharding: ranks per sharded group (inner sums are folded into an
                          // outer sum after every `group` ranks); 0 = one flat sum
    int32_t accum;        // 1: gradient accumulation, the result is added to what out[] holds
    int32_t unscale;      // 1: gradient scaler: flag non-finite results in *found_inf, then multiply by inv_scale
    float inv_scale;
    float* found_inf;     // one float, set to 1.0f (never cleared) when a non-finite value is seen
    float pre_c;          // pre (kPreDiv) or 1/pre (kPreMul)
    float post_c;         // post, or 1/post when post_mul
    int64_t S;
    float* out;           // grad shard (may be null only when fused and !cont and last)
    float* p;             // Adam state (fused only)
    float* m;
    float* v;
    uint16_t* p_lp;       // optional bf16 copy of the updated p (fused only)
    AdamConsts adam;
};

__device__ __forceinline__ float post_scale(float x, const RsArgs& a)
{
    return a.post_mul ? x * a.post_c : x / a.post_c;
}

// Shape of the rank walk.  A lane owns C chunks of E consecutive elements (E = 4
// for fp32 gradients, 8 for 16-bit ones: one 16-byte load per rank and chunk);
// chunk j of a lane lies B chunks after chunk j-1, so every load instruction is
// contiguous across the wave.  Ranks are taken G at a time, two such batches in
// flight: the next batch's G*C loads are issued before the current batch's adds
// wait for their data, and the adds run strictly in rank order.
//   wide  (G = 4, C = 1): four rank streams per batch.  Best for up to 8 ranks,
//         for small units (it makes the most workgroups) and for 16-bit
//         gradients at any rank count.
//   deep  (G = 1, C = 4): one rank stream at a time, four chunks of it.  Used
//         for fp32 gradients with many ranks, where the wide form loses
//         bandwidth to the number of streams open at once (a lone kernel on
//         MI355X: wide 6.5 TB/s at W = 8, 5.3 TB/s at W = 48; deep 6.4-6.6 TB/s
//         throughout).
// The host pads the pointer table to a multiple of kWideRanks with copies of the
// last pointer, so loads never need a predicate; the padding's adds are skipped.
constexpr int kWideRanks = 4;
template <int GT, bool DEEP>
struct WalkShape {
    static constexpr int E = GT != kF32 ? 8 : 4;
    static constexpr int G = DEEP ? 1 : kWideRanks;
    static constexpr int C = DEEP ? 4 : 1;
};

template <int GT, int G, int C>
__device__ __forceinline__ void load_batch(const void* const* grads, int32_t w0, const int64_t (&k)[C],
                                           u32x4 (&x)[G][C])
{
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int j = 0; j < C; ++j) {
            if constexpr (GT != kF32)
                x[g][j] = __builtin_nontemporal_load(
                    reinterpret_cast<const u32x4_a2*>(static_cast<const uint16_t*>(grads[w0 + g]) + k[j]));
            else
                x[g][j] = __builtin_nontemporal_load(
                    reinterpret_cast<const u32x4_a4*>(static_cast<const float*>(grads[w0 + g]) + k[j]));
        }
    }
}

// Adds the first n ranks of a batch, in rank order, to every chunk.  Hybrid
// sharding (Sec. 3.2.2): acc is the inner sum of the current sharded group;
// after every `group` ranks it is folded into outer and restarted at -0.0f.
template <int GT, int PRE, int G, int C, int E>
__device__ __forceinline__ void add_batch(const u32x4 (&x)[G][C], int32_t n, float pre_c, int32_t group,
                                          int32_t& cnt, float (&acc)[C][E], float (&outer)[C][E])
{
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (g < n) {   // uniform
#pragma unroll
            for (int j = 0; j < C; ++j) {
                float t[E];
                if constexpr (GT != kF32) {   // exact upcast of eight 16-bit gradients
                    t[0] = up_lo<GT>(x[g][j].x); t[1] = up_hi<GT>(x[g][j].x);
                    t[2] = up_lo<GT>(x[g][j].y); t[3] = up_hi<GT>(x[g][j].y);
                    t[4] = up_lo<GT>(x[g][j].z); t[5] = up_hi<GT>(x[g][j].z);
                    t[6] = up_lo<GT>(x[g][j].w); t[7] = up_hi<GT>(x[g][j].w);
                } else {
                    t[0] = u2f(x[g][j].x); t[1] = u2f(x[g][j].y); t[2] = u2f(x[g][j].z); t[3] = u2f(x[g][j].w);
                }
#pragma unroll
                for (int e = 0; e < E; ++e) acc[j][e] = acc[j][e] + pre_scale<PRE>(t[e], pre_c);
            }
            if (group > 0 && ++cnt == group) {   // uniform
#pragma unroll
                for (int j = 0; j < C; ++j) {
#pragma unroll
                    for (int e = 0; e < E; ++e) {
                        outer[j][e] = outer[j][e] + acc[j][e];
                        acc[j][e] = -0.0f;
                    }
                }
                cnt = 0;
            }
        }
    }
}

// The accumulator starts at -0.0f, the identity of IEEE addition ((-0) + x == x
// bit for bit, signed zeros included), which is the same as initialising it
// from rank 0's term; a later launch of a split W starts from the carried
// partial sum instead.  A lane whose later chunks fall past the end computes
// them on a copy of its first chunk (no predicated loads: predicates made the
// compiler serialise them) and skips their stores.
template <int GT, int PRE, bool FUSED, bool DEEP, int B>
__device__ __forceinline__ void reduce_body(const void* const* grads, const RsArgs& a, uint32_t bid)
{
    using Shape = WalkShape<GT, DEEP>;
    constexpr int E = Shape::E, G = Shape::G, C = Shape::C;
    constexpr int Q = E / 4;
    // The chunk grid is aligned on the primary fp32 output.
    float* __restrict__ master = FUSED ? a.p : a.out;
    const int64_t S = a.S;
    const int64_t head = head_elems(master, 4, S);
    const int64_t nvec = (S - head) / E;
    const int64_t c0 = static_cast<int64_t>(bid) * (B * C) + threadIdx.x;
    const int32_t W = a.W;

    if (c0 < nvec) {
        int64_t k[C];
        bool live[C];
#pragma unroll
        for (int j = 0; j < C; ++j) {
            const int64_t cj = c0 + static_cast<int64_t>(j) * B;
            live[j] = cj < nvec;
            k[j] = head + (live[j] ? cj : c0) * E;
        }
        float acc[C][E], outer[C][E];
        int32_t cnt = 0;
#pragma unroll
        for (int j = 0; j < C; ++j) {
            if (a.cont) {
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    const f32x4 t = *reinterpret_cast<const f32x4_a4*>(a.out + k[j] + 4 * q);
                    acc[j][4 * q] = t.x; acc[j][4 * q + 1] = t.y; acc[j][4 * q + 2] = t.z; acc[j][4 * q + 3] = t.w;
                }
            } else {
#pragma unroll
                for (int e = 0; e < E; ++e) acc[j][e] = -0.0f;
            }
#pragma unroll
            for (int e = 0; e < E; ++e) outer[j][e] = -0.0f;
        }

        // The optimizer state (and the accumulated gradient) of the lane's chunks.
        // The wide shape has the registers to fetch it ahead of the rank walk, off
        // the critical path of small launches; the deep shape fetches it after.
        f32x4 pv[C][Q], mv[C][Q], vv[C][Q], old[C][Q];
        auto fetch_state = [&]() {
#pragma unroll
            for (int j = 0; j < C; ++j) {
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    if constexpr (FUSED) {
                        pv[j][q] = *reinterpret_cast<const f32x4*>(a.p + k[j] + 4 * q);
                        mv[j][q] = *reinterpret_cast<const f32x4_a4*>(a.m + k[j] + 4 * q);
                        vv[j][q] = *reinterpret_cast<const f32x4_a4*>(a.v + k[j] + 4 * q);
                    }
                    if (a.accum) old[j][q] = *reinterpret_cast<const f32x4_a4*>(a.out + k[j] + 4 * q);
                }
            }
        };
        if constexpr (!DEEP) fetch_state();

        u32x4 xa[G][C], xb[G][C];
        const int32_t nbatch = (W + G - 1) / G;
        load_batch<GT, G, C>(grads, 0, k, xa);
        for (int32_t b = 0; b < nbatch; b += 2) {
            const bool has_b = b + 1 < nbatch;
            if (has_b) load_batch<GT, G, C>(grads, (b + 1) * G, k, xb);
            add_batch<GT, PRE, G, C, E>(xa, W - b * G, a.pre_c, a.group, cnt, acc, outer);
            if (b + 2 < nbatch) load_batch<GT, G, C>(grads, (b + 2) * G, k, xa);
            if (has_b) add_batch<GT, PRE, G, C, E>(xb, W - (b + 1) * G, a.pre_c, a.group, cnt, acc, outer);
        }

        if constexpr (DEEP) fetch_state();
#pragma unroll
        for (int j = 0; j < C; ++j) {
            if (!live[j]) continue;
            float (&r)[E] = acc[j];
            if (a.group > 0) {   // every sharded group has been folded: the outer sum is the result
#pragma unroll
                for (int e = 0; e < E; ++e) r[e] = outer[j][e];
            }
            if (a.last) {
#pragma unroll
                for (int e = 0; e < E; ++e) r[e] = post_scale(r[e], a);
            }
            if (a.accum) {
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    r[4 * q] = old[j][q].x + r[4 * q];
                    r[4 * q + 1] = old[j][q].y + r[4 * q + 1];
                    r[4 * q + 2] = old[j][q].z + r[4 * q + 2];
                    r[4 * q + 3] = old[j][q].w + r[4 * q + 3];
                }
            }
            if (a.unscale) {   // sharded gradient scaler (Sec. 4.4): check, then unscale
                bool bad = false;
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    bad |= (f2u(r[e]) & 0x7F800000u) == 0x7F800000u;
                    r[e] = r[e] * a.inv_scale;
                }
                if (bad) *a.found_inf = 1.0f;
            }
            if (a.out != nullptr) {
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    f32x4 o = {r[4 * q], r[4 * q + 1], r[4 * q + 2], r[4 * q + 3]};
                    *reinterpret_cast<f32x4_a4*>(a.out + k[j] + 4 * q) = o;
                }
            }
            if constexpr (FUSED) {
                uint32_t lp[E / 2];
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    adam_update4(pv[j][q], &r[4 * q], mv[j][q], vv[j][q], a.adam);
                    *reinterpret_cast<f32x4*>(a.p + k[j] + 4 * q) = pv[j][q];
                    *reinterpret_cast<f32x4_a4*>(a.m + k[j] + 4 * q) = mv[j][q];
                    *reinterpret_cast<f32x4_a4*>(a.v + k[j] + 4 * q) = vv[j][q];
                    lp[2 * q] = pack_bf16x2(pv[j][q].x, pv[j][q].y);
                    lp[2 * q + 1] = pack_bf16x2(pv[j][q].z, pv[j][q].w);
                }
                if (a.p_lp != nullptr) {
                    if constexpr (E == 8) {
                        u32x4 o = {lp[0], lp[1], lp[2], lp[3]};
                        *reinterpret_cast<u32x4_a2*>(a.p_lp + k[j]) = o;
                    } else {
                        u32x2 o = {lp[0], lp[1]};
                        *reinterpret_cast<u32x2_a2*>(a.p_lp + k[j]) = o;
                    }
                }
            }
        }
    }

    // ragged head / tail (fewer than 4 + E elements in total): one lane per element
    if (bid == 0) {
        const int64_t tail0 = head + nvec * E;
        const int64_t nrag = head + (S - tail0);
        const int t = threadIdx.x;
        if (t < nrag) {
            const int64_t k = t < head ? t : tail0 + (t - head);
            const float old_r = a.accum ? a.out[k] : 0.0f;
            float r = a.cont ? a.out[k] : -0.0f;
            float outer_r = -0.0f;
            int32_t cnt = 0;
            for (int32_t w = 0; w < W; ++w) {
                r = r + pre_scale<PRE>(load_grad<GT>(grads[w], k), a.pre_c);
                if (a.group > 0 && ++cnt == a.group) {
                    outer_r = outer_r + r;
                    r = -0.0f;
                    cnt = 0;
                }
            }
            if (a.group > 0) r = outer_r;
            if (a.last) r = post_scale(r, a);
            if (a.accum) r = old_r + r;
            if (a.unscale) {
                if ((f2u(r) & 0x7F800000u) == 0x7F800000u) *a.found_inf = 1.0f;
                r = r * a.inv_scale;
            }
            if (a.out != nullptr) a.out[k] = r;
            if constexpr (FUSED) {
                float pk = a.p[k], mk = a.m[k], vk = a.v[k];
                adam_update(pk, r, mk, vk, a.adam);
                a.p[k] = pk; a.m[k] = mk; a.v[k] = vk;
                if (a.p_lp != nullptr) a.p_lp[k] = static_cast<uint16_t>(bf16_rne(f2u(pk)));
            }
        }
    }
}

template <int GT, int PRE, bool FUSED, bool DEEP, int B>
__global__ __launch_bounds__(B) void reduce_kernel(PtrTable grads, RsArgs a)
{
    reduce_body<GT, PRE, FUSED, DEEP, B>(grads.p, a, blockIdx.x);
}

// Backward prefetching (Sec. 3.3.2) as one launch: the first n_reduce
// workgroups run the fused reduce-scatter + Adam of one unit, the rest the
// unshard of another unit.  The two do not depend on each other, so sharing a
// grid lets the drain of one overlap the ramp of the other without any
// cross-queue synchronisation.
template <int GT, int PRE>
__global__ __launch_bounds__(kBlock) void reduce_adam_unshard_kernel(PtrTable grads, RsArgs a, uint32_t n_reduce,
                                                                      PtrTable shards, int64_t S_next,
                                                                      uint16_t* __restrict__ out_base,
                                                                      int32_t tiles_per_shard)
{
    if (blockIdx.x < n_reduce)
        reduce_body<GT, PRE, true, false, kBlock>(grads.p, a, blockIdx.x);
    else
        unshard_lp_body<kBF16>(shards.p, S_next, out_base, tiles_per_shard, blockIdx.x - n_reduce);
}

// ---------------------------------------------------------------------------
// Batches of independent operations in one grid: up to kBatchOps fused
// reduce-scatter + Adam operations and up to kBatchOps unshards of other units.
// One launch floor for the whole batch, and the ramp and drain of the members
// overlap.  Workgroups [0, r_end[n_reduce-1]) serve the reduce operations in
// order, the rest the unshards.
// ---------------------------------------------------------------------------
constexpr int kBatchOps = 3;
constexpr int kBatchRanks = 32;    // rank pointers per batched operation

struct BatchReduceOp {
    const void* grads[kBatchRanks];
    RsArgs a;
};
struct BatchUnshardOp {
    const void* shards[kBatchRanks];
    int64_t S;
    uint16_t* out;
    int32_t tiles;
    int32_t pad_;
};
struct BatchArgs {
    int32_t n_reduce, n_unshard;
    uint32_t r_end[kBatchOps];     // exclusive end of each reduce operation's workgroup range
    uint32_t u_end[kBatchOps];     // same for the unshards, counted from the end of the reduce ranges
    BatchReduceOp r[kBatchOps];
    BatchUnshardOp u[kBatchOps];
};

template <int GT, int PRE>
__global__ __launch_bounds__(kBlock) void batch_kernel(BatchArgs b)
{
    uint32_t bid = blockIdx.x;
    const uint32_t n_red_blocks = b.n_reduce > 0 ? b.r_end[b.n_reduce - 1] : 0u;
    if (bid < n_red_blocks) {
        int32_t i = 0;
        uint32_t start = 0;
        while (bid >= b.r_end[i]) { start = b.r_end[i]; ++i; }     // uniform, at most kBatchOps - 1 steps
        reduce_body<GT, PRE, true, false, kBlock>(b.r[i].grads, b.r[i].a, bid - start);
    } else {
        bid -= n_red_blocks;
        int32_t i = 0;
        uint32_t start = 0;
        while (bid >= b.u_end[i]) { start = b.u_end[i]; ++i; }
        unshard_lp_body<kBF16>(b.u[i].shards, b.u[i].S, b.u[i].out, b.u[i].tiles, bid - start);
    }
}

// ---------------------------------------------------------------------------
// Adam on the shard (Sec. 5.4; state sharded as in Sec. 3)
// ---------------------------------------------------------------------------
// skip: optional device flag of the gradient scaler (Sec. 4.4); when it holds a
// non-zero value the step is skipped and p, m, v stay as they are.
__global__ __launch_bounds__(kBlock) void adam_kernel(float* __restrict__ p, const float* __restrict__ g,
                                                       float* __restrict__ m, float* __restrict__ v,
                                                       int64_t S, AdamConsts c, const float* __restrict__ skip)
{
    if (skip != nullptr && *skip != 0.0f) return;     // uniform over the whole grid
    const int64_t head = head_elems(p, 4, S);
    const int64_t nvec = (S - head) >> 2;
    const int64_t cidx = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (cidx < nvec) {
        const int64_t k = head + (cidx << 2);
        f32x4 pv = *reinterpret_cast<const f32x4*>(p + k);
        const f32x4 gv = __builtin_nontemporal_load(reinterpret_cast<const f32x4_a4*>(g + k));
        f32x4 mv = *reinterpret_cast<const f32x4_a4*>(m + k);
        f32x4 vv = *reinterpret_cast<const f32x4_a4*>(v + k);
        const float gg[4] = {gv.x, gv.y, gv.z, gv.w};
        adam_update4(pv, gg, mv, vv, c);
        *reinterpret_cast<f32x4*>(p + k) = pv;
        *reinterpret_cast<f32x4_a4*>(m + k) = mv;
        *reinterpret_cast<f32x4_a4*>(v + k) = vv;
    }
    if (blockIdx.x == 0) {
        const int64_t tail0 = head + (nvec << 2);
        const int64_t nrag = head + (S - tail0);
        const int t = threadIdx.x;
        if (t < nrag) {
            const int64_t k = t < head ? t : tail0 + (t - head);
            float pk = p[k], mk = m[k], vk = v[k];
            adam_update(pk, g[k], mk, vk, c);
            p[k] = pk; m[k] = mk; v[k] = vk;
        }
    }
}

// ---------------------------------------------------------------------------
// gradient accumulation without communication (Sec. 3.3.4): acc[k] += add[k]
// over the unsharded buffer; one binary32 addition per element
// ---------------------------------------------------------------------------
template <int GT>
__global__ __launch_bounds__(kBlock) void accumulate_kernel(float* __restrict__ acc, const void* __restrict__ add,
                                                             int64_t n)
{
    const int64_t head = head_elems(acc, 4, n);
    const int64_t nvec = (n - head) >> 2;
    const int64_t c = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (c < nvec) {
        const int64_t k = head + (c << 2);
        f32x4 a = *reinterpret_cast<const f32x4*>(acc + k);
        f32x4 b;
        if constexpr (GT != kF32) {
            const u32x2 h = __builtin_nontemporal_load(
                reinterpret_cast<const u32x2_a2*>(static_cast<const uint16_t*>(add) + k));
            b = f32x4{up_lo<GT>(h.x), up_hi<GT>(h.x), up_lo<GT>(h.y), up_hi<GT>(h.y)};
        } else {
            b = __builtin_nontemporal_load(reinterpret_cast<const f32x4_a4*>(static_cast<const float*>(add) + k));
        }
        a = a + b;
        *reinterpret_cast<f32x4*>(acc + k) = a;
    }
    if (blockIdx.x == 0) {
        const int64_t tail0 = head + (nvec << 2);
        const int64_t nrag = head + (n - tail0);
        const int t = threadIdx.x;
        if (t < nrag) {
            const int64_t k = t < head ? t : tail0 + (t - head);
            acc[k] = acc[k] + load_grad<GT>(add, k);
        }
    }
}

// ---------------------------------------------------------------------------
// gradient scaler bookkeeping (Sec. 4.4): tiny single-lane kernels so that no
// host round trip is needed between the reduce-scatter and the optimizer step
// ---------------------------------------------------------------------------
struct FlagTable {
    float* p[kMaxRanks];
};

// every rank's flag becomes the maximum of all flags (the all-reduce of found_inf)
__global__ void found_inf_combine_kernel(FlagTable flags, int32_t n)
{
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    float m = 0.0f;
    for (int32_t i = 0; i < n; ++i) {
        const float f = *flags.p[i];
        if (f > m) m = f;
    }
    for (int32_t i = 0; i < n; ++i) *flags.p[i] = m;
}

__global__ void scaler_update_kernel(float* scale, int32_t* growth_tracker, const float* found_inf, float growth,
                                     float backoff, int32_t growth_interval)
{
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    if (*found_inf != 0.0f) {
        *scale = *scale * backoff;
        *growth_tracker = 0;
    } else {
        int32_t t = *growth_tracker + 1;
        if (t == growth_interval) {
            *scale = *scale * growth;
            t = 0;
        }
        *growth_tracker = t;
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
int launch_status()
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        fsdp::set_last_hip_error(static_cast<int>(e));
        return FSDP_ERR_HIP;
    }
    return FSDP_OK;
}

inline bool misaligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Blocks of a 1-D grid must fit HIP's 2^31 - 1 limit; with >= 4 KiB per block
// that is > 8 TB of data, far beyond the 288 GB of HBM, but check anyway.
inline bool grid_ok(int64_t blocks) { return blocks > 0 && blocks <= 0x7FFFFFFFLL; }

bool is_pow2_float(float x, float* recip)
{
    int e = 0;
    const float m = std::frexp(x, &e);       // x = m * 2^e, m in [0.5, 1)
    if (m != 0.5f) return false;
    const float r = 1.0f / x;                 // exact for a power of two unless it leaves the normal range
    if (!std::isfinite(r) || r == 0.0f || std::fpclassify(r) == FP_SUBNORMAL || std::fpclassify(x) == FP_SUBNORMAL)
        return false;
    *recip = r;
    return true;
}

int check_adam_args(int64_t step, float lr, float b1, float b2, float eps)
{
    if (step < 1) return FSDP_ERR_INVALID_ARG;
    if (!std::isfinite(lr)) return FSDP_ERR_INVALID_ARG;
    if (!(b1 >= 0.0f && b1 < 1.0f) || !(b2 >= 0.0f && b2 < 1.0f)) return FSDP_ERR_INVALID_ARG;
    if (!(eps >= 0.0f) || !std::isfinite(eps)) return FSDP_ERR_INVALID_ARG;
    return FSDP_OK;
}

AdamConsts make_adam_consts(int64_t step, float lr, float b1, float b2, float eps)
{
    AdamConsts c;
    const float bc1 = static_cast<float>(1.0 - std::pow(static_cast<double>(b1), static_cast<double>(step)));
    const float bc2 = static_cast<float>(1.0 - std::pow(static_cast<double>(b2), static_cast<double>(step)));
    c.beta1 = b1;
    c.beta2 = b2;
    c.one_m_b1 = 1.0f - b1;
    c.one_m_b2 = 1.0f - b2;
    c.step_size = lr / bc1;
    c.sqrt_bc2 = std::sqrt(bc2);
    c.eps = eps;
    return c;
}

// the wide rank walk loads whole batches of kWideRanks ranks: repeat the last pointer up to the batch boundary
void pad_rank_table(PtrTable& tab, int32_t n)
{
    static_assert(kMaxRanks % kWideRanks == 0, "the padded table must fit");
    for (int32_t j = n; j % kWideRanks != 0; ++j) tab.p[j] = tab.p[n - 1];
}

// The deep rank walk pays for fp32 gradients from about ten rank streams on
// (4 % at 12 ranks), provided it still makes at least four workgroups per
// compute unit (256 of them on MI355X).
constexpr int32_t kDeepMinRanks = 10;
constexpr int64_t kDeepMinBlocks = 4 * 256;
std::atomic<int32_t> g_reduce_walk{FSDP_WALK_AUTO};      // fsdp_set_reduce_walk

template <int GT, int PRE, bool FUSED>
void launch_reduce(const PtrTable& tab, const RsArgs& a, hipStream_t st)
{
    constexpr int B = kReduceBlock;
    constexpr int E = WalkShape<GT, false>::E;
    if constexpr (GT == kF32) {   // 16-bit gradients measured no gain from the deep walk (6 % slower at 64 ranks)
        const int64_t deep_blocks = ceil_div(a.S / E + 1, B * WalkShape<GT, true>::C);
        const int32_t walk = g_reduce_walk.load(std::memory_order_relaxed);
        const bool deep = walk == FSDP_WALK_AUTO ? a.W >= kDeepMinRanks && deep_blocks >= kDeepMinBlocks
                                                 : walk == FSDP_WALK_DEEP;
        if (deep) {
            hipLaunchKernelGGL((reduce_kernel<GT, PRE, FUSED, true, B>), dim3(static_cast<uint32_t>(deep_blocks)),
                               dim3(B), 0, st, tab, a);
            return;
        }
    }
    const int64_t blocks = ceil_div(a.S / E + 1, B);
    hipLaunchKernelGGL((reduce_kernel<GT, PRE, FUSED, false, B>), dim3(static_cast<uint32_t>(blocks)), dim3(B), 0, st,
                       tab, a);
}

template <int GT, bool FUSED>
void launch_reduce_pre(int pre_mode, const PtrTable& tab, const RsArgs& a, hipStream_t st)
{
    if (pre_mode == kPreNone) launch_reduce<GT, kPreNone, FUSED>(tab, a, st);
    else if (pre_mode == kPreMul) launch_reduce<GT, kPreMul, FUSED>(tab, a, st);
    else launch_reduce<GT, kPreDiv, FUSED>(tab, a, st);
}

inline bool valid_dtype(fsdp_dtype_t d) { return d == FSDP_F32 || d == FSDP_BF16 || d == FSDP_F16; }
inline int64_t dtype_size(fsdp_dtype_t d) { return d == FSDP_F32 ? 4 : 2; }

// shared driver of fsdp_reduce_scatter_local and fsdp_reduce_scatter_adam_fused
struct ReduceOpts {
    int32_t num_groups = 1;      // hybrid sharding: sharded groups of L->world_size ranks, table group-major
    bool accumulate = false;     // add the result to what the output buffer holds
    bool unscale = false;        // gradient scaler: non-finite check + multiply by inv_scale
    float inv_scale = 1.0f;
    float* found_inf = nullptr;
};

// shared driver of the reduce-scatter entry points
int reduce_driver(const fsdp_layout_t* L, const void* const* grad_ptrs, fsdp_dtype_t grad_dtype, int32_t rank,
                  float pre, float post, float* out, bool fused, float* p, float* m, float* v, uint16_t* p_lp,
                  const AdamConsts& adam, hipStream_t st, const ReduceOpts& opt = ReduceOpts())
{
    const int32_t W = L->world_size * opt.num_groups;
    // these variants keep their state in one launch
    if ((opt.num_groups > 1 || opt.accumulate || opt.unscale) && W > kMaxRanks) return FSDP_ERR_INVALID_ARG;
    const int64_t S = L->S;
    const int64_t esz = dtype_size(grad_dtype);
    if (!grid_ok(ceil_div(S / 4 + 1, kBlock))) return FSDP_ERR_OVERFLOW;

    float pre_c = pre;
    int pre_mode = kPreDiv;
    float recip;
    if (pre == 1.0f) pre_mode = kPreNone;
    else if (is_pow2_float(pre, &recip)) { pre_mode = kPreMul; pre_c = recip; }
    float post_c = post;
    int32_t post_mul = 0;
    if (is_pow2_float(post, &recip)) { post_mul = 1; post_c = recip; }

    for (int32_t w0 = 0; w0 < W; w0 += kMaxRanks) {
        const int32_t nw = W - w0 < kMaxRanks ? W - w0 : kMaxRanks;
        PtrTable tab = {};
        for (int32_t j = 0; j < nw; ++j)
            tab.p[j] = static_cast<const char*>(grad_ptrs[w0 + j]) + static_cast<int64_t>(rank) * S * esz;
        pad_rank_table(tab, nw);
        RsArgs a = {};
        a.W = nw;
        a.cont = w0 > 0;
        a.last = w0 + nw == W;
        a.group = opt.num_groups > 1 ? L->world_size : 0;
        a.accum = opt.accumulate ? 1 : 0;
        a.unscale = opt.unscale ? 1 : 0;
        a.inv_scale = opt.inv_scale;
        a.found_inf = opt.found_inf;
        a.pre_c = pre_c;
        a.post_mul = post_mul;
        a.post_c = post_c;
        a.S = S;
        a.out = out;
        a.p = p; a.m = m; a.v = v; a.p_lp = p_lp;
        a.adam = adam;
        const bool fuse_now = fused && a.last;
        if (grad_dtype == FSDP_BF16) {
            if (fuse_now) launch_reduce_pre<kBF16, true>(pre_mode, tab, a, st);
            else launch_reduce_pre<kBF16, false>(pre_mode, tab, a, st);
        } else if (grad_dtype == FSDP_F16) {
            if (fuse_now) launch_reduce_pre<kF16, true>(pre_mode, tab, a, st);
            else launch_reduce_pre<kF16, false>(pre_mode, tab, a, st);
        } else {
            if (fuse_now) launch_reduce_pre<kF32, true>(pre_mode, tab, a, st);
            else launch_reduce_pre<kF32, false>(pre_mode, tab, a, st);
        }
        const int rc = launch_status();
        if (rc != FSDP_OK) return rc;
    }
    return FSDP_OK;
}

int check_reduce_args(const fsdp_layout_t* L, const void* const* grad_ptrs, fsdp_dtype_t grad_dtype, int32_t rank,
                      float pre, float post, int32_t num_groups = 1)
{
    if (!L || !grad_ptrs) return FSDP_ERR_NULL_PTR;
    if (num_groups < 1) return FSDP_ERR_INVALID_ARG;
    if (!valid_dtype(grad_dtype)) return FSDP_ERR_BAD_DTYPE;
    if (rank < 0 || rank >= L->world_size) return FSDP_ERR_RANK_RANGE;
    if (!std::isfinite(pre) || !std::isfinite(post) || !(pre > 0.0f) || !(post > 0.0f)) return FSDP_ERR_INVALID_ARG;
    const uintptr_t al = static_cast<uintptr_t>(dtype_size(grad_dtype));
    const int64_t nptr = static_cast<int64_t>(L->world_size) * num_groups;
    if (nptr > 0x7FFFFFFF) return FSDP_ERR_OVERFLOW;
    for (int64_t w = 0; w < nptr; ++w) {
        if (!grad_ptrs[w]) return FSDP_ERR_NULL_PTR;
        if (misaligned(grad_ptrs[w], al)) return FSDP_ERR_INVALID_ARG;
    }
    return FSDP_OK;
}

}  // namespace

extern "C" {

int fsdp_set_reduce_walk(int32_t walk)
{
    if (walk != FSDP_WALK_AUTO && walk != FSDP_WALK_WIDE && walk != FSDP_WALK_DEEP) return FSDP_ERR_INVALID_ARG;
    g_reduce_walk.store(walk, std::memory_order_relaxed);
    return FSDP_OK;
}

int fsdp_flatten_shard(const fsdp_layout_t* L, const void* const* param_ptrs, float* const* shard_ptrs,
                       void* hip_stream)
{
    if (!L || !param_ptrs || !shard_ptrs) return FSDP_ERR_NULL_PTR;
    const int32_t W = L->world_size;
    const int64_t S = L->S;
    for (int32_t i = 0; i < L->num_params; ++i) {
        if (L->numel[i] == 0) continue;
        if (!param_ptrs[i]) return FSDP_ERR_NULL_PTR;
        if (misaligned(param_ptrs[i], 4)) return FSDP_ERR_INVALID_ARG;
    }
    for (int32_t w = 0; w < W; ++w) {
        if (!shard_ptrs[w]) return FSDP_ERR_NULL_PTR;
        if (misaligned(shard_ptrs[w], 4)) return FSDP_ERR_INVALID_ARG;
    }
    const int64_t tiles = ceil_div(S + 3, kPackTile);
    if (!grid_ok(tiles * kMaxRanks)) return FSDP_ERR_OVERFLOW;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);

    // Non-empty segments in flat order: the parameters, then the pad.
    std::vector<const float*> seg_src;
    std::vector<int64_t> seg_off;
    try {
        for (int32_t i = 0; i < L->num_params; ++i) {
            if (L->numel[i] == 0) continue;
            seg_src.push_back(static_cast<const float*>(param_ptrs[i]));
            seg_off.push_back(L->off[i]);
        }
        if (L->pad > 0) {
            seg_src.push_back(nullptr);
            seg_off.push_back(L->N);
        }
        seg_off.push_back(L->P);
    } catch (const std::bad_alloc&) {
        return FSDP_ERR_OOM;
    }
    const int64_t nsegs = static_cast<int64_t>(seg_src.size());

    // One launch covers the flat range where a batch of <= kMaxSegs segments
    // meets a batch of <= kMaxRanks shards.
    for (int64_t s0 = 0; s0 < nsegs; s0 += kMaxSegs) {
        const int32_t ns = static_cast<int32_t>(nsegs - s0 < kMaxSegs ? nsegs - s0 : kMaxSegs);
        SegTable segs = {};
        for (int32_t j = 0; j < ns; ++j) {
            segs.src[j] = seg_src[s0 + j];
            segs.off[j] = seg_off[s0 + j];
        }
        segs.off[ns] = seg_off[s0 + ns];
        const int64_t B0 = segs.off[0], B1 = segs.off[ns];
        const int32_t wa = static_cast<int32_t>(B0 / S), wb = static_cast<int32_t>((B1 - 1) / S);
        for (int32_t w0 = wa; w0 <= wb; w0 += kMaxRanks) {
            const int32_t nw = wb - w0 + 1 < kMaxRanks ? wb - w0 + 1 : kMaxRanks;
            MutPtrTable dsts = {};
            for (int32_t j = 0; j < nw; ++j) dsts.p[j] = shard_ptrs[w0 + j];
            const int64_t lo = static_cast<int64_t>(w0) * S, hi = static_cast<int64_t>(w0 + nw) * S;
            const int64_t R0 = B0 > lo ? B0 : lo, R1 = B1 < hi ? B1 : hi;
            hipLaunchKernelGGL(pack_kernel, dim3(static_cast<uint32_t>(tiles * nw)), dim3(kBlock), 0, st, segs, ns,
                               dsts, w0, S, R0, R1, static_cast<int32_t>(tiles));
            const int rc = launch_status();
            if (rc != FSDP_OK) return rc;
        }
    }
    return FSDP_OK;
}

int fsdp_unshard(const fsdp_layout_t* L, const float* const* shard_ptrs, void* flat_out, fsdp_dtype_t out_dtype,
                 void* hip_stream)
{
    if (!L || !shard_ptrs || !flat_out) return FSDP_ERR_NULL_PTR;
    if (!valid_dtype(out_dtype)) return FSDP_ERR_BAD_DTYPE;
    const int32_t W = L->world_size;
    const int64_t S = L->S;
    for (int32_t w = 0; w < W; ++w) {
        if (!shard_ptrs[w]) return FSDP_ERR_NULL_PTR;
        if (misaligned(shard_ptrs[w], 4)) return FSDP_ERR_INVALID_ARG;
    }
    const bool lp = out_dtype != FSDP_F32;
    if (misaligned(flat_out, lp ? 2 : 4)) return FSDP_ERR_INVALID_ARG;
    // One destination vector per lane measured fastest on MI355X for the cast
    // (more, shorter workgroups hide the ramp of small units better).
    const int64_t vec = lp ? 8 : 4;
    const int64_t tiles = ceil_div(S / vec + 1, kBlock);
    if (!grid_ok(tiles * kMaxRanks)) return FSDP_ERR_OVERFLOW;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);

    for (int32_t w0 = 0; w0 < W; w0 += kMaxRanks) {
        const int32_t nw = W - w0 < kMaxRanks ? W - w0 : kMaxRanks;
        PtrTable tab = {};
        for (int32_t j = 0; j < nw; ++j) tab.p[j] = shard_ptrs[w0 + j];
        const dim3 grid(static_cast<uint32_t>(tiles * nw));
        if (lp) {
            uint16_t* base = static_cast<uint16_t*>(flat_out) + static_cast<int64_t>(w0) * S;
            if (out_dtype == FSDP_F16)
                hipLaunchKernelGGL(unshard_lp_kernel<kF16>, grid, dim3(kBlock), 0, st, tab, S, base,
                                   static_cast<int32_t>(tiles));
            else
                hipLaunchKernelGGL(unshard_lp_kernel<kBF16>, grid, dim3(kBlock), 0, st, tab, S, base,
                                   static_cast<int32_t>(tiles));
        } else {
            float* base = static_cast<float*>(flat_out) + static_cast<int64_t>(w0) * S;
            hipLaunchKernelGGL(unshard_f32_kernel, grid, dim3(kBlock), 0, st, tab, S, base,
                               static_cast<int32_t>(tiles));
        }
        const int rc = launch_status();
        if (rc != FSDP_OK) return rc;
    }
    return FSDP_OK;
}

int fsdp_reduce_scatter_local(const fsdp_layout_t* L, const void* const* grad_ptrs, fsdp_dtype_t grad_dtype,
                              int32_t rank, float pre_div, float post_div, float* grad_shard_out, void* hip_stream)
{
    int rc = check_reduce_args(L, grad_ptrs, grad_dtype, rank, pre_div, post_div);
    if (rc != FSDP_OK) return rc;
    if (!grad_shard_out) return FSDP_ERR_NULL_PTR;
    if (misaligned(grad_shard_out, 4)) return FSDP_ERR_INVALID_ARG;
    const AdamConsts none = {};
    return reduce_driver(L, grad_ptrs, grad_dtype, rank, pre_div, post_div, grad_shard_out, false, nullptr, nullptr,
                         nullptr, nullptr, none, static_cast<hipStream_t>(hip_stream));
}

static int adam_step_impl(const fsdp_layout_t* L, float* p_shard, const float* g_shard, float* exp_avg,
                          float* exp_avg_sq, int64_t step, float lr, float beta1, float beta2, float eps,
                          const float* skip, void* hip_stream)
{
    if (!L || !p_shard || !g_shard || !exp_avg || !exp_avg_sq) return FSDP_ERR_NULL_PTR;
    int rc = check_adam_args(step, lr, beta1, beta2, eps);
    if (rc != FSDP_OK) return rc;
    if (misaligned(p_shard, 4) || misaligned(g_shard, 4) || misaligned(exp_avg, 4) || misaligned(exp_avg_sq, 4) ||
        (skip && misaligned(skip, 4)))
        return FSDP_ERR_INVALID_ARG;
    const int64_t blocks = ceil_div(L->S / 4 + 1, kBlock);
    if (!grid_ok(blocks)) return FSDP_ERR_OVERFLOW;
    const AdamConsts c = make_adam_consts(step, lr, beta1, beta2, eps);
    hipLaunchKernelGGL(adam_kernel, dim3(static_cast<uint32_t>(blocks)), dim3(kBlock), 0,
                       static_cast<hipStream_t>(hip_stream), p_shard, g_shard, exp_avg, exp_avg_sq, L->S, c, skip);
    return launch_status();
}

int fsdp_shard_adam_step(const fsdp_layout_t* L, float* p_shard, const float* g_shard, float* exp_avg,
                         float* exp_avg_sq, int64_t step, float lr, float beta1, float beta2, float eps,
                         void* hip_stream)
{
    return adam_step_impl(L, p_shard, g_shard, exp_avg, exp_avg_sq, step, lr, beta1, beta2, eps, nullptr, hip_stream);
}

int fsdp_shard_adam_step_guarded(const fsdp_layout_t* L, float* p_shard, const float* g_shard, float* exp_avg,
                                 float* exp_avg_sq, int64_t step, float lr, float beta1, float beta2, float eps,
                                 const float* found_inf, void* hip_stream)
{
    if (!found_inf) return FSDP_ERR_NULL_PTR;
    return adam_step_impl(L, p_shard, g_shard, exp_avg, exp_avg_sq, step, lr, beta1, beta2, eps, found_inf,
                          hip_stream);
}

int fsdp_reduce_scatter_adam_fused(const fsdp_layout_t* L, const void* const* grad_ptrs, fsdp_dtype_t grad_dtype,
                                   int32_t rank, float pre_div, float post_div, float* grad_shard_out,
                                   float* p_shard, float* exp_avg, float* exp_avg_sq, int64_t step, float lr,
                                   float beta1, float beta2, float eps, void* p_lp_out, void* hip_stream)
{
    int rc = check_reduce_args(L, grad_ptrs, grad_dtype, rank, pre_div, post_div);
    if (rc != FSDP_OK) return rc;
    if (!p_shard || !exp_avg || !exp_avg_sq) return FSDP_ERR_NULL_PTR;
    rc = check_adam_args(step, lr, beta1, beta2, eps);
    if (rc != FSDP_OK) return rc;
    if (L->world_size > kMaxRanks && !grad_shard_out) return FSDP_ERR_NULL_PTR;
    if (misaligned(p_shard, 4) || misaligned(exp_avg, 4) || misaligned(exp_avg_sq, 4) ||
        (grad_shard_out && misaligned(grad_shard_out, 4)) || (p_lp_out && misaligned(p_lp_out, 2)))
        return FSDP_ERR_INVALID_ARG;
    const AdamConsts c = make_adam_consts(step, lr, beta1, beta2, eps);
    return reduce_driver(L, grad_ptrs, grad_dtype, rank, pre_div, post_div, grad_shard_out, true, p_shard, exp_avg,
                         exp_avg_sq, static_cast<uint16_t*>(p_lp_out), c, static_cast<hipStream_t>(hip_stream));
}

int fsdp_reduce_scatter_adam_prefetch_unshard(const fsdp_layout_t* L, const void* const* grad_ptrs,
                                              fsdp_dtype_t grad_dtype, int32_t rank, float pre_div, float post_div,
                                              float* grad_shard_out, float* p_shard, float* exp_avg,
                                              float* exp_avg_sq, int64_t step, float lr, float beta1, float beta2,
                                              float eps, void* p_lp_out, const fsdp_layout_t* next_layout,
                                              const float* const* next_shard_ptrs, void* next_flat_out,
                                              fsdp_dtype_t next_out_dtype, void* hip_stream)
{
    // validate both halves before anything is launched
    int rc = check_reduce_args(L, grad_ptrs, grad_dtype, rank, pre_div, post_div);
    if (rc != FSDP_OK) return rc;
    if (!p_shard || !exp_avg || !exp_avg_sq) return FSDP_ERR_NULL_PTR;
    rc = check_adam_args(step, lr, beta1, beta2, eps);
    if (rc != FSDP_OK) return rc;
    if (L->world_size > kMaxRanks && !grad_shard_out) return FSDP_ERR_NULL_PTR;
    if (misaligned(p_shard, 4) || misaligned(exp_avg, 4) || misaligned(exp_avg_sq, 4) ||
        (grad_shard_out && misaligned(grad_shard_out, 4)) || (p_lp_out && misaligned(p_lp_out, 2)))
        return FSDP_ERR_INVALID_ARG;
    const fsdp_layout_t* N = next_layout;
    if (!N || !next_shard_ptrs || !next_flat_out) return FSDP_ERR_NULL_PTR;
    if (!valid_dtype(next_out_dtype)) return FSDP_ERR_BAD_DTYPE;
    for (int32_t w = 0; w < N->world_size; ++w) {
        if (!next_shard_ptrs[w]) return FSDP_ERR_NULL_PTR;
        if (misaligned(next_shard_ptrs[w], 4)) return FSDP_ERR_INVALID_ARG;
    }
    if (misaligned(next_flat_out, static_cast<uintptr_t>(dtype_size(next_out_dtype)))) return FSDP_ERR_INVALID_ARG;

    const int64_t E = grad_dtype == FSDP_F32 ? 4 : 8;
    const int64_t n_reduce = ceil_div(L->S / E + 1, kBlock);
    const int64_t tiles = ceil_div(N->S / 8 + 1, kBlock);
    const int64_t n_unshard = tiles * N->world_size;
    // Sharing a grid pays while the fixed cost of a launch (about 2 us of ramp
    // and drain) is visible next to the smaller half; for large halves the
    // shared kernel's register budget costs the unshard more than it saves.
    const int64_t reduce_bytes = dtype_size(grad_dtype) * L->P + 24 * L->S;
    const int64_t unshard_bytes = 6 * N->P;
    const bool small_half = (reduce_bytes < unshard_bytes ? reduce_bytes : unshard_bytes) <= kOneLaunchMaxBytes;
    const bool one_launch = small_half && L->world_size <= kMaxRanks && N->world_size <= kMaxRanks &&
                            next_out_dtype == FSDP_BF16 && grid_ok(n_reduce + n_unshard);
    if (!one_launch) {   // same results from the two separate entry points, one after the other
        rc = fsdp_reduce_scatter_adam_fused(L, grad_ptrs, grad_dtype, rank, pre_div, post_div, grad_shard_out, p_shard,
                                            exp_avg, exp_avg_sq, step, lr, beta1, beta2, eps, p_lp_out, hip_stream);
        if (rc != FSDP_OK) return rc;
        return fsdp_unshard(N, next_shard_ptrs, next_flat_out, next_out_dtype, hip_stream);
    }

    const int64_t esz = dtype_size(grad_dtype);
    PtrTable gtab = {}, stab = {};
    for (int32_t w = 0; w < L->world_size; ++w)
        gtab.p[w] = static_cast<const char*>(grad_ptrs[w]) + static_cast<int64_t>(rank) * L->S * esz;
    pad_rank_table(gtab, L->world_size);
    for (int32_t w = 0; w < N->world_size; ++w) stab.p[w] = next_shard_ptrs[w];
    RsArgs a = {};
    int pre_mode = kPreDiv;
    float recip;
    a.pre_c = pre_div;
    if (pre_div == 1.0f) pre_mode = kPreNone;
    else if (is_pow2_float(pre_div, &recip)) { pre_mode = kPreMul; a.pre_c = recip; }
    a.post_c = post_div;
    if (is_pow2_float(post_div, &recip)) { a.post_mul = 1; a.post_c = recip; }
    a.W = L->world_size;
    a.cont = 0;
    a.last = 1;
    a.S = L->S;
    a.out = grad_shard_out;
    a.p = p_shard; a.m = exp_avg; a.v = exp_avg_sq; a.p_lp = static_cast<uint16_t*>(p_lp_out);
    a.adam = make_adam_consts(step, lr, beta1, beta2, eps);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const dim3 grid(static_cast<uint32_t>(n_reduce + n_unshard));
    const uint32_t nr = static_cast<uint32_t>(n_reduce);
    uint16_t* out_base = static_cast<uint16_t*>(next_flat_out);
    const int32_t tl = static_cast<int32_t>(tiles);
#define FSDP_LAUNCH_COMBINED(BF, PRE) \
    hipLaunchKernelGGL((reduce_adam_unshard_kernel<BF, PRE>), grid, dim3(kBlock), 0, st, gtab, a, nr, stab, N->S, \
                       out_base, tl)
    if (grad_dtype == FSDP_BF16) {
        if (pre_mode == kPreNone) FSDP_LAUNCH_COMBINED(kBF16, kPreNone);
        else if (pre_mode == kPreMul) FSDP_LAUNCH_COMBINED(kBF16, kPreMul);
        else FSDP_LAUNCH_COMBINED(kBF16, kPreDiv);
    } else if (grad_dtype == FSDP_F16) {
        if (pre_mode == kPreNone) FSDP_LAUNCH_COMBINED(kF16, kPreNone);
        else if (pre_mode == kPreMul) FSDP_LAUNCH_COMBINED(kF16, kPreMul);
        else FSDP_LAUNCH_COMBINED(kF16, kPreDiv);
    } else {
        if (pre_mode == kPreNone) FSDP_LAUNCH_COMBINED(kF32, kPreNone);
        else if (pre_mode == kPreMul) FSDP_LAUNCH_COMBINED(kF32, kPreMul);
        else FSDP_LAUNCH_COMBINED(kF32, kPreDiv);
    }
#undef FSDP_LAUNCH_COMBINED
    return launch_status();
}

int fsdp_reduce_scatter_hybrid(const fsdp_layout_t* L, const void* const* grad_ptrs, fsdp_dtype_t grad_dtype,
                               int32_t num_groups, int32_t rank, float pre_div, float post_div,
                               float* grad_shard_out, void* hip_stream)
{
    int rc = check_reduce_args(L, grad_ptrs, grad_dtype, rank, pre_div, post_div, num_groups);
    if (rc != FSDP_OK) return rc;
    if (!grad_shard_out) return FSDP_ERR_NULL_PTR;
    if (misaligned(grad_shard_out, 4)) return FSDP_ERR_INVALID_ARG;
    const AdamConsts none = {};
    ReduceOpts opt;
    opt.num_groups = num_groups;
    return reduce_driver(L, grad_ptrs, grad_dtype, rank, pre_div, post_div, grad_shard_out, false, nullptr, nullptr,
                         nullptr, nullptr, none, static_cast<hipStream_t>(hip_stream), opt);
}

int fsdp_reduce_scatter_accumulate(const fsdp_layout_t* L, const void* const* grad_ptrs, fsdp_dtype_t grad_dtype,
                                   int32_t rank, float pre_div, float post_div, float* grad_shard_acc,
                                   void* hip_stream)
{
    int rc = check_reduce_args(L, grad_ptrs, grad_dtype, rank, pre_div, post_div);
    if (rc != FSDP_OK) return rc;
    if (!grad_shard_acc) return FSDP_ERR_NULL_PTR;
    if (misaligned(grad_shard_acc, 4)) return FSDP_ERR_INVALID_ARG;
    const AdamConsts none = {};
    ReduceOpts opt;
    opt.accumulate = true;
    return reduce_driver(L, grad_ptrs, grad_dtype, rank, pre_div, post_div, grad_shard_acc, false, nullptr, nullptr,
                         nullptr, nullptr, none, static_cast<hipStream_t>(hip_stream), opt);
}

int fsdp_grad_accumulate(const fsdp_layout_t* L, float* grad_acc, const void* grad_add, fsdp_dtype_t add_dtype,
                         void* hip_stream)
{
    if (!L || !grad_acc || !grad_add) return FSDP_ERR_NULL_PTR;
    if (!valid_dtype(add_dtype)) return FSDP_ERR_BAD_DTYPE;
    if (misaligned(grad_acc, 4) || misaligned(grad_add, static_cast<uintptr_t>(dtype_size(add_dtype))))
        return FSDP_ERR_INVALID_ARG;
    const int64_t blocks = ceil_div(L->P / 4 + 1, kBlock);
    if (!grid_ok(blocks)) return FSDP_ERR_OVERFLOW;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const dim3 grid(static_cast<uint32_t>(blocks));
    if (add_dtype == FSDP_BF16)
        hipLaunchKernelGGL(accumulate_kernel<kBF16>, grid, dim3(kBlock), 0, st, grad_acc, grad_add, L->P);
    else if (add_dtype == FSDP_F16)
        hipLaunchKernelGGL(accumulate_kernel<kF16>, grid, dim3(kBlock), 0, st, grad_acc, grad_add, L->P);
    else
        hipLaunchKernelGGL(accumulate_kernel<kF32>, grid, dim3(kBlock), 0, st, grad_acc, grad_add, L->P);
    return launch_status();
}

int fsdp_cast_shard(const fsdp_layout_t* L, const float* shard, void* lp_shard_out, fsdp_dtype_t lp_dtype,
                    void* hip_stream)
{
    if (!L || !shard || !lp_shard_out) return FSDP_ERR_NULL_PTR;
    if (lp_dtype != FSDP_BF16 && lp_dtype != FSDP_F16) return FSDP_ERR_BAD_DTYPE;
    if (misaligned(shard, 4) || misaligned(lp_shard_out, 2)) return FSDP_ERR_INVALID_ARG;
    const int64_t tiles = ceil_div(L->S / 8 + 1, kBlock);
    if (!grid_ok(tiles)) return FSDP_ERR_OVERFLOW;
    PtrTable tab = {};
    tab.p[0] = shard;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (lp_dtype == FSDP_F16)
        hipLaunchKernelGGL(unshard_lp_kernel<kF16>, dim3(static_cast<uint32_t>(tiles)), dim3(kBlock), 0, st, tab, L->S,
                           static_cast<uint16_t*>(lp_shard_out), static_cast<int32_t>(tiles));
    else
        hipLaunchKernelGGL(unshard_lp_kernel<kBF16>, dim3(static_cast<uint32_t>(tiles)), dim3(kBlock), 0, st, tab,
                           L->S, static_cast<uint16_t*>(lp_shard_out), static_cast<int32_t>(tiles));
    return launch_status();
}

int fsdp_unshard_lp(const fsdp_layout_t* L, const void* const* lp_shard_ptrs, void* flat_out, void* hip_stream)
{
    if (!L || !lp_shard_ptrs || !flat_out) return FSDP_ERR_NULL_PTR;
    const int32_t W = L->world_size;
    const int64_t S = L->S;
    for (int32_t w = 0; w < W; ++w) {
        if (!lp_shard_ptrs[w]) return FSDP_ERR_NULL_PTR;
        if (misaligned(lp_shard_ptrs[w], 2)) return FSDP_ERR_INVALID_ARG;
    }
    if (misaligned(flat_out, 2)) return FSDP_ERR_INVALID_ARG;
    const int64_t tiles = ceil_div(S / 8 + 1, kBlock);
    if (!grid_ok(tiles * kMaxRanks)) return FSDP_ERR_OVERFLOW;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    for (int32_t w0 = 0; w0 < W; w0 += kMaxRanks) {
        const int32_t nw = W - w0 < kMaxRanks ? W - w0 : kMaxRanks;
        PtrTable tab = {};
        for (int32_t j = 0; j < nw; ++j) tab.p[j] = lp_shard_ptrs[w0 + j];
        uint16_t* base = static_cast<uint16_t*>(flat_out) + static_cast<int64_t>(w0) * S;
        hipLaunchKernelGGL(gather_lp_kernel, dim3(static_cast<uint32_t>(tiles * nw)), dim3(kBlock), 0, st, tab, S,
                           base, static_cast<int32_t>(tiles));
        const int rc = launch_status();
        if (rc != FSDP_OK) return rc;
    }
    return FSDP_OK;
}

int fsdp_reduce_scatter_unscale(const fsdp_layout_t* L, const void* const* grad_ptrs, fsdp_dtype_t grad_dtype,
                                int32_t rank, float pre_div, float post_div, float inv_scale, float* grad_shard_out,
                                float* found_inf, void* hip_stream)
{
    int rc = check_reduce_args(L, grad_ptrs, grad_dtype, rank, pre_div, post_div);
    if (rc != FSDP_OK) return rc;
    if (!grad_shard_out || !found_inf) return FSDP_ERR_NULL_PTR;
    if (misaligned(grad_shard_out, 4) || misaligned(found_inf, 4)) return FSDP_ERR_INVALID_ARG;
    if (!std::isfinite(inv_scale) || !(inv_scale > 0.0f)) return FSDP_ERR_INVALID_ARG;
    const AdamConsts none = {};
    ReduceOpts opt;
    opt.unscale = true;
    opt.inv_scale = inv_scale;
    opt.found_inf = found_inf;
    return reduce_driver(L, grad_ptrs, grad_dtype, rank, pre_div, post_div, grad_shard_out, false, nullptr, nullptr,
                         nullptr, nullptr, none, static_cast<hipStream_t>(hip_stream), opt);
}

int fsdp_found_inf_combine(float* const* found_inf_ptrs, int32_t num_ranks, void* hip_stream)
{
    if (!found_inf_ptrs) return FSDP_ERR_NULL_PTR;
    if (num_ranks <= 0 || num_ranks > kMaxRanks) return FSDP_ERR_INVALID_ARG;
    FlagTable tab = {};
    for (int32_t i = 0; i < num_ranks; ++i) {
        if (!found_inf_ptrs[i]) return FSDP_ERR_NULL_PTR;
        if (misaligned(found_inf_ptrs[i], 4)) return FSDP_ERR_INVALID_ARG;
        tab.p[i] = found_inf_ptrs[i];
    }
    hipLaunchKernelGGL(found_inf_combine_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(hip_stream), tab,
                       num_ranks);
    return launch_status();
}

int fsdp_grad_scaler_update(float* scale, int32_t* growth_tracker, const float* found_inf, float growth_factor,
                            float backoff_factor, int32_t growth_interval, void* hip_stream)
{
    if (!scale || !growth_tracker || !found_inf) return FSDP_ERR_NULL_PTR;
    if (misaligned(scale, 4) || misaligned(growth_tracker, 4) || misaligned(found_inf, 4)) return FSDP_ERR_INVALID_ARG;
    if (!(growth_factor > 1.0f) || !std::isfinite(growth_factor) || !(backoff_factor > 0.0f) ||
        !(backoff_factor < 1.0f) || growth_interval < 1)
        return FSDP_ERR_INVALID_ARG;
    hipLaunchKernelGGL(scaler_update_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(hip_stream), scale,
                       growth_tracker, found_inf, growth_factor, backoff_factor, growth_interval);
    return launch_status();
}

}  // extern "C"

// ---- batches ----------------------------------------------------------------

struct fsdp_batch {
    struct ReduceRec {
        const fsdp_layout_t* L;
        std::vector<const void*> grads;      // already advanced to the rank's slice
        fsdp_dtype_t dtype;
        int32_t rank;
        float pre, post;
        float *out, *p, *m, *v;
        uint16_t* p_lp;
        float lr, beta1, beta2, eps;
        std::vector<const void*> raw;        // the caller's table, for the single-operation fallback
    };
    struct UnshardRec {
        const fsdp_layout_t* L;
        std::vector<const float*> shards;
        void* out;
        fsdp_dtype_t dtype;
    };
    struct Op {
        bool is_reduce;
        size_t index;
    };
    std::vector<ReduceRec> reduces;
    std::vector<UnshardRec> unshards;
    std::vector<Op> order;
};

namespace {

struct ReduceKind {
    int gt, pre_mode;
    bool operator==(const ReduceKind& o) const { return gt == o.gt && pre_mode == o.pre_mode; }
};

int pre_mode_of(float pre) {
    float r;
    if (pre == 1.0f) return kPreNone;
    return is_pow2_float(pre, &r) ? kPreMul : kPreDiv;
}

template <int GT>
void launch_batch_pre(const ReduceKind& k, const BatchArgs& b, uint32_t blocks, hipStream_t st)
{
    if (k.pre_mode == kPreNone)
        hipLaunchKernelGGL((batch_kernel<GT, kPreNone>), dim3(blocks), dim3(kBlock), 0, st, b);
    else if (k.pre_mode == kPreMul)
        hipLaunchKernelGGL((batch_kernel<GT, kPreMul>), dim3(blocks), dim3(kBlock), 0, st, b);
    else
        hipLaunchKernelGGL((batch_kernel<GT, kPreDiv>), dim3(blocks), dim3(kBlock), 0, st, b);
}
void launch_batch_grid(const ReduceKind& k, const BatchArgs& b, uint32_t blocks, hipStream_t st)
{
    if (k.gt == kBF16) launch_batch_pre<kBF16>(k, b, blocks, st);
    else if (k.gt == kF16) launch_batch_pre<kF16>(k, b, blocks, st);
    else launch_batch_pre<kF32>(k, b, blocks, st);
}

}  // namespace

extern "C" {

int fsdp_batch_create(fsdp_batch_t** out)
{
    if (!out) return FSDP_ERR_NULL_PTR;
    *out = new (std::nothrow) fsdp_batch;
    return *out ? FSDP_OK : FSDP_ERR_OOM;
}

void fsdp_batch_destroy(fsdp_batch_t* b) { delete b; }

int fsdp_batch_clear(fsdp_batch_t* b)
{
    if (!b) return FSDP_ERR_NULL_PTR;
    b->reduces.clear();
    b->unshards.clear();
    b->order.clear();
    return FSDP_OK;
}

int fsdp_batch_add_unshard(fsdp_batch_t* b, const fsdp_layout_t* L, const float* const* shard_ptrs, void* flat_out,
                           fsdp_dtype_t out_dtype)
{
    if (!b || !L || !shard_ptrs || !flat_out) return FSDP_ERR_NULL_PTR;
    if (!valid_dtype(out_dtype)) return FSDP_ERR_BAD_DTYPE;
    for (int32_t w = 0; w < L->world_size; ++w) {
        if (!shard_ptrs[w]) return FSDP_ERR_NULL_PTR;
        if (misaligned(shard_ptrs[w], 4)) return FSDP_ERR_INVALID_ARG;
    }
    if (misaligned(flat_out, static_cast<uintptr_t>(dtype_size(out_dtype)))) return FSDP_ERR_INVALID_ARG;
    try {
        fsdp_batch::UnshardRec r;
        r.L = L;
        r.shards.assign(shard_ptrs, shard_ptrs + L->world_size);
        r.out = flat_out;
        r.dtype = out_dtype;
        b->unshards.push_back(std::move(r));
        b->order.push_back({false, b->unshards.size() - 1});
    } catch (const std::bad_alloc&) {
        return FSDP_ERR_OOM;
    }
    return FSDP_OK;
}

int fsdp_batch_add_reduce_scatter_adam(fsdp_batch_t* b, const fsdp_layout_t* L, const void* const* grad_ptrs,
                                       fsdp_dtype_t grad_dtype, int32_t rank, float pre_div, float post_div,
                                       float* grad_shard_out, float* p_shard, float* exp_avg, float* exp_avg_sq,
                                       float lr, float beta1, float beta2, float eps, void* p_lp_out)
{
    if (!b) return FSDP_ERR_NULL_PTR;
    int rc = check_reduce_args(L, grad_ptrs, grad_dtype, rank, pre_div, post_div);
    if (rc != FSDP_OK) return rc;
    if (!p_shard || !exp_avg || !exp_avg_sq) return FSDP_ERR_NULL_PTR;
    rc = check_adam_args(1, lr, beta1, beta2, eps);
    if (rc != FSDP_OK) return rc;
    if (L->world_size > kMaxRanks && !grad_shard_out) return FSDP_ERR_NULL_PTR;
    if (misaligned(p_shard, 4) || misaligned(exp_avg, 4) || misaligned(exp_avg_sq, 4) ||
        (grad_shard_out && misaligned(grad_shard_out, 4)) || (p_lp_out && misaligned(p_lp_out, 2)))
        return FSDP_ERR_INVALID_ARG;
    try {
        fsdp_batch::ReduceRec r;
        r.L = L;
        r.raw.assign(grad_ptrs, grad_ptrs + L->world_size);
        const int64_t off = static_cast<int64_t>(rank) * L->S * dtype_size(grad_dtype);
        for (int32_t w = 0; w < L->world_size; ++w) r.grads.push_back(static_cast<const char*>(grad_ptrs[w]) + off);
        r.dtype = grad_dtype;
        r.rank = rank;
        r.pre = pre_div;
        r.post = post_div;
        r.out = grad_shard_out;
        r.p = p_shard; r.m = exp_avg; r.v = exp_avg_sq;
        r.p_lp = static_cast<uint16_t*>(p_lp_out);
        r.lr = lr; r.beta1 = beta1; r.beta2 = beta2; r.eps = eps;
        b->reduces.push_back(std::move(r));
        b->order.push_back({true, b->reduces.size() - 1});
    } catch (const std::bad_alloc&) {
        return FSDP_ERR_OOM;
    }
    return FSDP_OK;
}

int fsdp_batch_launch(const fsdp_batch_t* b, int64_t step, void* hip_stream)
{
    if (!b) return FSDP_ERR_NULL_PTR;
    if (step < 1) return FSDP_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);

    // Greedy grouping in insertion order.  A grid takes up to kBatchOps reduce
    // operations of one kernel kind and up to kBatchOps bf16 unshards, each with
    // at most kBatchRanks ranks, and at most one operation above
    // kOneLaunchMaxBytes (see the prefetch entry point).  Anything else is
    // issued through its own entry point.
    BatchArgs g = {};
    ReduceKind kind = {kF32, kPreNone};
    bool have_kind = false;
    int large = 0;
    uint32_t r_blocks = 0, u_blocks = 0;

    auto flush = [&]() -> int {
        if (g.n_reduce == 0 && g.n_unshard == 0) return FSDP_OK;
        int rc = FSDP_OK;
        // a grid without reduce operations never enters the reduce code, so any instantiation serves
        if (g.n_reduce == 0) kind = ReduceKind{kF32, kPreNone};
        if (g.n_reduce == 1 && g.n_unshard == 0 && large > 0) {
            // the lone update of a unit too large to share a grid goes through the stand-alone kernel,
            // which may choose the deep rank walk
            PtrTable tab = {};
            for (int32_t w = 0; w < kBatchRanks; ++w) tab.p[w] = g.r[0].grads[w];
            if (kind.gt == kBF16) launch_reduce_pre<kBF16, true>(kind.pre_mode, tab, g.r[0].a, st);
            else if (kind.gt == kF16) launch_reduce_pre<kF16, true>(kind.pre_mode, tab, g.r[0].a, st);
            else launch_reduce_pre<kF32, true>(kind.pre_mode, tab, g.r[0].a, st);
        } else {
            launch_batch_grid(kind, g, r_blocks + u_blocks, st);
        }
        rc = launch_status();
        g = BatchArgs{};
        have_kind = false;
        large = 0;
        r_blocks = u_blocks = 0;
        return rc;
    };

    for (const fsdp_batch::Op& op : b->order) {
        if (op.is_reduce) {
            const fsdp_batch::ReduceRec& r = b->reduces[op.index];
            const int32_t W = r.L->world_size;
            const int64_t bytes = dtype_size(r.dtype) * r.L->P + 24 * r.L->S;
            const int64_t E = r.dtype == FSDP_F32 ? 4 : 8;
            const int64_t nb = ceil_div(r.L->S / E + 1, kBlock);
            const bool batchable = W <= kBatchRanks && grid_ok(nb + r_blocks + u_blocks);
            if (!batchable) {
                int rc = flush();
                if (rc != FSDP_OK) return rc;
                rc = fsdp_reduce_scatter_adam_fused(r.L, r.raw.data(), r.dtype, r.rank, r.pre, r.post, r.out, r.p, r.m, r.v,
                                                    step, r.lr, r.beta1, r.beta2, r.eps, r.p_lp, hip_stream);
                if (rc != FSDP_OK) return rc;
                continue;
            }
            const ReduceKind k = {static_cast<int>(r.dtype), pre_mode_of(r.pre)};
            const bool is_large = bytes > kOneLaunchMaxBytes;
            if (g.n_reduce == kBatchOps || (have_kind && !(k == kind)) || (is_large && large > 0)) {
                const int rc = flush();
                if (rc != FSDP_OK) return rc;
            }
            kind = k;
            have_kind = true;
            large += is_large ? 1 : 0;
            BatchReduceOp& o = g.r[g.n_reduce];
            for (int32_t w = 0; w < kBatchRanks; ++w) o.grads[w] = r.grads[w < W ? w : W - 1];   // padded for whole groups
            RsArgs& a = o.a;
            a = RsArgs{};
            float recip;
            a.pre_c = r.pre;
            if (k.pre_mode == kPreMul) { is_pow2_float(r.pre, &recip); a.pre_c = recip; }
            a.post_c = r.post;
            if (is_pow2_float(r.post, &recip)) { a.post_mul = 1; a.post_c = recip; }
            a.W = W;
            a.last = 1;
            a.S = r.L->S;
            a.out = r.out;
            a.p = r.p; a.m = r.m; a.v = r.v; a.p_lp = r.p_lp;
            a.adam = make_adam_consts(step, r.lr, r.beta1, r.beta2, r.eps);
            r_blocks += static_cast<uint32_t>(nb);
            g.r_end[g.n_reduce] = r_blocks;
            ++g.n_reduce;
        } else {
            const fsdp_batch::UnshardRec& u = b->unshards[op.index];
            const int32_t W = u.L->world_size;
            const int64_t bytes = 6 * u.L->P;
            const int64_t tiles = ceil_div(u.L->S / 8 + 1, kBlock);
            const bool batchable = W <= kBatchRanks && u.dtype == FSDP_BF16 && grid_ok(tiles * W + r_blocks + u_blocks);
            if (!batchable) {
                int rc = flush();
                if (rc != FSDP_OK) return rc;
                rc = fsdp_unshard(u.L, u.shards.data(), u.out, u.dtype, hip_stream);
                if (rc != FSDP_OK) return rc;
                continue;
            }
            const bool is_large = bytes > kOneLaunchMaxBytes;
            if (g.n_unshard == kBatchOps || (is_large && large > 0)) {
                const int rc = flush();
                if (rc != FSDP_OK) return rc;
            }
            large += is_large ? 1 : 0;
            BatchUnshardOp& o = g.u[g.n_unshard];
            for (int32_t w = 0; w < kBatchRanks; ++w) o.shards[w] = u.shards[w < W ? w : W - 1];
            o.S = u.L->S;
            o.out = static_cast<uint16_t*>(u.out);
            o.tiles = static_cast<int32_t>(tiles);
            u_blocks += static_cast<uint32_t>(tiles * W);
            g.u_end[g.n_unshard] = u_blocks;
            ++g.n_unshard;
        }
    }
    return flush();
}

}  // extern "C"
