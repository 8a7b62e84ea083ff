// Unshard kernels: the gather of W shards into the unsharded FlatParameter
// (Sec. 3.2.1), fused with the full-to-low precision cast (Sec. 4.4).
#pragma once

#include "device_common.h"

namespace {

// ---------------------------------------------------------------------------
// unshard: flat_out[w*S + k] = cast(shard_w[k])   (Sec. 3.2.1 gather, Sec. 4.4 cast)
// grid = nshards * tiles_per_shard blocks; block b serves shard b / tiles and
// tile b % tiles.  A tile is kBlock destination vectors of 16 bytes.
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

// The same cast + gather in single-wave workgroups, one destination vector of 8
// bytes (four 16-bit values) per lane: a 16-byte load of four floats (any
// 4-byte alignment) and an 8-byte store, both contiguous across the wave, no
// LDS.  Measured on MI355X over 1 GiB of output: 7.0 TB/s against 6.5 TB/s for
// the form above; the same lane work in workgroups of 128 or 256 lanes stays at
// 6.5-6.6 TB/s, so this form only exists as a stand-alone kernel.  The host
// takes it when every shard's loads are 16-byte aligned: with loads that are
// only 4-byte aligned this form drops to 6.4 TB/s, and realigning through LDS
// inside a single-wave workgroup to 4.7 TB/s (the round trip through LDS
// lengthens the life of waves that have nothing else in flight), both below
// the form above, which realigns through LDS at no cost.
constexpr int kLightBlock = 64;
// grid = (tiles per shard, shards): the shard's pointer is fetched together with the other arguments, a wave's
// whole life being two memory round trips
template <int LP>
__global__ __launch_bounds__(kLightBlock) void unshard_lp_light_kernel(PtrTable shards, int64_t S,
                                                                        uint16_t* __restrict__ out_base)
{
    const int32_t w = blockIdx.y;
    const int32_t tile = blockIdx.x;
    const float* __restrict__ src = static_cast<const float*>(shards.p[w]);
    uint16_t* __restrict__ dst = out_base + static_cast<int64_t>(w) * S;
    const int lane = threadIdx.x;

    // Elements up to the destination's next 128-byte boundary (0..63): every wave then stores four whole
    // cache lines.  (Aligned to 8 bytes only, a shard slot that starts off a line boundary, as with an odd
    // shard size, makes every wave's store end in two partial lines: 15 % slower.)
    const int64_t h128 = ((128u - (static_cast<uint32_t>(reinterpret_cast<uintptr_t>(dst)) & 127u)) & 127u) >> 1;
    const int64_t head = h128 < S ? h128 : S;
    const int64_t nvec = (S - head) >> 2;
    const int64_t c = static_cast<int64_t>(tile) * kLightBlock + lane;
    if (c < nvec) {
        const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_a4*>(src + head + (c << 2)));
        const u32x2 o = {pack_lp2<LP>(v.x, v.y), pack_lp2<LP>(v.z, v.w)};
        __builtin_nontemporal_store(o, reinterpret_cast<u32x2*>(dst + head + (c << 2)));
    }
    if (tile == 0) {   // ragged head (at most 63 elements) and tail (at most 3) of this shard
        const int64_t tail0 = head + (nvec << 2);
        const int64_t ntail = S - tail0;
        if (lane < head) dst[lane] = static_cast<uint16_t>(cast_lp<LP>(src[lane]));
        if (lane < ntail) dst[tail0 + lane] = static_cast<uint16_t>(cast_lp<LP>(src[tail0 + lane]));
    }
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

// Gather of 16-bit shards (the AllGather in the low precision, Sec. 4.4):
// flat_lp[w*S + k] = lp_shard_w[k]; 16-byte destination vectors, sources only
// 2-byte aligned.  bid = index of the workgroup among the launch's gather
// workgroups, as in unshard_lp_body.
template <int B = kBlock>
__device__ __forceinline__ void gather_lp_body(const void* const* shards, int64_t S, uint16_t* __restrict__ out_base,
                                               int32_t tiles_per_shard, uint32_t bid)
{
    const int32_t w = bid / tiles_per_shard;
    const int32_t tile = bid - w * tiles_per_shard;
    const uint16_t* __restrict__ src = static_cast<const uint16_t*>(shards[w]);
    uint16_t* __restrict__ dst = out_base + static_cast<int64_t>(w) * S;

    const int64_t head = head_elems(dst, 2, S);
    const int64_t nvec = (S - head) >> 3;
    const int64_t c = static_cast<int64_t>(tile) * B + threadIdx.x;
    if (c < nvec) {
        const u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const u32x4_a2*>(src + head + (c << 3)));
        __builtin_nontemporal_store(a, reinterpret_cast<u32x4*>(dst + head + (c << 3)));
    }
    if (tile == 0) {
        const int64_t tail0 = head + (nvec << 3);
        const int64_t ntail = S - tail0;
        const int t = threadIdx.x;
        if (t < head) dst[t] = src[t];
        if (t >= 32 && t - 32 < ntail) dst[tail0 + t - 32] = src[tail0 + t - 32];
    }
}

// stand-alone: single-wave workgroups (a plain 16-byte copy measures 2 % faster in them than in 256-lane ones)
__global__ __launch_bounds__(kLightBlock) void gather_lp_kernel(PtrTable shards, int64_t S,
                                                                 uint16_t* __restrict__ out_base,
                                                                 int32_t tiles_per_shard)
{
    gather_lp_body<kLightBlock>(shards.p, S, out_base, tiles_per_shard, blockIdx.x);
}

}  // namespace
