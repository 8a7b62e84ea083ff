// flatten + pad + shard (Sec. 3.2.1): the LDS-staged ragged pack kernel.
#pragma once

#include "device_common.h"

namespace {

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

}  // namespace
