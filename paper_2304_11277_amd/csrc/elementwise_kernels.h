// Stand-alone Adam on the shard (Sec. 5.4), unsharded gradient accumulation
// (Sec. 3.3.4) and the gradient scaler's bookkeeping kernels (Sec. 4.4).
#pragma once

#include "reduce_kernels.h"

namespace {

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

}  // namespace
