// Reduce-scatter rank share (Sec. 3, eq. (1); hybrid sharding Sec. 3.2.2;
// gradient accumulation Sec. 3.3.4; gradient scaler Sec. 4.4) with the optional
// fused Adam epilogue (Sec. 5.4), and the one-launch backward prefetch
// (Sec. 3.3.2) built from it and the unshard body.
#pragma once

#include "device_common.h"
#include "unshard_kernels.h"

namespace {

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
    int32_t cont;         // 1: the sum continues from out[] (a later launch of a split W; with hybrid groups the
                          // launches split between groups and out[] carries the sum over the groups so far)
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
//   wide  (C = 1): one chunk per lane, the most workgroups.  G, the ranks per
//         batch, is what measured fastest on MI355X with cold buffers: 4 for the
//         fused kernels on 16-bit gradients (with the Adam state fetched before
//         the walk), 1 for the fused kernels on fp32 gradients (state fetched
//         after the walk; 3-9 % faster than G = 4 from 7 M-element units up),
//         2 resp. 1 for the reduce-scatter alone (13 % faster than G = 4 at 64
//         ranks: the more rank streams, the shallower the best queue per lane).
//   deep  (G = 1, C = 4): one rank stream at a time, four chunks of it, so a
//         workgroup reads 16 KiB of a rank in one piece.  Taken from about 1.4
//         such workgroups per compute unit on when there are many ranks (the
//         host's rule and its measurements: deep_walk_pays).
//   half  (C = 1, G = 1, E = 4 also for 16-bit gradients, which are then loaded 8
//         bytes at a time; no load ahead): the lightest wave.  Its reads and
//         writes of p, m, v are 16 bytes per lane, contiguous across the wave,
//         where a lane that owns eight 16-bit gradients touches 32 bytes of each
//         state array, so that each of its instructions covers only every other
//         16 bytes of its span.  In single-wave workgroups, and with only one
//         load in flight per lane, the occupancy (8 waves per SIMD at 48
//         registers) is what keeps the memory busy: measured, this mix of reads
//         and read-modify-writes moves faster when each wave asks for little at a
//         time (deep_walk_pays / half_walk_pays on the host carry the figures).
// The host pads the pointer table to a multiple of kMaxWideRanks with copies of
// the last pointer, so loads never need a predicate; the padding's adds are
// skipped.
constexpr int kMaxWideRanks = 4;
template <int GT, bool FUSED, bool DEEP, bool HALF = false>
struct WalkShape {
    static constexpr int E = (GT != kF32 && !HALF) ? 8 : 4;
    static constexpr int G = (DEEP || HALF) ? 1 : (GT == kF32 ? 1 : (FUSED ? kMaxWideRanks : 2));
    static constexpr int C = DEEP ? 4 : 1;
    // fetch p, m, v (and the accumulated gradient) before the rank walk rather than after it
    static constexpr bool kStateFirst = !DEEP && !HALF && GT != kF32;
    // issue the next batch's loads before the current batch's adds wait for their data
    static constexpr bool kLookahead = !HALF;
};

// what one rank's load of a chunk returns: 16 bytes, or 8 bytes for a half chunk of 16-bit gradients
template <int GT, int E>
struct GradVec {
    using type = u32x4;
};
template <>
struct GradVec<kBF16, 4> {
    using type = u32x2;
};
template <>
struct GradVec<kF16, 4> {
    using type = u32x2;
};

template <int GT, int G, int C, int E>
__device__ __forceinline__ void load_batch(const void* const* grads, int32_t w0, const int64_t (&k)[C],
                                           typename GradVec<GT, E>::type (&x)[G][C])
{
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int j = 0; j < C; ++j) {
            if constexpr (GT != kF32 && E == 4)
                x[g][j] = __builtin_nontemporal_load(
                    reinterpret_cast<const u32x2_a2*>(static_cast<const uint16_t*>(grads[w0 + g]) + k[j]));
            else if constexpr (GT != kF32)
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
template <int GT, int PRE, int G, int C, int E, bool HYBRID>
__device__ __forceinline__ void add_batch(const typename GradVec<GT, E>::type (&x)[G][C], int32_t n, float pre_c,
                                          int32_t group, int32_t& cnt, float (&acc)[C][E], float (&outer)[C][E])
{
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (g < n) {   // uniform
#pragma unroll
            for (int j = 0; j < C; ++j) {
                float t[E];
                if constexpr (GT != kF32 && E == 4) {   // exact upcast of four 16-bit gradients
                    t[0] = up_lo<GT>(x[g][j].x); t[1] = up_hi<GT>(x[g][j].x);
                    t[2] = up_lo<GT>(x[g][j].y); t[3] = up_hi<GT>(x[g][j].y);
                } else if constexpr (GT != kF32) {   // exact upcast of eight 16-bit gradients
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
            if (HYBRID && group > 0 && ++cnt == group) {   // uniform
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
//
// PLAIN instantiations serve the launches that use none of the variants (no
// hybrid groups, no accumulation, no unscaling, no carried partial sum): the
// second set of accumulators and the old gradient then take no registers.
template <int GT, int PRE, bool FUSED, bool DEEP, int B, bool PLAIN, bool HALF = false>
__device__ __forceinline__ void reduce_body(const void* const* grads, const RsArgs& a, uint32_t bid)
{
    using Shape = WalkShape<GT, FUSED, DEEP, HALF>;
    constexpr int E = Shape::E, G = Shape::G, C = Shape::C;
    constexpr int Q = E / 4;
    const int32_t group = PLAIN ? 0 : a.group;
    const bool cont = !PLAIN && a.cont, accum = !PLAIN && a.accum, unscale = !PLAIN && a.unscale;
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
#pragma unroll
            for (int e = 0; e < E; ++e) {
                acc[j][e] = -0.0f;
                outer[j][e] = -0.0f;
            }
            if (cont) {   // the carried partial sum: the flat sum, or with hybrid groups the sum over the groups so far
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    const f32x4 t = *reinterpret_cast<const f32x4_a4*>(a.out + k[j] + 4 * q);
                    if (group > 0) {   // uniform
                        outer[j][4 * q] = t.x; outer[j][4 * q + 1] = t.y; outer[j][4 * q + 2] = t.z; outer[j][4 * q + 3] = t.w;
                    } else {
                        acc[j][4 * q] = t.x; acc[j][4 * q + 1] = t.y; acc[j][4 * q + 2] = t.z; acc[j][4 * q + 3] = t.w;
                    }
                }
            }
        }

        // The optimizer state (and the accumulated gradient) of the lane's chunks:
        // fetched ahead of the rank walk (WalkShape::kStateFirst) or after it, and
        // then one chunk ahead of the chunk being updated, so that the state of
        // at most two chunks is held in registers at a time.
        f32x4 pv[C][Q], mv[C][Q], vv[C][Q], old[C][Q];
        auto fetch_state = [&](int j) {
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                if constexpr (FUSED) {
                    pv[j][q] = *reinterpret_cast<const f32x4*>(a.p + k[j] + 4 * q);
                    mv[j][q] = *reinterpret_cast<const f32x4_a4*>(a.m + k[j] + 4 * q);
                    vv[j][q] = *reinterpret_cast<const f32x4_a4*>(a.v + k[j] + 4 * q);
                }
                if (accum) old[j][q] = *reinterpret_cast<const f32x4_a4*>(a.out + k[j] + 4 * q);
            }
        };
        if constexpr (Shape::kStateFirst) {
#pragma unroll
            for (int j = 0; j < C; ++j) fetch_state(j);
        }

        typename GradVec<GT, E>::type xa[G][C], xb[G][C];
        const int32_t nbatch = (W + G - 1) / G;
        if constexpr (!Shape::kLookahead) {   // one batch in flight per lane: the occupancy keeps the memory system busy
            for (int32_t b = 0; b < nbatch; ++b) {
                load_batch<GT, G, C, E>(grads, b * G, k, xa);
                add_batch<GT, PRE, G, C, E, !PLAIN>(xa, W - b * G, a.pre_c, group, cnt, acc, outer);
            }
        } else {
        load_batch<GT, G, C, E>(grads, 0, k, xa);
        for (int32_t b = 0; b < nbatch; b += 2) {
            const bool has_b = b + 1 < nbatch;
            if (has_b) load_batch<GT, G, C, E>(grads, (b + 1) * G, k, xb);
            add_batch<GT, PRE, G, C, E, !PLAIN>(xa, W - b * G, a.pre_c, group, cnt, acc, outer);
            if (b + 2 < nbatch) load_batch<GT, G, C, E>(grads, (b + 2) * G, k, xa);
            if (has_b) add_batch<GT, PRE, G, C, E, !PLAIN>(xb, W - (b + 1) * G, a.pre_c, group, cnt, acc, outer);
        }
        }

        if constexpr (!Shape::kStateFirst) fetch_state(0);
#pragma unroll
        for (int j = 0; j < C; ++j) {
            if constexpr (!Shape::kStateFirst) {
                if (j + 1 < C) fetch_state(j + 1);
            }
            if (!live[j]) continue;
            float (&r)[E] = acc[j];
            if (group > 0) {   // every sharded group has been folded: the outer sum is the result
#pragma unroll
                for (int e = 0; e < E; ++e) r[e] = outer[j][e];
            }
            if (a.last) {
#pragma unroll
                for (int e = 0; e < E; ++e) r[e] = post_scale(r[e], a);
            }
            if (accum) {
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    r[4 * q] = old[j][q].x + r[4 * q];
                    r[4 * q + 1] = old[j][q].y + r[4 * q + 1];
                    r[4 * q + 2] = old[j][q].z + r[4 * q + 2];
                    r[4 * q + 3] = old[j][q].w + r[4 * q + 3];
                }
            }
            if (unscale) {   // sharded gradient scaler (Sec. 4.4): check, then unscale
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
            const float old_r = accum ? a.out[k] : 0.0f;
            float r = cont && group == 0 ? a.out[k] : -0.0f;
            float outer_r = cont && group > 0 ? a.out[k] : -0.0f;
            int32_t cnt = 0;
            for (int32_t w = 0; w < W; ++w) {
                r = r + pre_scale<PRE>(load_grad<GT>(grads[w], k), a.pre_c);
                if (group > 0 && ++cnt == group) {
                    outer_r = outer_r + r;
                    r = -0.0f;
                    cnt = 0;
                }
            }
            if (group > 0) r = outer_r;
            if (a.last) r = post_scale(r, a);
            if (accum) r = old_r + r;
            if (unscale) {
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

template <int GT, int PRE, bool FUSED, bool DEEP, int B, bool PLAIN, bool HALF = false>
__global__ __launch_bounds__(B) void reduce_kernel(PtrTable grads, RsArgs a)
{
    reduce_body<GT, PRE, FUSED, DEEP, B, PLAIN, HALF>(grads.p, a, blockIdx.x);
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
        reduce_body<GT, PRE, true, false, kBlock, true>(grads.p, a, blockIdx.x);
    else
        unshard_lp_body<kBF16>(shards.p, S_next, out_base, tiles_per_shard, blockIdx.x - n_reduce);
}

}  // namespace
