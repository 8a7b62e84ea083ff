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
// Layout of the sources: device_common.h (casts, vector types, pointer tables);
// unshard_kernels.h; pack_kernel.h (LDS-staged ragged pack); reduce_kernels.h
// (the reduce-scatter body with its Adam epilogue, the single and the
// one-launch prefetch kernels); batch_kernel.h; elementwise_kernels.h (Adam,
// gradient accumulation, gradient-scaler bookkeeping); this file holds the host
// side: argument checks, launch helpers and the extern "C" entry points.
//
// Build flags that matter for bit-exactness: -ffp-contract=off (no fused
// multiply-add), IEEE-correct fp32 divide and sqrt (hipcc's default), fp32
// denormals kept (gfx950's default).
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <new>
#include <vector>

#include "fsdp_internal.h"

#include "device_common.h"
#include "unshard_kernels.h"
#include "pack_kernel.h"
#include "reduce_kernels.h"
#include "batch_kernel.h"
#include "elementwise_kernels.h"

namespace {

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

// the wide rank walk loads whole batches of up to kMaxWideRanks ranks: repeat the last pointer up to the batch boundary
void pad_rank_table(PtrTable& tab, int32_t n)
{
    static_assert(kMaxRanks % kMaxWideRanks == 0, "the padded table must fit");
    for (int32_t j = n; j % kMaxWideRanks != 0; ++j) tab.p[j] = tab.p[n - 1];
}

// Which rank walk the library takes by itself.  Measured on MI355X with the
// fused kernels over cold buffers (ratio of the deep walk's time to the wide
// one's; a deep workgroup covers 1024 chunks, MI355X has 256 compute units):
//   below ~1.4 deep workgroups per compute unit the deep walk starves the chip
//     (1 M elements: 1.2-1.8 with 16-bit gradients, 1.1-1.2 with fp32);
//   from there to ~2.5 per compute unit it wins at every rank count
//     (3-4 M 16-bit elements: 0.88-0.98; 2 M fp32: 0.92-0.93);
//   beyond that it keeps winning with many rank streams (64 ranks: 0.90-0.98 up
//     to 113 M elements), is even at 16 ranks (0.97-1.02; the GPT-3-175B block:
//     1156-1162 us against 1158-1188 us, fp32 gradients 1796 against 1853 us)
//     and loses at 8 ranks (1.02-1.10 from 6 M to 32 M elements).
// Below eight ranks the two are within noise of each other and the wide walk,
// with four times the workgroups, is kept.
constexpr int32_t kDeepMinRanks = 8;
constexpr int32_t kDeepAlwaysRanks = 16;      // from this many ranks on, deep at every size above the minimum
constexpr int64_t kDeepMinBlocks = 360;       // ~1.4 deep workgroups per compute unit
constexpr int64_t kDeepFewRanksMaxBlocks = 640;

// does the library's own choice of rank walk fall on the deep one?
inline bool deep_walk_pays(int gt, int32_t W, int64_t S)
{
    const int64_t E = gt == kF32 ? 4 : 8;
    const int64_t deep_blocks = ceil_div(S / E + 1, kReduceBlock * WalkShape<kF32, true, true>::C);
    if (W < kDeepMinRanks || deep_blocks < kDeepMinBlocks) return false;
    return W >= kDeepAlwaysRanks || deep_blocks < kDeepFewRanksMaxBlocks;
}
// May a fused update above kOneLaunchMaxBytes share a grid with an unshard above
// it?  Measured: with fp32 gradients (34 registers in the shared kernel) pairing
// a 336 MB update with a 302 MB unshard is 5 % faster than two launches, and 6 %
// on 64-rank units of 3.2 M elements; from 8.4 M elements per shard on the
// stand-alone kernel is the better one, and with 16-bit gradients (86 registers)
// pairing changes nothing.  A layout that asks for the deep walk gets the
// stand-alone kernel.
constexpr int64_t kPairMaxShard = 8 * 256 * 1024 * 4;      // 8.4 M elements
inline bool pairs_with_large_unshard(const fsdp_layout_t* L, int gt)
{
    return gt == kF32 && L->reduce_walk != FSDP_WALK_DEEP && L->S < kPairMaxShard;
}

// The half-chunk walk (plain fused updates only): single-wave workgroups, one load in flight per lane.  Measured
// on MI355X against the better of the wide and the deep walk, cold buffers (ratio of times):
//   16-bit gradients: 0.86-0.98 for 2 to 16 ranks at every shard size from 1 M to 113 M elements (the GPT-3-175B
//     block over 16 ranks: 1052 against 1163 us on the same buffers), even at 24 ranks, 1.0-1.13 from 32 ranks on
//     (the serial walk over the ranks is then too long a chain), and 1.1-1.4 below 1 M elements;
//   fp32 gradients: 0.92-0.99 from 8 ranks and 16 M elements on, 1.0-1.07 below 8 M elements.
constexpr int kHalfBlock = 64;
constexpr int32_t kHalf16MaxRanks = 16;
constexpr int64_t kHalf16MinShard = 1 << 20;
constexpr int32_t kHalfF32MinRanks = 8;
constexpr int64_t kHalfF32MinShard = 12 << 20;
inline bool half_walk_pays(int gt, int32_t W, int64_t S)
{
    if (gt == kF32) return W >= kHalfF32MinRanks && S >= kHalfF32MinShard;
    return W <= kHalf16MaxRanks && S >= kHalf16MinShard;
}
// does a plain fused stand-alone update take the half-chunk walk?
inline bool takes_half(int32_t walk, int gt, int32_t W, int64_t S)
{
    return walk == FSDP_WALK_AUTO ? half_walk_pays(gt, W, S) : walk == FSDP_WALK_HALF;
}

// does a launch that does not take the half-chunk walk take the deep one?  (A hint for the half-chunk walk leaves
// this choice to the library.)
inline bool walks_deep(int32_t walk, int gt, int32_t W, int64_t S)
{
    return walk == FSDP_WALK_AUTO || walk == FSDP_WALK_HALF ? deep_walk_pays(gt, W, S) : walk == FSDP_WALK_DEEP;
}
// would a stand-alone reduce kernel of this unit take the deep walk (the layout's hint, else the library's choice)?
inline bool wants_deep(const fsdp_layout_t* L, int gt) { return walks_deep(L->reduce_walk, gt, L->world_size, L->S); }

// walk: the layout's hint (FSDP_WALK_*).  The fused deep kernels exist in a
// plain instantiation as well, for launches that use no hybrid groups,
// accumulation, unscaling or carried partial sum: 109 instead of 152 registers
// with 16-bit gradients, 76 instead of 92 with fp32 ones.  Measured on MI355X
// with 113 M-element shards over 16 ranks: 5 % faster with fp32 gradients,
// within the run-to-run spread with bf16 ones (the kernels are bound by the
// memory system's handling of the read / write mix, not by occupancy).  The
// wide stand-alone kernels keep the one full instantiation: their plain form
// (84 instead of 102 registers) measured 3 % slower on 3.2 M-element shards
// over 64 ranks.
template <int GT, int PRE, bool FUSED>
void launch_reduce(const PtrTable& tab, const RsArgs& a, int32_t walk, hipStream_t st)
{
    constexpr int B = kReduceBlock;
    constexpr int E = WalkShape<GT, FUSED, false>::E;
    const bool plain = a.group == 0 && !a.cont && !a.accum && !a.unscale;
    if constexpr (FUSED) {
        if (plain && takes_half(walk, GT, a.W, a.S)) {
            const dim3 grid(static_cast<uint32_t>(ceil_div(a.S / 4 + 1, kHalfBlock * WalkShape<GT, true, false, true>::C)));
            hipLaunchKernelGGL((reduce_kernel<GT, PRE, true, false, kHalfBlock, true, true>), grid, dim3(kHalfBlock), 0, st,
                               tab, a);
            return;
        }
    }
    const bool deep = walks_deep(walk, GT, a.W, a.S);
    const dim3 block(B);
    if (deep) {
        const dim3 grid(static_cast<uint32_t>(ceil_div(a.S / E + 1, B * WalkShape<GT, FUSED, true>::C)));
        if constexpr (FUSED) {
            if (plain) {
                hipLaunchKernelGGL((reduce_kernel<GT, PRE, true, true, B, true>), grid, block, 0, st, tab, a);
                return;
            }
        }
        hipLaunchKernelGGL((reduce_kernel<GT, PRE, FUSED, true, B, false>), grid, block, 0, st, tab, a);
        return;
    }
    const dim3 grid(static_cast<uint32_t>(ceil_div(a.S / E + 1, B)));
    hipLaunchKernelGGL((reduce_kernel<GT, PRE, FUSED, false, B, false>), grid, block, 0, st, tab, a);
}

template <int GT, bool FUSED>
void launch_reduce_pre(int pre_mode, const PtrTable& tab, const RsArgs& a, int32_t walk, hipStream_t st)
{
    if (pre_mode == kPreNone) launch_reduce<GT, kPreNone, FUSED>(tab, a, walk, st);
    else if (pre_mode == kPreMul) launch_reduce<GT, kPreMul, FUSED>(tab, a, walk, st);
    else launch_reduce<GT, kPreDiv, FUSED>(tab, a, walk, st);
}

// Does the single-wave unshard read every shard with aligned 16-byte loads?  Shard w's loads start `head`
// elements in, where head brings its slot of the flat buffer to a 128-byte boundary.
bool light_unshard_fits(const float* const* shard_ptrs, int32_t W, int64_t S, const void* flat_out)
{
    if (S / 4 + 1 > 0x7FFFFFFFLL * kLightBlock) return false;       // tiles per shard must fit the grid's x dimension
    for (int32_t w = 0; w < W; ++w) {
        const uintptr_t dst = reinterpret_cast<uintptr_t>(flat_out) + static_cast<uintptr_t>(w) * static_cast<uintptr_t>(S) * 2;
        const uintptr_t head = ((128 - (dst & 127)) & 127) >> 1;
        if ((reinterpret_cast<uintptr_t>(shard_ptrs[w]) + 4 * head) & 15) return false;
    }
    return true;
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
    // Accumulation needs the old value of out[] until the end, so it cannot carry a partial sum there.
    if (opt.accumulate && W > kMaxRanks) return FSDP_ERR_INVALID_ARG;
    // More ranks than one launch takes: several launches, the partial sum carried in out[].  With hybrid
    // groups a launch takes whole groups, so that only the sum over the groups is carried.
    int32_t per_launch = kMaxRanks;
    if (opt.num_groups > 1) {
        if (L->world_size > kMaxRanks) return FSDP_ERR_INVALID_ARG;
        per_launch = kMaxRanks / L->world_size * L->world_size;
    }
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

    for (int32_t w0 = 0; w0 < W; w0 += per_launch) {
        const int32_t nw = W - w0 < per_launch ? W - w0 : per_launch;
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
        a.unscale = opt.unscale && a.last ? 1 : 0;     // the check and the unscaling act on the finished sum
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
            if (fuse_now) launch_reduce_pre<kBF16, true>(pre_mode, tab, a, L->reduce_walk, st);
            else launch_reduce_pre<kBF16, false>(pre_mode, tab, a, L->reduce_walk, st);
        } else if (grad_dtype == FSDP_F16) {
            if (fuse_now) launch_reduce_pre<kF16, true>(pre_mode, tab, a, L->reduce_walk, st);
            else launch_reduce_pre<kF16, false>(pre_mode, tab, a, L->reduce_walk, st);
        } else {
            if (fuse_now) launch_reduce_pre<kF32, true>(pre_mode, tab, a, L->reduce_walk, st);
            else launch_reduce_pre<kF32, false>(pre_mode, tab, a, L->reduce_walk, st);
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
    // One destination vector per lane.  The cast takes single-wave workgroups
    // with 8-byte vectors when every shard's 16-byte loads are aligned, else
    // workgroups of kBlock lanes with 16-byte vectors and an LDS window.
    const bool light = lp && light_unshard_fits(shard_ptrs, W, S, flat_out);
    const int64_t tiles = light ? ceil_div(S / 4 + 1, kLightBlock) : ceil_div(S / (lp ? 8 : 4) + 1, kBlock);
    if (!grid_ok(tiles * kMaxRanks)) return FSDP_ERR_OVERFLOW;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);

    for (int32_t w0 = 0; w0 < W; w0 += kMaxRanks) {
        const int32_t nw = W - w0 < kMaxRanks ? W - w0 : kMaxRanks;
        PtrTable tab = {};
        for (int32_t j = 0; j < nw; ++j) tab.p[j] = shard_ptrs[w0 + j];
        const dim3 grid(static_cast<uint32_t>(tiles * nw));
        if (light) {
            uint16_t* base = static_cast<uint16_t*>(flat_out) + static_cast<int64_t>(w0) * S;
            const dim3 grid2(static_cast<uint32_t>(tiles), static_cast<uint32_t>(nw));
            if (out_dtype == FSDP_F16)
                hipLaunchKernelGGL(unshard_lp_light_kernel<kF16>, grid2, dim3(kLightBlock), 0, st, tab, S, base);
            else
                hipLaunchKernelGGL(unshard_lp_light_kernel<kBF16>, grid2, dim3(kLightBlock), 0, st, tab, S, base);
        } else if (lp) {
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
    // and drain) is visible next to the smaller half.  For large halves it
    // still pays with fp32 gradients (5 % on 300 MB halves; the shared kernel
    // then needs 34 registers) up to the shard size given by
    // pairs_with_large_unshard; with 16-bit gradients (84 registers) sharing a
    // grid gains nothing on large halves, and their updates keep the
    // stand-alone kernel, which may take the deep walk.
    const int64_t reduce_bytes = dtype_size(grad_dtype) * L->P + 24 * L->S;
    const int64_t unshard_bytes = 6 * N->P;
    const bool small_half = (reduce_bytes < unshard_bytes ? reduce_bytes : unshard_bytes) <= kOneLaunchMaxBytes;
    const bool pair_large = pairs_with_large_unshard(L, static_cast<int>(grad_dtype));
    const bool one_launch = (small_half || pair_large) && L->world_size <= kMaxRanks &&
                            N->world_size <= kMaxRanks &&
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

int fsdp_reduce_scatter_hybrid_adam_fused(const fsdp_layout_t* L, const void* const* grad_ptrs, fsdp_dtype_t grad_dtype,
                                          int32_t num_groups, int32_t rank, float pre_div, float post_div,
                                          float* grad_shard_out, float* p_shard, float* exp_avg, float* exp_avg_sq,
                                          int64_t step, float lr, float beta1, float beta2, float eps, void* p_lp_out,
                                          void* hip_stream)
{
    int rc = check_reduce_args(L, grad_ptrs, grad_dtype, rank, pre_div, post_div, num_groups);
    if (rc != FSDP_OK) return rc;
    if (!p_shard || !exp_avg || !exp_avg_sq) return FSDP_ERR_NULL_PTR;
    rc = check_adam_args(step, lr, beta1, beta2, eps);
    if (rc != FSDP_OK) return rc;
    if (static_cast<int64_t>(L->world_size) * num_groups > kMaxRanks && !grad_shard_out) return FSDP_ERR_NULL_PTR;
    if (misaligned(p_shard, 4) || misaligned(exp_avg, 4) || misaligned(exp_avg_sq, 4) ||
        (grad_shard_out && misaligned(grad_shard_out, 4)) || (p_lp_out && misaligned(p_lp_out, 2)))
        return FSDP_ERR_INVALID_ARG;
    const AdamConsts c = make_adam_consts(step, lr, beta1, beta2, eps);
    ReduceOpts opt;
    opt.num_groups = num_groups;
    return reduce_driver(L, grad_ptrs, grad_dtype, rank, pre_div, post_div, grad_shard_out, true, p_shard, exp_avg,
                         exp_avg_sq, static_cast<uint16_t*>(p_lp_out), c, static_cast<hipStream_t>(hip_stream), opt);
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

int fsdp_reduce_scatter_accumulate_adam_fused(const fsdp_layout_t* L, const void* const* grad_ptrs,
                                              fsdp_dtype_t grad_dtype, int32_t rank, float pre_div, float post_div,
                                              float* grad_shard_acc, float* p_shard, float* exp_avg, float* exp_avg_sq,
                                              int64_t step, float lr, float beta1, float beta2, float eps,
                                              void* p_lp_out, void* hip_stream)
{
    int rc = check_reduce_args(L, grad_ptrs, grad_dtype, rank, pre_div, post_div);
    if (rc != FSDP_OK) return rc;
    if (!grad_shard_acc || !p_shard || !exp_avg || !exp_avg_sq) return FSDP_ERR_NULL_PTR;
    rc = check_adam_args(step, lr, beta1, beta2, eps);
    if (rc != FSDP_OK) return rc;
    if (misaligned(grad_shard_acc, 4) || misaligned(p_shard, 4) || misaligned(exp_avg, 4) || misaligned(exp_avg_sq, 4) ||
        (p_lp_out && misaligned(p_lp_out, 2)))
        return FSDP_ERR_INVALID_ARG;
    const AdamConsts c = make_adam_consts(step, lr, beta1, beta2, eps);
    ReduceOpts opt;
    opt.accumulate = true;
    return reduce_driver(L, grad_ptrs, grad_dtype, rank, pre_div, post_div, grad_shard_acc, true, p_shard, exp_avg,
                         exp_avg_sq, static_cast<uint16_t*>(p_lp_out), c, static_cast<hipStream_t>(hip_stream), opt);
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
    const bool light = light_unshard_fits(&shard, 1, L->S, lp_shard_out);
    const int64_t tiles = light ? ceil_div(L->S / 4 + 1, kLightBlock) : ceil_div(L->S / 8 + 1, kBlock);
    if (!grid_ok(tiles)) return FSDP_ERR_OVERFLOW;
    PtrTable tab = {};
    tab.p[0] = shard;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    uint16_t* out = static_cast<uint16_t*>(lp_shard_out);
    const dim3 grid(static_cast<uint32_t>(tiles));
    if (light && lp_dtype == FSDP_F16)
        hipLaunchKernelGGL(unshard_lp_light_kernel<kF16>, grid, dim3(kLightBlock), 0, st, tab, L->S, out);
    else if (light)
        hipLaunchKernelGGL(unshard_lp_light_kernel<kBF16>, grid, dim3(kLightBlock), 0, st, tab, L->S, out);
    else if (lp_dtype == FSDP_F16)
        hipLaunchKernelGGL(unshard_lp_kernel<kF16>, grid, dim3(kBlock), 0, st, tab, L->S, out, static_cast<int32_t>(tiles));
    else
        hipLaunchKernelGGL(unshard_lp_kernel<kBF16>, grid, dim3(kBlock), 0, st, tab, L->S, out, static_cast<int32_t>(tiles));
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
    const int64_t tiles = ceil_div(S / 8 + 1, kLightBlock);
    if (!grid_ok(tiles * kMaxRanks)) return FSDP_ERR_OVERFLOW;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    for (int32_t w0 = 0; w0 < W; w0 += kMaxRanks) {
        const int32_t nw = W - w0 < kMaxRanks ? W - w0 : kMaxRanks;
        PtrTable tab = {};
        for (int32_t j = 0; j < nw; ++j) tab.p[j] = lp_shard_ptrs[w0 + j];
        uint16_t* base = static_cast<uint16_t*>(flat_out) + static_cast<int64_t>(w0) * S;
        hipLaunchKernelGGL(gather_lp_kernel, dim3(static_cast<uint32_t>(tiles * nw)), dim3(kLightBlock), 0, st, tab, S,
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
    if (num_ranks <= 0) return FSDP_ERR_INVALID_ARG;
    for (int32_t i = 0; i < num_ranks; ++i) {
        if (!found_inf_ptrs[i]) return FSDP_ERR_NULL_PTR;
        if (misaligned(found_inf_ptrs[i], 4)) return FSDP_ERR_INVALID_ARG;
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    // one launch: every flag of the table (an optional carried flag, then `count` of the caller's from `first` on)
    // becomes the maximum over the table
    auto combine = [&](float* carried, int32_t first, int32_t count) {
        FlagTable tab = {};
        int32_t k = 0;
        if (carried) tab.p[k++] = carried;
        for (int32_t i = 0; i < count; ++i) tab.p[k++] = found_inf_ptrs[first + i];
        hipLaunchKernelGGL(found_inf_combine_kernel, dim3(1), dim3(64), 0, st, tab, k);
        return launch_status();
    };
    if (num_ranks <= kMaxRanks) return combine(nullptr, 0, num_ranks);
    // More flags than one table holds: a forward sweep in which each table also holds a flag of the table before
    // (the running maximum), then a backward sweep that hands the last table's result to the earlier ones.
    const int32_t per = kMaxRanks - 1;
    int32_t last_first = 0;
    for (int32_t first = 0; first < num_ranks; first += per) {
        const int32_t count = num_ranks - first < per ? num_ranks - first : per;
        const int rc = combine(first > 0 ? found_inf_ptrs[first - per] : nullptr, first, count);
        if (rc != FSDP_OK) return rc;
        last_first = first;
    }
    for (int32_t first = last_first - per; first >= 0; first -= per) {
        const int rc = combine(found_inf_ptrs[last_first], first, per);
        if (rc != FSDP_OK) return rc;
    }
    return FSDP_OK;
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
// A batch is planned while it is recorded: every fsdp_batch_add_* call either
// joins the last grid of the plan or opens a new step, and writes the member's
// kernel arguments once.  fsdp_batch_launch walks the plan and only fills in
// the Adam constants that depend on the step count.

namespace {

struct ReduceKind {
    int gt, pre_mode;
    bool operator==(const ReduceKind& o) const { return gt == o.gt && pre_mode == o.pre_mode; }
};

struct AdamHyper {
    float lr, beta1, beta2, eps;
    bool operator==(const AdamHyper& o) const
    {
        return lr == o.lr && beta1 == o.beta1 && beta2 == o.beta2 && eps == o.eps;
    }
};

int pre_mode_of(float pre)
{
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

struct fsdp_batch {
    // operations that cannot share a grid are kept as the caller gave them and
    // issued through their own entry points
    struct ReduceRec {
        const fsdp_layout_t* L;
        std::vector<const void*> raw;        // the caller's table
        fsdp_dtype_t dtype;
        int32_t rank;
        float pre, post;
        float *out, *p, *m, *v;
        uint16_t* p_lp;
        AdamHyper hyper;
    };
    struct UnshardRec {
        const fsdp_layout_t* L;
        std::vector<const void*> shards;
        void* out;
        fsdp_dtype_t dtype;
        bool lp;                             // the shards are 16-bit already: plain gather (fsdp_unshard_lp)
    };
    // one grid: up to kBatchOps reduce members of one kernel kind and up to
    // kBatchOps unshard members, their rank pointers in one pool
    struct Grid {
        BatchArgs args = {};                 // complete except for the members' Adam constants
        ReduceKind kind = {kF32, kPreNone};
        AdamHyper hyper[kBatchOps] = {};
        const fsdp_layout_t* u_layout[kBatchOps] = {};   // layouts of the unshard members
        int32_t walk0 = FSDP_WALK_AUTO;      // rank-walk hint of the first reduce member's layout
        int32_t n_ptrs = 0;
        int large_r = 0, large_u = 0;
        bool pairable = true;                // may a large unshard join the grid's large update?
        uint32_t r_blocks = 0, u_blocks = 0;
    };
    struct Step {
        enum Kind { kGrid, kReduce, kUnshard } kind;
        size_t index;                        // into grids, reduces or unshards
    };
    std::vector<ReduceRec> reduces;
    std::vector<UnshardRec> unshards;
    std::vector<Grid> grids;
    std::vector<Step> steps;

    Grid* open_grid() { return !steps.empty() && steps.back().kind == Step::kGrid ? &grids[steps.back().index] : nullptr; }
    Grid* new_grid()
    {
        grids.emplace_back();
        steps.push_back({Step::kGrid, grids.size() - 1});
        return &grids.back();
    }
};

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
    b->grids.clear();
    b->steps.clear();
    return FSDP_OK;
}

static int batch_add_unshard_impl(fsdp_batch_t* b, const fsdp_layout_t* L, const void* const* shard_ptrs, void* flat_out,
                                  fsdp_dtype_t out_dtype, bool lp)
{
    const int32_t W = L->world_size;
    const int64_t bytes = (lp ? 4 : 6) * L->P;
    const int64_t tiles = ceil_div(L->S / 8 + 1, kBlock);
    // A grid takes up to kBatchOps 16-bit unshards of at most kMaxRanks ranks
    // each while the pointer pool lasts; of the operations above
    // kOneLaunchMaxBytes at most one of each kind, and both kinds together only
    // with fp32 gradients (see the prefetch entry point).
    const bool batchable = W <= kMaxRanks && (lp || out_dtype == FSDP_BF16) && grid_ok(tiles * W);
    try {
        if (!batchable) {
            fsdp_batch::UnshardRec r;
            r.L = L;
            r.shards.assign(shard_ptrs, shard_ptrs + W);
            r.out = flat_out;
            r.dtype = out_dtype;
            r.lp = lp;
            b->unshards.push_back(std::move(r));
            b->steps.push_back({fsdp_batch::Step::kUnshard, b->unshards.size() - 1});
            return FSDP_OK;
        }
        const bool is_large = bytes > kOneLaunchMaxBytes;
        fsdp_batch::Grid* g = b->open_grid();
        if (!g || g->args.n_unshard == kBatchOps || g->n_ptrs + W > kBatchPtrs ||
            !grid_ok(tiles * W + g->r_blocks + g->u_blocks) ||
            (is_large && (g->large_u > 0 || (g->large_r > 0 && !g->pairable))))
            g = b->new_grid();
        g->large_u += is_large ? 1 : 0;
        g->u_layout[g->args.n_unshard] = L;
        BatchUnshardOp& o = g->args.u[g->args.n_unshard];
        o.ptr0 = g->n_ptrs;
        for (int32_t w = 0; w < W; ++w) g->args.ptrs[g->n_ptrs++] = shard_ptrs[w];
        o.S = L->S;
        o.out = static_cast<uint16_t*>(flat_out);
        o.tiles = static_cast<int32_t>(tiles);
        o.lp = lp ? 1 : 0;
        g->u_blocks += static_cast<uint32_t>(tiles * W);
        g->args.u_end[g->args.n_unshard] = g->u_blocks;
        ++g->args.n_unshard;
    } catch (const std::bad_alloc&) {
        return FSDP_ERR_OOM;
    }
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
    return batch_add_unshard_impl(b, L, reinterpret_cast<const void* const*>(shard_ptrs), flat_out, out_dtype, false);
}

int fsdp_batch_add_unshard_lp(fsdp_batch_t* b, const fsdp_layout_t* L, const void* const* lp_shard_ptrs, void* flat_out)
{
    if (!b || !L || !lp_shard_ptrs || !flat_out) return FSDP_ERR_NULL_PTR;
    for (int32_t w = 0; w < L->world_size; ++w) {
        if (!lp_shard_ptrs[w]) return FSDP_ERR_NULL_PTR;
        if (misaligned(lp_shard_ptrs[w], 2)) return FSDP_ERR_INVALID_ARG;
    }
    if (misaligned(flat_out, 2)) return FSDP_ERR_INVALID_ARG;
    // the dtype is not looked at: a gather moves either 16-bit kind
    return batch_add_unshard_impl(b, L, lp_shard_ptrs, flat_out, FSDP_BF16, true);
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

    const int32_t W = L->world_size;
    const int32_t W_padded = (W + kMaxWideRanks - 1) / kMaxWideRanks * kMaxWideRanks;   // whole wide batches
    const int64_t bytes = dtype_size(grad_dtype) * L->P + 24 * L->S;
    const int64_t E = grad_dtype == FSDP_F32 ? 4 : 8;
    const int64_t nb = ceil_div(L->S / E + 1, kBlock);
    const bool batchable = W <= kMaxRanks && grid_ok(nb);
    const AdamHyper hyper = {lr, beta1, beta2, eps};
    try {
        if (!batchable) {
            fsdp_batch::ReduceRec r;
            r.L = L;
            r.raw.assign(grad_ptrs, grad_ptrs + W);
            r.dtype = grad_dtype;
            r.rank = rank;
            r.pre = pre_div;
            r.post = post_div;
            r.out = grad_shard_out;
            r.p = p_shard; r.m = exp_avg; r.v = exp_avg_sq;
            r.p_lp = static_cast<uint16_t*>(p_lp_out);
            r.hyper = hyper;
            b->reduces.push_back(std::move(r));
            b->steps.push_back({fsdp_batch::Step::kReduce, b->reduces.size() - 1});
            return FSDP_OK;
        }
        const ReduceKind k = {static_cast<int>(grad_dtype), pre_mode_of(pre_div)};
        const bool is_large = bytes > kOneLaunchMaxBytes;
        const bool pairable = pairs_with_large_unshard(L, k.gt);
        fsdp_batch::Grid* g = b->open_grid();
        if (!g || g->args.n_reduce == kBatchOps || (g->args.n_reduce > 0 && !(k == g->kind)) ||
            g->n_ptrs + W_padded > kBatchPtrs || !grid_ok(nb + g->r_blocks + g->u_blocks) ||
            (is_large && (g->large_r > 0 || (g->large_u > 0 && !pairable))))
            g = b->new_grid();
        if (g->args.n_reduce == 0) {
            g->kind = k;
            g->walk0 = L->reduce_walk;
        }
        g->large_r += is_large ? 1 : 0;
        if (is_large) g->pairable = pairable;
        BatchReduceOp& o = g->args.r[g->args.n_reduce];
        o.ptr0 = g->n_ptrs;
        const int64_t off = static_cast<int64_t>(rank) * L->S * dtype_size(grad_dtype);
        for (int32_t w = 0; w < W_padded; ++w)     // the padding repeats the last rank's pointer; its adds are skipped
            g->args.ptrs[g->n_ptrs++] = static_cast<const char*>(grad_ptrs[w < W ? w : W - 1]) + off;
        RsArgs& a = o.a;
        a = RsArgs{};
        float recip;
        a.pre_c = pre_div;
        if (k.pre_mode == kPreMul) { is_pow2_float(pre_div, &recip); a.pre_c = recip; }
        a.post_c = post_div;
        if (is_pow2_float(post_div, &recip)) { a.post_mul = 1; a.post_c = recip; }
        a.W = W;
        a.last = 1;
        a.S = L->S;
        a.out = grad_shard_out;
        a.p = p_shard; a.m = exp_avg; a.v = exp_avg_sq; a.p_lp = static_cast<uint16_t*>(p_lp_out);
        g->hyper[g->args.n_reduce] = hyper;
        g->r_blocks += static_cast<uint32_t>(nb);
        g->args.r_end[g->args.n_reduce] = g->r_blocks;
        ++g->args.n_reduce;
    } catch (const std::bad_alloc&) {
        return FSDP_ERR_OOM;
    }
    return FSDP_OK;
}

namespace {
// a grid whose only member is one unshard goes out through the stand-alone entry point
inline bool lone_unshard(const fsdp_batch::Grid& g) { return g.args.n_reduce == 0 && g.args.n_unshard == 1; }
// ... and so does a grid whose only member is one update: the stand-alone kernel may take the deep or the half-chunk
// walk, and for a small update its few kernel arguments save half a microsecond against the shared kernel's 4 KiB
inline bool lone_update(const fsdp_batch::Grid& g) { return g.args.n_reduce == 1 && g.args.n_unshard == 0; }

// launches of one plan step: (kernel, updates, unshards, workgroups) of launch j of the step; returns the count
int32_t step_launches(const fsdp_batch_t* b, const fsdp_batch::Step& s, int32_t j, int32_t* kernel, int32_t* n_upd,
                      int32_t* n_uns, int64_t* wgs)
{
    if (s.kind == fsdp_batch::Step::kGrid) {
        const fsdp_batch::Grid& g = b->grids[s.index];
        const bool lone = lone_update(g);
        *kernel = lone ? FSDP_KERNEL_REDUCE : FSDP_KERNEL_BATCH;
        *n_upd = g.args.n_reduce;
        *n_uns = g.args.n_unshard;
        *wgs = static_cast<int64_t>(g.r_blocks) + g.u_blocks;
        if (lone_unshard(g)) {   // issued through fsdp_unshard / fsdp_unshard_lp, which choose their own kernel and grid
            const BatchUnshardOp& o = g.args.u[0];
            const fsdp_layout_t* UL = g.u_layout[0];
            const bool light = !o.lp && light_unshard_fits(reinterpret_cast<const float* const*>(g.args.ptrs + o.ptr0),
                                                           UL->world_size, UL->S, o.out);
            *kernel = o.lp ? FSDP_KERNEL_GATHER_LP : (light ? FSDP_KERNEL_UNSHARD_LP_LIGHT : FSDP_KERNEL_UNSHARD_LP);
            *wgs = (light ? ceil_div(UL->S / 4 + 1, kLightBlock)
                          : ceil_div(UL->S / 8 + 1, o.lp ? kLightBlock : kBlock)) * UL->world_size;
        }
        if (lone) {   // the stand-alone kernel sizes its own grid by the rank walk it takes
            const RsArgs& a = g.args.r[0].a;
            const int64_t E = g.kind.gt == kF32 ? 4 : 8;
            const bool deep = walks_deep(g.walk0, g.kind.gt, a.W, a.S);
            *wgs = takes_half(g.walk0, g.kind.gt, a.W, a.S) ? ceil_div(a.S / 4 + 1, kHalfBlock * WalkShape<kBF16, true, false, true>::C)
                                                           : ceil_div(a.S / E + 1, deep ? kReduceBlock * 4 : kReduceBlock);
        }
        return 1;
    }
    if (s.kind == fsdp_batch::Step::kReduce) {
        const fsdp_batch::ReduceRec& r = b->reduces[s.index];
        *kernel = FSDP_KERNEL_REDUCE;
        *n_upd = 1;
        *n_uns = 0;
        const int64_t E = r.dtype == FSDP_F32 ? 4 : 8;
        const bool deep = wants_deep(r.L, static_cast<int>(r.dtype));
        *wgs = ceil_div(r.L->S / E + 1, deep ? kReduceBlock * 4 : kReduceBlock);
        return static_cast<int32_t>(ceil_div(r.L->world_size, kMaxRanks));
    }
    const fsdp_batch::UnshardRec& u = b->unshards[s.index];
    const int32_t n = static_cast<int32_t>(ceil_div(u.L->world_size, kMaxRanks));
    const int32_t nw = j + 1 < n ? kMaxRanks : u.L->world_size - j * kMaxRanks;
    const bool light = !u.lp && u.dtype != FSDP_F32 &&
                       light_unshard_fits(reinterpret_cast<const float* const*>(u.shards.data()), u.L->world_size, u.L->S, u.out);
    *kernel = u.lp ? FSDP_KERNEL_GATHER_LP
                   : (u.dtype == FSDP_F32 ? FSDP_KERNEL_UNSHARD_F32
                                          : (light ? FSDP_KERNEL_UNSHARD_LP_LIGHT : FSDP_KERNEL_UNSHARD_LP));
    *n_upd = 0;
    *n_uns = 1;
    *wgs = light ? ceil_div(u.L->S / 4 + 1, kLightBlock) * nw
                 : ceil_div(u.L->S / (!u.lp && u.dtype == FSDP_F32 ? 4 : 8) + 1, u.lp ? kLightBlock : kBlock) * nw;
    return n;
}
}  // namespace

int fsdp_batch_launch_count(const fsdp_batch_t* b, int32_t* count)
{
    if (!b || !count) return FSDP_ERR_NULL_PTR;
    int64_t n = 0;
    int32_t k, nu, ns;
    int64_t w;
    for (const fsdp_batch::Step& s : b->steps) n += step_launches(b, s, 0, &k, &nu, &ns, &w);
    if (n > 0x7FFFFFFF) return FSDP_ERR_OVERFLOW;
    *count = static_cast<int32_t>(n);
    return FSDP_OK;
}

int fsdp_batch_launch_info(const fsdp_batch_t* b, int32_t i, int32_t* kernel, int32_t* n_updates, int32_t* n_unshards,
                           int64_t* workgroups)
{
    if (!b) return FSDP_ERR_NULL_PTR;
    if (i < 0) return FSDP_ERR_RANK_RANGE;
    int64_t first = 0;
    for (const fsdp_batch::Step& s : b->steps) {
        int32_t k, nu, ns;
        int64_t w;
        const int32_t n = step_launches(b, s, 0, &k, &nu, &ns, &w);
        if (i < first + n) {
            step_launches(b, s, static_cast<int32_t>(i - first), &k, &nu, &ns, &w);
            if (kernel) *kernel = k;
            if (n_updates) *n_updates = nu;
            if (n_unshards) *n_unshards = ns;
            if (workgroups) *workgroups = w;
            return FSDP_OK;
        }
        first += n;
    }
    return FSDP_ERR_RANK_RANGE;
}

const char* fsdp_kernel_name(int32_t kernel)
{
    switch (kernel) {
        case FSDP_KERNEL_BATCH: return "batch_kernel";
        case FSDP_KERNEL_REDUCE: return "reduce_kernel";
        case FSDP_KERNEL_UNSHARD_LP: return "unshard_lp_kernel";
        case FSDP_KERNEL_UNSHARD_F32: return "unshard_f32_kernel";
        case FSDP_KERNEL_GATHER_LP: return "gather_lp_kernel";
        case FSDP_KERNEL_UNSHARD_LP_LIGHT: return "unshard_lp_light_kernel";
        default: return nullptr;
    }
}

int fsdp_batch_launch(const fsdp_batch_t* b, int64_t step, void* hip_stream)
{
    if (!b) return FSDP_ERR_NULL_PTR;
    if (step < 1) return FSDP_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    // the step-dependent Adam constants, computed once per distinct set of hyper-parameters
    AdamHyper last_hyper = {};
    AdamConsts last_consts = {};
    bool have_consts = false;
    auto consts_for = [&](const AdamHyper& h) -> const AdamConsts& {
        if (!have_consts || !(h == last_hyper)) {
            last_consts = make_adam_consts(step, h.lr, h.beta1, h.beta2, h.eps);
            last_hyper = h;
            have_consts = true;
        }
        return last_consts;
    };

    for (const fsdp_batch::Step& s : b->steps) {
        int rc = FSDP_OK;
        if (s.kind == fsdp_batch::Step::kReduce) {
            const fsdp_batch::ReduceRec& r = b->reduces[s.index];
            rc = fsdp_reduce_scatter_adam_fused(r.L, r.raw.data(), r.dtype, r.rank, r.pre, r.post, r.out, r.p, r.m, r.v,
                                                step, r.hyper.lr, r.hyper.beta1, r.hyper.beta2, r.hyper.eps, r.p_lp,
                                                hip_stream);
        } else if (s.kind == fsdp_batch::Step::kUnshard) {
            const fsdp_batch::UnshardRec& u = b->unshards[s.index];
            rc = u.lp ? fsdp_unshard_lp(u.L, u.shards.data(), u.out, hip_stream)
                      : fsdp_unshard(u.L, reinterpret_cast<const float* const*>(u.shards.data()), u.out, u.dtype,
                                     hip_stream);
        } else {
            const fsdp_batch::Grid& g = b->grids[s.index];
            if (lone_unshard(g)) {
                const BatchUnshardOp& o = g.args.u[0];
                const fsdp_layout_t* UL = g.u_layout[0];
                rc = o.lp ? fsdp_unshard_lp(UL, g.args.ptrs + o.ptr0, o.out, hip_stream)
                          : fsdp_unshard(UL, reinterpret_cast<const float* const*>(g.args.ptrs + o.ptr0), o.out, FSDP_BF16,
                                         hip_stream);
                if (rc != FSDP_OK) return rc;
                continue;
            }
            BatchArgs a = g.args;
            for (int32_t i = 0; i < a.n_reduce; ++i) a.r[i].a.adam = consts_for(g.hyper[i]);
            if (lone_update(g)) {
                // the stand-alone kernel, which may take the deep or the half-chunk rank walk
                PtrTable tab = {};
                const int32_t W_padded = (a.r[0].a.W + kMaxWideRanks - 1) / kMaxWideRanks * kMaxWideRanks;
                for (int32_t w = 0; w < W_padded; ++w) tab.p[w] = a.ptrs[a.r[0].ptr0 + w];
                if (g.kind.gt == kBF16) launch_reduce_pre<kBF16, true>(g.kind.pre_mode, tab, a.r[0].a, g.walk0, st);
                else if (g.kind.gt == kF16) launch_reduce_pre<kF16, true>(g.kind.pre_mode, tab, a.r[0].a, g.walk0, st);
                else launch_reduce_pre<kF32, true>(g.kind.pre_mode, tab, a.r[0].a, g.walk0, st);
            } else {
                // a grid without reduce members never enters the reduce code, so any instantiation serves
                launch_batch_grid(a.n_reduce > 0 ? g.kind : ReduceKind{kF32, kPreNone}, a, g.r_blocks + g.u_blocks, st);
            }
            rc = launch_status();
        }
        if (rc != FSDP_OK) return rc;
    }
    return FSDP_OK;
}

}  // extern "C"
