/*
 * fsdp_flat.h -- C ABI of libfsdp_flat: the per-rank FlatParameter data path of
 * Fully Sharded Data Parallel (arXiv 2304.11277) for AMD MI355X (gfx950).
 *
 * Notation (Sec. 3.2.1): a unit has p parameters with numels n_i,
 * off_i = sum_{j<i} n_j, N = off_p; W is the sharding factor (full sharding:
 * the world size); S = ceil(N / W) is the shard size, P = S * W the padded
 * FlatParameter size, pad = P - N (at most W - 1).
 *
 * Conventions shared by every entry point
 *  - Return value: FSDP_OK (0) or a negative fsdp_status_t.  All argument
 *    checks happen on the host before anything is launched; on error nothing
 *    has been launched and no output is written.
 *  - "dev" pointers are device (HBM) addresses; pointer *tables* (param_ptrs,
 *    shard_ptrs, grad_ptrs) are HOST arrays of device addresses and are read
 *    during the call only.  The caller owns every device buffer; the library
 *    owns only fsdp_layout_t (host memory).
 *  - Compute calls are asynchronous on hip_stream (a hipStream_t passed as
 *    void*; NULL = the default stream) of the current device.  They never
 *    synchronise, never allocate and may be captured in a HIP graph (kernel
 *    arguments, the Adam step count and its bias corrections among them, are
 *    then fixed at capture: re-capture, or update the graph's kernel nodes, to
 *    advance the step).
 *  - Device buffers need only element alignment (4 B for fp32, 2 B for bf16),
 *    so contiguous shards base + w * S with odd S are legal.  Buffers of
 *    different roles must not overlap.
 *  - bf16 is the upper half of an IEEE binary32 pattern (uint16_t).
 *  - A layout is immutable after init; calls that share a layout may run
 *    concurrently from several host threads and on several streams.  The
 *    library keeps no mutable state of its own besides the per-thread value
 *    behind fsdp_last_hip_error().
 */
#ifndef FSDP_FLAT_H
#define FSDP_FLAT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fsdp_layout fsdp_layout_t;   /* opaque, library-owned, host memory */
typedef struct fsdp_batch fsdp_batch_t;     /* opaque, library-owned, host memory */

/* FSDP_F16 is IEEE binary16; both 16-bit kinds travel as uint16_t bit patterns.
 * A 4-byte integer at the ABI.  For C++ translation units the underlying type
 * is fixed, so that any integer a caller passes is a representable value and
 * the library's range check (FSDP_ERR_BAD_DTYPE) is well defined. */
#ifdef __cplusplus
typedef enum fsdp_dtype : int32_t { FSDP_F32 = 0, FSDP_BF16 = 1, FSDP_F16 = 2 } fsdp_dtype_t;
#else
typedef enum fsdp_dtype { FSDP_F32 = 0, FSDP_BF16 = 1, FSDP_F16 = 2 } fsdp_dtype_t;
#endif

typedef enum {
    FSDP_OK = 0,
    FSDP_ERR_INVALID_ARG = -1,  /* non-positive count, negative dim, N == 0, bad factor / hyper-parameter,
                                   misaligned device pointer */
    FSDP_ERR_NULL_PTR = -2,     /* a required pointer (or table entry) is NULL */
    FSDP_ERR_OVERFLOW = -3,     /* a numel or 4 * P does not fit in int64 */
    FSDP_ERR_OOM = -4,          /* host allocation failed */
    FSDP_ERR_BAD_DTYPE = -5,    /* dtype enum out of range */
    FSDP_ERR_RANK_RANGE = -6,   /* rank or parameter index out of range */
    FSDP_ERR_HIP = -7           /* a kernel launch failed; see fsdp_last_hip_error() */
} fsdp_status_t;

/* Maximum number of rank pointers one kernel launch takes; larger W is split
 * into several launches by the library (results are unchanged). */
#define FSDP_MAX_RANKS_PER_LAUNCH 64

/* ---- layout (Sec. 3.2.1: flatten-concat-pad-chunk) -------------------------
 * dims:  host, all parameters' dims concatenated in parameter order.
 * ndims: host [num_params]; 0 = scalar (numel 1); a zero dim = numel 0 (legal).
 * Computes off_i (exclusive prefix sum), N, S, P, pad.  Host only; touches no
 * device.  *out must be released with fsdp_layout_destroy. */
int fsdp_layout_init(const int64_t* dims, const int32_t* ndims, int32_t num_params,
                     int32_t world_size, fsdp_layout_t** out);
void fsdp_layout_destroy(fsdp_layout_t* layout);           /* NULL is a no-op */

/* fsdp_layout_init with a tuning hint that is stored in the (immutable) layout:
 * how the reduce-scatter kernels of Sec. 3 / eq. (1) walk the W rank buffers
 * for this unit.  Both walks add in rank order and give the same bits.
 *   FSDP_WALK_WIDE: a lane owns one 16-byte chunk (and loads one to four ranks
 *                   at a time, by gradient dtype);
 *   FSDP_WALK_DEEP: a lane owns four chunks and loads one rank at a time;
 *   FSDP_WALK_HALF: fused updates without hybrid groups, accumulation or
 *                   unscaling and with at most 64 ranks (others: as AUTO
 *                   without it): a lane owns four elements (with 16-bit
 *                   gradients an 8-byte load per rank), keeps one load in
 *                   flight and reads and writes p, m, v contiguously across
 *                   the wave, in workgroups of 64 lanes;
 *   FSDP_WALK_AUTO (what fsdp_layout_init uses): the library's choice, from
 *                   measurements on MI355X.  Fused updates that use none of
 *                   the variants: half with 16-bit gradients up to 16 ranks
 *                   from 1 Mi elements per shard on, and with fp32 gradients
 *                   from 8 ranks and 12 Mi elements on.  Otherwise deep when
 *                   the shard fills at least 360 deep workgroups (1.5 M fp32
 *                   or 2.9 M 16-bit elements) and the unit has 16 ranks or
 *                   more, or 8 to 15 ranks and fewer than 640 deep
 *                   workgroups; else wide.
 * The hint applies to the stand-alone reduce kernels (fsdp_reduce_scatter_local,
 * _adam_fused, _hybrid, _accumulate, _unscale, the two-launch form of
 * _prefetch_unshard and a batch's lone large update); kernels that share a grid
 * with an unshard always walk wide.  Any other value: FSDP_ERR_INVALID_ARG. */
enum { FSDP_WALK_AUTO = 0, FSDP_WALK_WIDE = 1, FSDP_WALK_DEEP = 2, FSDP_WALK_HALF = 3 };
int fsdp_layout_init_ex(const int64_t* dims, const int32_t* ndims, int32_t num_params,
                        int32_t world_size, int32_t reduce_walk, fsdp_layout_t** out);

/* Queries (host only).  Any out pointer may be NULL to skip that field. */
int fsdp_layout_info(const fsdp_layout_t* layout, int64_t* numel /*N*/, int64_t* padded /*P*/,
                     int64_t* shard /*S*/, int64_t* pad, int32_t* num_params, int32_t* world_size);
int fsdp_layout_param(const fsdp_layout_t* layout, int32_t i, int64_t* offset /*off_i*/,
                      int64_t* numel /*n_i*/);

/* Sec. 3.2.3: the original parameters are views into the unsharded
 * FlatParameter.  *out = flat_base + off_i * sizeof(dtype); zero bytes move. */
int fsdp_view_ptr(const fsdp_layout_t* layout, void* flat_base, fsdp_dtype_t dtype, int32_t i,
                  void** out);

/* Convention of this library (the paper's eq. (1) is a plain sum): split the
 * data-parallel mean's divisor W as pre * post, pre being the smallest power of
 * two that divides W with pre * pre >= W or, if there is none, the largest power
 * of two dividing W.  W=8 -> (4,2), 12 -> (4,3), 16 -> (4,4), 64 -> (8,8),
 * 6 -> (2,3), odd W -> (1,W).  A power-of-two pre makes the pre-divide exact. */
int fsdp_default_divide_factors(int32_t world_size, float* pre, float* post);

/* ---- Sec. 3.2.1: build the sharded FlatParameter ---------------------------
 * param_ptrs: host [p] of dev fp32 arrays, parameter i holding n_i elements in
 *             row-major order (entries with n_i == 0 are ignored, may be NULL).
 * shard_ptrs: host [W] of dev fp32 arrays of S elements each (written).
 * shard_w[k] = flat[w * S + k] where flat = concat_i(param_i) followed by pad
 * zeros (+0.0f).  Every element of every shard is written exactly once. */
int fsdp_flatten_shard(const fsdp_layout_t* layout, const void* const* param_ptrs,
                       float* const* shard_ptrs, void* hip_stream);

/* ---- Sec. 3 / 3.2.1 unshard (AllGather with even inputs into one tensor),
 * fused with Sec. 4.4's full-to-low precision cast of each local shard -------
 * shard_ptrs: host [W] of dev fp32 shards, S elements each (read).
 * flat_out:   dev, P elements of out_dtype (written, pad included).
 * FSDP_BF16: flat_out[w * S + k] = bf16_rne(shard_w[k]) -- round to nearest,
 * ties to even; NaN keeps sign and top payload bits and is made quiet;
 * denormals are rounded, not flushed.  FSDP_F16: the same with IEEE binary16
 * (overflow gives Inf, small results land on the subnormal grid).
 * FSDP_F32: plain gather copy. */
int fsdp_unshard(const fsdp_layout_t* layout, const float* const* shard_ptrs, void* flat_out,
                 fsdp_dtype_t out_dtype, void* hip_stream);

/* ---- Sec. 3 / Sec. 3.2.2 eq. (1): ReduceScatter, this rank's share ----------
 * grad_ptrs: host [W] of dev unsharded gradient buffers (P elements of
 *            grad_dtype each); only elements [rank * S, (rank + 1) * S) of each
 *            are read.
 * grad_shard_out: dev fp32 [S] (written).
 * out[k] = ((x_0 / pre) + (x_1 / pre) + ... + (x_{W-1} / pre)) / post with
 * x_w = (float) grad_w[rank * S + k] (bf16 and fp16 upcasts are exact); strictly in rank
 * order, one binary32 division and addition per rank, no fused multiply-add,
 * accumulator initialised from rank 0's term.  pre, post: finite and > 0. */
int fsdp_reduce_scatter_local(const fsdp_layout_t* layout, const void* const* grad_ptrs,
                              fsdp_dtype_t grad_dtype, int32_t rank, float pre_div, float post_div,
                              float* grad_shard_out, void* hip_stream);

/* ---- Sec. 3 / Sec. 5.4: optimizer step on the sharded state (Adam) ---------
 * p_shard, exp_avg, exp_avg_sq: dev fp32 [S], updated in place; g_shard: dev
 * fp32 [S], read.  step >= 1 is the step count after increment.
 * m = b1 m + (1 - b1) g;  v = b2 v + (1 - b2) g g;
 * p = p - (lr / (1 - b1^step)) * (m / (sqrt(v) / sqrt(1 - b2^step) + eps)).
 * binary32 element arithmetic, bias corrections evaluated in binary64 on the
 * host.  Requires lr finite, 0 <= b1, b2 < 1, eps >= 0. */
int fsdp_shard_adam_step(const fsdp_layout_t* layout, float* p_shard, const float* g_shard,
                         float* exp_avg, float* exp_avg_sq, int64_t step, float lr, float beta1,
                         float beta2, float eps, void* hip_stream);

/* ---- fused reduce-scatter + Adam (same results as the two calls above) -----
 * The reduced gradient stays in registers.  grad_shard_out (dev fp32 [S]) and
 * p_lp_out (dev bf16 [S], receives bf16_rne of the updated p_shard, i.e. the
 * next unshard's local cast) may each be NULL to skip that output.  With
 * W > FSDP_MAX_RANKS_PER_LAUNCH, grad_shard_out is required (it carries the
 * partial sum between launches). */
int fsdp_reduce_scatter_adam_fused(const fsdp_layout_t* layout, const void* const* grad_ptrs,
                                   fsdp_dtype_t grad_dtype, int32_t rank, float pre_div,
                                   float post_div, float* grad_shard_out, float* p_shard,
                                   float* exp_avg, float* exp_avg_sq, int64_t step, float lr,
                                   float beta1, float beta2, float eps, void* p_lp_out,
                                   void* hip_stream);

/* ---- Sec. 3.3.2 backward prefetching as ONE launch ---------------------------
 * The fused reduce-scatter + Adam of one unit (arguments as above) together
 * with the unshard of another unit (next_*: arguments as fsdp_unshard), which
 * must not depend on each other: the buffers of the two halves must not
 * overlap.  The paper issues the next AllGather before the current
 * ReduceScatter on separate streams; here both share one grid, so the drain of
 * one half overlaps the ramp of the other with no cross-queue synchronisation.
 * Results are bit-identical to calling fsdp_reduce_scatter_adam_fused and
 * fsdp_unshard one after the other, which is also what happens (two launches)
 * when either W exceeds FSDP_MAX_RANKS_PER_LAUNCH, when next_out_dtype is
 * FSDP_F32, or when both halves move more than 128 MiB and the gradients are
 * 16-bit or the shard has 8.4 M elements or more (measured: the shared grid
 * pays for large fp32 halves, not for 16-bit ones). */
int fsdp_reduce_scatter_adam_prefetch_unshard(const fsdp_layout_t* layout, const void* const* grad_ptrs,
                                              fsdp_dtype_t grad_dtype, int32_t rank, float pre_div,
                                              float post_div, float* grad_shard_out, float* p_shard,
                                              float* exp_avg, float* exp_avg_sq, int64_t step, float lr,
                                              float beta1, float beta2, float eps, void* p_lp_out,
                                              const fsdp_layout_t* next_layout,
                                              const float* const* next_shard_ptrs, void* next_flat_out,
                                              fsdp_dtype_t next_out_dtype, void* hip_stream);

/* ---- Sec. 3.2.2 hybrid sharding: reduce-scatter inside each sharded group,
 * then all-reduce of the shards across the groups -- this rank's result --------
 * layout was built with world_size = F, the sharding factor; the world has
 * num_groups * F ranks.  grad_ptrs: host [num_groups * F], group-major
 * (grad_ptrs[i * F + l] = local rank l of sharded group i), P elements each;
 * rank = this rank's position l in its sharded group.
 * inner_i = (x_{i,0} / pre) + ... + (x_{i,F-1} / pre) in local-rank order,
 * out[k] = (inner_0 + inner_1 + ... ) / post in group order (eq. (1): the sum
 * over all ranks as a sum over groups of group sums; in binary32 this two-level
 * order is its own result).  num_groups = 1 equals fsdp_reduce_scatter_local bit
 * for bit.  Requires F <= FSDP_MAX_RANKS_PER_LAUNCH; more ranks in total than
 * that are taken as several launches of whole groups, with the same bits. */
int fsdp_reduce_scatter_hybrid(const fsdp_layout_t* layout, const void* const* grad_ptrs,
                               fsdp_dtype_t grad_dtype, int32_t num_groups, int32_t rank,
                               float pre_div, float post_div, float* grad_shard_out, void* hip_stream);
/* The same reduction with the sharded Adam step (Sec. 5.4) applied to the result
 * while it is in registers: what fsdp_reduce_scatter_adam_fused is to
 * fsdp_reduce_scatter_local, with the same outputs, options and bits as
 * fsdp_reduce_scatter_hybrid followed by fsdp_shard_adam_step.  grad_shard_out
 * may be NULL unless num_groups * F > FSDP_MAX_RANKS_PER_LAUNCH (it then carries
 * the sum over the groups between launches); p_lp_out may be NULL. */
int fsdp_reduce_scatter_hybrid_adam_fused(const fsdp_layout_t* layout, const void* const* grad_ptrs,
                                          fsdp_dtype_t grad_dtype, int32_t num_groups, int32_t rank,
                                          float pre_div, float post_div, float* grad_shard_out,
                                          float* p_shard, float* exp_avg, float* exp_avg_sq, int64_t step,
                                          float lr, float beta1, float beta2, float eps, void* p_lp_out,
                                          void* hip_stream);

/* ---- Sec. 3.3.4 gradient accumulation --------------------------------------
 * With communication: every micro-batch is reduce-scattered and added to the
 * sharded gradient the rank keeps: grad_shard_acc[k] = grad_shard_acc[k] +
 * reduce_scatter(...)[k] (arguments as fsdp_reduce_scatter_local; the buffer is
 * read and written).  Requires W <= FSDP_MAX_RANKS_PER_LAUNCH. */
int fsdp_reduce_scatter_accumulate(const fsdp_layout_t* layout, const void* const* grad_ptrs,
                                   fsdp_dtype_t grad_dtype, int32_t rank, float pre_div,
                                   float post_div, float* grad_shard_acc, void* hip_stream);
/* The last micro-batch of an accumulation with communication: the same update
 * of grad_shard_acc (read and written; it ends holding the whole accumulated
 * gradient) and, in the same launch, the sharded Adam step (Sec. 5.4) on that
 * gradient: the bits of fsdp_reduce_scatter_accumulate followed by
 * fsdp_shard_adam_step.  p_lp_out may be NULL.  Requires
 * W <= FSDP_MAX_RANKS_PER_LAUNCH. */
int fsdp_reduce_scatter_accumulate_adam_fused(const fsdp_layout_t* layout, const void* const* grad_ptrs,
                                              fsdp_dtype_t grad_dtype, int32_t rank, float pre_div,
                                              float post_div, float* grad_shard_acc, float* p_shard,
                                              float* exp_avg, float* exp_avg_sq, int64_t step, float lr,
                                              float beta1, float beta2, float eps, void* p_lp_out,
                                              void* hip_stream);
/* Without communication: the rank adds a micro-batch's unsharded gradient to
 * its own unsharded fp32 accumulator, grad_acc[k] = grad_acc[k] + grad_add[k]
 * for the P elements of the flat gradient (grad_add: fp32 or bf16), and
 * reduce-scatters once after the last micro-batch. */
int fsdp_grad_accumulate(const fsdp_layout_t* layout, float* grad_acc, const void* grad_add,
                         fsdp_dtype_t add_dtype, void* hip_stream);

/* ---- Sec. 4.4: the low-precision copy of the local shard, kept per rank -----
 * fsdp_cast_shard: lp_shard_out[k] = cast(shard[k]) (bf16 or fp16) for the S elements of
 * one fp32 shard (the one cast per FlatParameter that Sec. 4.4 places before the forward pass).
 * fsdp_reduce_scatter_adam_fused can also write it (p_lp_out) while the updated
 * shard is still in registers, which saves this pass in every later iteration.
 * fsdp_unshard_lp: the AllGather in the low precision, flat_out[w * S + k] =
 * lp_shard_w[k]; lp_shard_ptrs: host [W] of dev bf16 shards (S each); flat_out:
 * dev bf16 [P].  Together they give exactly fsdp_unshard(..., FSDP_BF16). */
int fsdp_cast_shard(const fsdp_layout_t* layout, const float* shard, void* lp_shard_out,
                    fsdp_dtype_t lp_dtype /* FSDP_BF16 or FSDP_F16 */, void* hip_stream);
int fsdp_unshard_lp(const fsdp_layout_t* layout, const void* const* lp_shard_ptrs, void* flat_out,
                    void* hip_stream);

/* ---- Sec. 4.4: FP16 training and the sharded gradient scaler ----------------
 * The loss is multiplied by `scale`, so gradients arrive scaled.  Each rank
 * sees only its shard of the reduced gradient, so the non-finite check must be
 * combined over all ranks before any rank steps (a local scaler would let some
 * ranks step and others skip).  All state lives on the device; nothing here
 * needs a host round trip.
 *
 * fsdp_reduce_scatter_unscale: fsdp_reduce_scatter_local, then for each element
 * of the result: if it is Inf or NaN, *found_inf = 1.0f (the flag is only ever
 * set, the caller clears it before the first unit); then it is multiplied by
 * inv_scale (= 1 / scale, finite, > 0) and stored.  found_inf: dev, one float.
 * fsdp_found_inf_combine: the all-reduce (max) of the ranks' flags:
 * found_inf_ptrs is a host array of num_ranks dev flags, each of which
 * receives the maximum (more than FSDP_MAX_RANKS_PER_LAUNCH flags take several launches).  (Simulated ranks may also simply share one flag.)
 * fsdp_shard_adam_step_guarded: fsdp_shard_adam_step that reads *found_inf on
 * the device and leaves p, m, v untouched when it is non-zero.
 * fsdp_grad_scaler_update: dynamic loss scaling on the device: *found_inf != 0
 * -> *scale *= backoff_factor, *growth_tracker = 0; otherwise the tracker is
 * incremented and, on reaching growth_interval, *scale *= growth_factor and the
 * tracker restarts.  Requires growth_factor > 1, 0 < backoff_factor < 1,
 * growth_interval >= 1. */
int fsdp_reduce_scatter_unscale(const fsdp_layout_t* layout, const void* const* grad_ptrs,
                                fsdp_dtype_t grad_dtype, int32_t rank, float pre_div, float post_div,
                                float inv_scale, float* grad_shard_out, float* found_inf,
                                void* hip_stream);
int fsdp_found_inf_combine(float* const* found_inf_ptrs, int32_t num_ranks, void* hip_stream);
int fsdp_shard_adam_step_guarded(const fsdp_layout_t* layout, float* p_shard, const float* g_shard,
                                 float* exp_avg, float* exp_avg_sq, int64_t step, float lr,
                                 float beta1, float beta2, float eps, const float* found_inf,
                                 void* hip_stream);
int fsdp_grad_scaler_update(float* scale, int32_t* growth_tracker, const float* found_inf,
                            float growth_factor, float backoff_factor, int32_t growth_interval,
                            void* hip_stream);

/* ---- batches of independent operations in few launches ----------------------
 * For units as small as a transformer block one kernel launch costs about as
 * much as a third of the data movement (an empty kernel takes ~3 us back to
 * back on MI355X), which is the paper's point about many small collectives
 * (Sec. 3.2.1).  A batch records fused reduce-scatter + Adam operations and
 * unshards that do NOT depend on each other (e.g. the updates of units i..i+2
 * and the prefetched unshards of units i+3..i+5, Sec. 3.3.2 / 3.3.3) and issues
 * them in as few grids as possible: up to 6 + 6 operations share one grid, their
 * rank pointers one pool of 376 (twelve 8-rank members fit, and so does one
 * 64-rank update next to one 64-rank unshard).
 * Results are bit-identical to issuing the operations one by one.  Operations
 * that cannot share a grid (W > 64, fp32 / fp16 unshard output, a second
 * operation of the same kind above 128 MiB, an update above 128 MiB next to an
 * unshard above 128 MiB unless the gradients are fp32 and the shard has fewer
 * than 8.4 M elements, different gradient dtype or divide mode) are issued
 * through their own kernels, in order, and so is an operation left alone in its
 * grid when the stand-alone kernel is the faster one (an unshard; an update
 * above 128 MiB).  The grids are planned and their kernel
 * arguments written while the batch is recorded; a launch only fills in the
 * Adam constants that depend on the step count.
 * The batch copies the pointer tables; layouts and device buffers must stay
 * valid while the batch is used.  A batch may be launched any number of times;
 * `step` is the Adam step count (after increment) of every update in it.  A
 * batch is not thread-safe while it is being modified; launching an unmodified
 * batch from several threads is. */
int  fsdp_batch_create(fsdp_batch_t** out);
void fsdp_batch_destroy(fsdp_batch_t* batch);                /* NULL is a no-op */
int  fsdp_batch_clear(fsdp_batch_t* batch);
int  fsdp_batch_add_unshard(fsdp_batch_t* batch, const fsdp_layout_t* layout,
                            const float* const* shard_ptrs, void* flat_out, fsdp_dtype_t out_dtype);
/* The Sec. 4.4 hand-off as a batch member: the gather of fsdp_unshard_lp (the
 * ranks' 16-bit shards, e.g. written by p_lp_out below, into the flat buffer). */
int  fsdp_batch_add_unshard_lp(fsdp_batch_t* batch, const fsdp_layout_t* layout,
                               const void* const* lp_shard_ptrs, void* flat_out);
int  fsdp_batch_add_reduce_scatter_adam(fsdp_batch_t* batch, const fsdp_layout_t* layout,
                                        const void* const* grad_ptrs, fsdp_dtype_t grad_dtype,
                                        int32_t rank, float pre_div, float post_div,
                                        float* grad_shard_out /* may be NULL */, float* p_shard,
                                        float* exp_avg, float* exp_avg_sq, float lr, float beta1,
                                        float beta2, float eps, void* p_lp_out /* may be NULL */);
int  fsdp_batch_launch(const fsdp_batch_t* batch, int64_t step, void* hip_stream);
/* How the recorded batch is issued (host only; for profiling and reports): the
 * number of kernel launches of one fsdp_batch_launch call and, for launch i,
 * which kernel it is (fsdp_kernel_name gives its name as profilers show it,
 * without template arguments), how many updates and unshards it carries and its
 * grid size in workgroups.  Any out pointer may be NULL. */
typedef enum {
    FSDP_KERNEL_BATCH = 0,        /* batch_kernel: several operations in one grid */
    FSDP_KERNEL_REDUCE = 1,       /* reduce_kernel: one reduce-scatter (+ Adam) */
    FSDP_KERNEL_UNSHARD_LP = 2,   /* unshard_lp_kernel: cast + gather to bf16 / fp16 */
    FSDP_KERNEL_UNSHARD_F32 = 3,  /* unshard_f32_kernel: fp32 gather */
    FSDP_KERNEL_GATHER_LP = 4,    /* gather_lp_kernel: gather of 16-bit shards */
    FSDP_KERNEL_UNSHARD_LP_LIGHT = 5  /* unshard_lp_light_kernel: the cast + gather in single-wave workgroups */
} fsdp_kernel_t;
int  fsdp_batch_launch_count(const fsdp_batch_t* batch, int32_t* count);
int  fsdp_batch_launch_info(const fsdp_batch_t* batch, int32_t i, int32_t* kernel, int32_t* n_updates,
                            int32_t* n_unshards, int64_t* workgroups);
const char* fsdp_kernel_name(int32_t kernel);     /* NULL for an unknown value */

/* Last hipError_t seen by this thread inside the library (0 if none). */
int fsdp_last_hip_error(void);
/* Static string for a fsdp_status_t. */
const char* fsdp_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* FSDP_FLAT_H */
