/*
 * CPU oracle for the per-rank FlatParameter data path of FSDP
 * (arXiv 2304.11277).  TEST INFRASTRUCTURE ONLY: nothing in the product path
 * may call, link or import this file.  It shares no code with the HIP
 * library; it is written from the paper's definitions, one plain loop per
 * definition, with no blocking, fusion or reordering.
 *
 * Build: gcc -O2 -std=c99 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 * (-ffp-contract=off: every binary32 operation below is one IEEE-754
 * round-to-nearest-even operation, never fused.)  The OpenMP pragmas split
 * loops over independent output elements only; the order of operations that
 * produce any one element is untouched.
 *
 * Parity pins (tests/test_oracle_*.py): every function here is pinned to
 * something other than itself; see each function's comment.
 *
 * Notation (Sec. 3.2.1): p parameters with numels n_i, off_i = sum_{j<i} n_j,
 * N = off_p, sharding factor F = W (full sharding), S = ceil(N / W),
 * P = S * W, pad = P - N.
 */
#include <stdint.h>
#include <string.h>
#include <math.h>

/* ---------------------------------------------------------------- layout */

/* Sec. 3.2.1, flatten-concat-chunk: the FlatParameter is the concatenation of
 * the p flattened parameters, padded on the right to a size divisible by the
 * sharding factor, then cut into W equal chunks.  An empty dims list is a
 * scalar (numel 1); a zero dim gives numel 0.
 * Pins: the paper's worked example (Fig. 3: a 4x3 Linear on 16 ranks gives one
 * element per rank and the last rank holds the pad); pad <= W - 1 (Sec. 3.2.1).
 * Returns 0, or -1 on a non-positive W / p or a negative dim. */
int orc_layout(const int64_t *dims, const int32_t *ndims, int32_t p, int32_t W,
               int64_t *off /* p+1 */, int64_t *S_out, int64_t *P_out, int64_t *pad_out)
{
    if (p <= 0 || W <= 0) return -1;
    int64_t d = 0, acc = 0;
    for (int32_t i = 0; i < p; ++i) {
        int64_t n = 1;
        for (int32_t k = 0; k < ndims[i]; ++k) {
            if (dims[d] < 0) return -1;
            n *= dims[d++];
        }
        off[i] = acc;
        acc += n;
    }
    off[p] = acc;
    int64_t N = acc;
    int64_t S = (N + W - 1) / W;
    *S_out = S;
    *P_out = S * W;
    *pad_out = S * W - N;
    return 0;
}

/* Sec. 3.2.1: flat = concat_i(flatten(param_i)) in the given order, then
 * pad zeros (+0.0f) on the right up to P elements.
 * Pin: equals numpy.concatenate + zero fill; views recover every parameter. */
void orc_flatten_pad(const float *const *params, const int64_t *numel, int32_t p,
                     int64_t P, float *flat)
{
    int64_t pos = 0;
    for (int32_t i = 0; i < p; ++i) {
        for (int64_t k = 0; k < numel[i]; ++k) flat[pos + k] = params[i][k];
        pos += numel[i];
    }
    for (int64_t k = pos; k < P; ++k) flat[k] = 0.0f;
}

/* Sec. 3.2.1: rank w's chunk is flat[w*S, (w+1)*S). */
void orc_chunk(const float *flat, int64_t S, int32_t w, float *shard)
{
    for (int64_t k = 0; k < S; ++k) shard[k] = flat[(int64_t)w * S + k];
}

/* ------------------------------------------------------------------ cast */

/* Sec. 4.4 (native mixed precision): full-to-low precision cast of the local
 * shard.  The paper names BF16 as a common low precision and fixes no rounding
 * mode; this build's reading is IEEE round-to-nearest, ties-to-even, on the
 * upper 16 bits of the binary32 pattern.  NaN keeps its sign and top payload
 * bits and is forced quiet.  Denormals are rounded, not flushed.  Integer
 * arithmetic only, so no FPU mode can change it.
 * Pins: hand vectors (ties, overflow to Inf, denormal tie), torch's CPU
 * float32->bfloat16 conversion over every non-NaN bit pattern, and a
 * nearest-neighbour search in exact arithmetic. */
uint16_t orc_bf16_rne(uint32_t u)
{
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu) != 0u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    return (uint16_t)((u + 0x7FFFu + lsb) >> 16);
}

void orc_cast_bf16(const float *x, int64_t n, uint16_t *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < n; ++k) {
        uint32_t u;
        memcpy(&u, &x[k], 4);
        y[k] = orc_bf16_rne(u);
    }
}

/* exhaustive helper for the pin tests: casts the bit patterns [first, first+count) */
void orc_cast_bf16_bits(uint32_t first, int64_t count, uint16_t *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < count; ++k) y[k] = orc_bf16_rne(first + (uint32_t)k);
}

/* --------------------------------------------------------------- unshard */

/* Sec. 3 / 3.2.1 (AllGather with even inputs into one output tensor) with
 * Sec. 4.4 (each rank casts its local shard, the collective runs in the low
 * precision): flat_lp[w*S + k] = bf16(shard_w[k]).  The pad is gathered too.
 * Pin: concat of shards == flat buffer; views of the gathered buffer equal the
 * cast of the original parameters. */
void orc_unshard_bf16(const float *const *shards, int32_t W, int64_t S, uint16_t *flat_lp)
{
    for (int32_t w = 0; w < W; ++w)
        orc_cast_bf16(shards[w], S, flat_lp + (int64_t)w * S);
}

/* Full-precision unshard: the same gather without the cast. */
void orc_unshard_f32(const float *const *shards, int32_t W, int64_t S, float *flat)
{
    for (int32_t w = 0; w < W; ++w) {
        const float *s = shards[w];
        float *d = flat + (int64_t)w * S;
#pragma omp parallel for schedule(static)
        for (int64_t k = 0; k < S; ++k) d[k] = s[k];
    }
}

/* Low-precision gather: when every rank keeps the bf16 cast of its own shard
 * (Sec. 4.4: one full-to-low cast per FlatParameter, collectives in the low
 * precision), the unshard is the plain AllGather of those bf16 shards:
 * flat_lp[w*S + k] = lp_shard_w[k].
 * Pins: numpy.concatenate; equals orc_unshard_bf16 of the fp32 shards when
 * lp_shard_w = cast(shard_w). */
void orc_gather_lp(const uint16_t *const *lp_shards, int32_t W, int64_t S, uint16_t *flat_lp)
{
    for (int32_t w = 0; w < W; ++w)
        for (int64_t k = 0; k < S; ++k) flat_lp[(int64_t)w * S + k] = lp_shards[w][k];
}

/* -------------------------------------------------------- reduce-scatter */

static inline float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* Sec. 3 and Sec. 3.2.2 eq. (1): the reduced gradient is the sum over ranks of
 * the rank gradients; ReduceScatter leaves rank r with chunk r of that sum.
 * The paper writes a plain sum; the data-parallel mean is obtained by dividing
 * by factors pre and post with pre * post = W (this build's reading, both are
 * explicit arguments).  The order is fixed: ranks 0, 1, ..., W-1, one binary32
 * division and one binary32 addition per rank, the accumulator initialised from
 * rank 0's term (not from +0, so a -0 survives).
 * slices[w] points at element r*S of rank w's unsharded gradient buffer.
 * Pins: exact-rational re-evaluation with explicit rounding on tiny inputs,
 * integer-valued gradients (exact mean), identical ranks, an order witness. */
void orc_reduce_slices_f32(const float *const *slices, int32_t W, int64_t S,
                           float pre, float post, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < S; ++k) {
        float acc = slices[0][k] / pre;
        for (int32_t w = 1; w < W; ++w) acc = acc + slices[w][k] / pre;
        out[k] = acc / post;
    }
}

/* Same with bf16 gradient buffers: the upcast to binary32 is exact, all
 * arithmetic and the output are binary32 (Sec. 4.4: the reduction precision is
 * chosen independently of the parameter precision). */
void orc_reduce_slices_bf16(const uint16_t *const *slices, int32_t W, int64_t S,
                            float pre, float post, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < S; ++k) {
        float acc = bf16_to_f32(slices[0][k]) / pre;
        for (int32_t w = 1; w < W; ++w) acc = acc + bf16_to_f32(slices[w][k]) / pre;
        out[k] = acc / post;
    }
}

/* Reduce-scatter from the full unsharded buffers (P elements each). */
void orc_reduce_scatter_f32(const float *const *gradbufs, int32_t W, int64_t S, int32_t r,
                            float pre, float post, float *out)
{
    const float *sl[W];
    for (int32_t w = 0; w < W; ++w) sl[w] = gradbufs[w] + (int64_t)r * S;
    orc_reduce_slices_f32(sl, W, S, pre, post, out);
}

void orc_reduce_scatter_bf16(const uint16_t *const *gradbufs, int32_t W, int64_t S, int32_t r,
                             float pre, float post, float *out)
{
    const uint16_t *sl[W];
    for (int32_t w = 0; w < W; ++w) sl[w] = gradbufs[w] + (int64_t)r * S;
    orc_reduce_slices_bf16(sl, W, S, pre, post, out);
}

/* The definition "reduce, then scatter" taken literally: the whole reduced
 * buffer of P elements (an all-reduce), from which rank r's result is the
 * slice [r*S, (r+1)*S).  Used to check the sliced form above. */
void orc_reduce_full_f32(const float *const *gradbufs, int32_t W, int64_t P,
                         float pre, float post, float *full)
{
    orc_reduce_slices_f32(gradbufs, W, P, pre, post, full);
}

/* ------------------------------------------------------ hybrid sharding */

/* Sec. 3.2.2: with sharding factor F < W the W ranks form G = W / F sharded
 * groups S_1..S_G; gradients are reduce-scattered inside each sharded group and
 * the sharded results are then all-reduced across the groups (the replicate
 * group of this rank's position).  Eq. (1): sum_r g_r = sum_i sum_{r in S_i} g_r.
 * In real arithmetic the two agree; in binary32 the two-level order is its own
 * result, fixed here as: inner sums over the F ranks of a group in local-rank
 * order (terms divided by pre first, accumulator started from the group's
 * first term), outer sum over the groups in group order (accumulator started
 * from group 0's inner sum), then one division by post; pre * post = W.
 * slices[i*F + l] points at this rank position's slice (S elements) of the
 * gradient buffer of local rank l in group i.
 * Pins: integer gradients (exact, equals the flat sum), exact-rational model,
 * a witness where the two-level and the flat order differ, G = 1 equals the
 * flat reduce-scatter bit for bit. */
void orc_reduce_slices_hybrid_f32(const float *const *slices, int32_t G, int32_t F, int64_t S,
                                  float pre, float post, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < S; ++k) {
        float outer = 0.0f;
        for (int32_t i = 0; i < G; ++i) {
            float inner = slices[(int64_t)i * F][k] / pre;
            for (int32_t l = 1; l < F; ++l) inner = inner + slices[(int64_t)i * F + l][k] / pre;
            outer = (i == 0) ? inner : outer + inner;
        }
        out[k] = outer / post;
    }
}

void orc_reduce_slices_hybrid_bf16(const uint16_t *const *slices, int32_t G, int32_t F, int64_t S,
                                   float pre, float post, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < S; ++k) {
        float outer = 0.0f;
        for (int32_t i = 0; i < G; ++i) {
            float inner = bf16_to_f32(slices[(int64_t)i * F][k]) / pre;
            for (int32_t l = 1; l < F; ++l) inner = inner + bf16_to_f32(slices[(int64_t)i * F + l][k]) / pre;
            outer = (i == 0) ? inner : outer + inner;
        }
        out[k] = outer / post;
    }
}

/* ------------------------------------------------ gradient accumulation */

/* Sec. 3.3.4.  With communication: every micro-batch is reduce-scattered and
 * the rank keeps adding the sharded result to its sharded gradient
 * (acc[k] = acc[k] + new[k], S elements).  Without communication: the rank
 * adds its own unsharded gradients locally (same operation on P elements) and
 * reduce-scatters once at the end.  One binary32 addition per element, the
 * running sum on the left.
 * Pins: numpy's float32 addition (a library routine), integer exactness, and
 * the two variations agreeing exactly on integer-valued gradients. */
void orc_accumulate_f32(float *acc, const float *add, int64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < n; ++k) acc[k] = acc[k] + add[k];
}

/* bf16 micro-batch gradients accumulated into a binary32 buffer (exact upcast). */
void orc_accumulate_bf16(float *acc, const uint16_t *add, int64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < n; ++k) acc[k] = acc[k] + bf16_to_f32(add[k]);
}

/* ------------------------------------------- fp16 and the gradient scaler */

/* Sec. 4.4 names FP16 as the other common low precision.  binary32 -> binary16,
 * round to nearest even, written from the two formats' definitions: overflow
 * goes to Inf, results below the smallest normal half are rounded onto the
 * subnormal grid (quantum 2^-24), NaN keeps sign and the top ten payload bits
 * and is made quiet.
 * Pins: numpy's float32 -> float16 conversion over every non-NaN pattern, hand
 * vectors, exact nearest-neighbour search. */
uint16_t orc_f16_rne(uint32_t u)
{
    uint32_t sign = (u >> 16) & 0x8000u;
    uint32_t exp = (u >> 23) & 0xFFu;
    uint32_t man = u & 0x007FFFFFu;
    if (exp == 0xFFu) {
        if (man == 0) return (uint16_t)(sign | 0x7C00u);
        return (uint16_t)(sign | 0x7C00u | 0x0200u | (man >> 13));
    }
    if (exp == 0) return (uint16_t)sign;                 /* binary32 zero / subnormal: far below 2^-25 */
    int32_t e = (int32_t)exp - 127;
    if (e > 15) return (uint16_t)(sign | 0x7C00u);
    if (e >= -14) {
        uint32_t h = ((uint32_t)(e + 15) << 10) | (man >> 13);
        uint32_t rem = man & 0x1FFFu;
        if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) h += 1;   /* a carry walks into the exponent, up to Inf */
        return (uint16_t)(sign | h);
    }
    uint32_t m = man | 0x00800000u;                      /* 1.man as a 24-bit integer, value m * 2^(e-23) */
    int32_t shift = -1 - e;                              /* to units of 2^-24 */
    if (shift > 31) return (uint16_t)sign;
    uint32_t h = m >> shift;
    uint32_t rem = m & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (h & 1u))) h += 1;
    return (uint16_t)(sign | h);
}

void orc_cast_f16(const float *x, int64_t n, uint16_t *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < n; ++k) {
        uint32_t u;
        memcpy(&u, &x[k], 4);
        y[k] = orc_f16_rne(u);
    }
}

void orc_cast_f16_bits(uint32_t first, int64_t count, uint16_t *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < count; ++k) y[k] = orc_f16_rne(first + (uint32_t)k);
}

/* binary16 -> binary32, exact (every half is representable).
 * Pin: numpy's float16 -> float32 over all 65536 patterns. */
static inline float f16_to_f32(uint16_t h)
{
    uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
    uint32_t exp = (h >> 10) & 0x1Fu;
    uint32_t man = h & 0x03FFu;
    uint32_t u;
    if (exp == 0x1Fu) {
        u = sign | 0x7F800000u | (man << 13);
    } else if (exp != 0) {
        u = sign | ((exp + 112u) << 23) | (man << 13);
    } else if (man == 0) {
        u = sign;
    } else {                                              /* subnormal half: man * 2^-24, normalise */
        int32_t e = -1;
        do { man <<= 1; ++e; } while ((man & 0x0400u) == 0);
        u = sign | ((uint32_t)(112 - e) << 23) | ((man & 0x03FFu) << 13);
    }
    float f;
    memcpy(&f, &u, 4);
    return f;
}

void orc_upcast_f16(const uint16_t *h, int64_t n, float *y)
{
    for (int64_t k = 0; k < n; ++k) y[k] = f16_to_f32(h[k]);
}

void orc_unshard_f16(const float *const *shards, int32_t W, int64_t S, uint16_t *flat_lp)
{
    for (int32_t w = 0; w < W; ++w)
        orc_cast_f16(shards[w], S, flat_lp + (int64_t)w * S);
}

void orc_reduce_slices_f16(const uint16_t *const *slices, int32_t W, int64_t S,
                           float pre, float post, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < S; ++k) {
        float acc = f16_to_f32(slices[0][k]) / pre;
        for (int32_t w = 1; w < W; ++w) acc = acc + f16_to_f32(slices[w][k]) / pre;
        out[k] = acc / post;
    }
}

/* Sec. 4.4, sharded gradient scaler.  The loss is multiplied by `scale`, so the
 * reduced gradient shard is multiplied by inv_scale = 1/scale (one binary32
 * multiplication per element) and checked: found_inf is 1 when any element of
 * the reduced shard is Inf or NaN (the check looks at the value before the
 * multiplication, as the gradient scaler the paper cites does).  Each rank sees
 * only its shard, so the flags of all ranks are combined (a max) before any
 * rank decides to step; a scaler that looked at the local shard only would let
 * some ranks step and others skip.  Returns this shard's flag.
 * Pins: torch's non-finite-check-and-unscale routine on the CPU; the combined
 * flag equals the flag of the whole unsharded gradient. */
float orc_unscale_check(float *g, int64_t n, float inv_scale)
{
    float found = 0.0f;
    for (int64_t k = 0; k < n; ++k) {
        if (isinf(g[k]) || isnan(g[k])) found = 1.0f;
        g[k] = g[k] * inv_scale;
    }
    return found;
}

/* combine of the per-rank flags: every rank ends up with the maximum */
float orc_found_inf_combine(const float *flags, int32_t W)
{
    float m = 0.0f;
    for (int32_t w = 0; w < W; ++w)
        if (flags[w] > m) m = flags[w];
    return m;
}

/* Scale update of dynamic loss scaling (the gradient scaler the paper cites):
 * after a step with a non-finite gradient the scale is multiplied by backoff
 * and the streak of good steps restarts; after growth_interval good steps in a
 * row it is multiplied by growth.
 * Pin: torch's scale-update routine on the CPU, over a random flag sequence. */
void orc_scaler_update(float *scale, int32_t *growth_tracker, float found_inf,
                       float growth, float backoff, int32_t growth_interval)
{
    if (found_inf != 0.0f) {
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

/* ------------------------------------------------------------------ Adam */

/* Sec. 5.4 names Adam with its two optimizer states per parameter, kept
 * sharded (Sec. 3); the paper prints no update rule.  This build's reading is
 * the original Adam of Kingma & Ba with bias correction, eps added to the
 * bias-corrected sqrt(v) outside the root, no weight decay, no amsgrad.
 * t >= 1 is the step count after increment.  bc1 = 1 - beta1^t and
 * bc2 = 1 - beta2^t are evaluated in binary64 and rounded to binary32; every
 * per-element operation is one binary32 operation in the order written.
 * Pins: closed form at t = 1 from zero state (step = -lr * g / (|g| + eps)),
 * zero gradient leaves p unchanged, torch.optim.Adam in binary64 over several
 * steps, the binary64 evaluation below. */
void orc_adam_f32(float *p, const float *g, float *m, float *v, int64_t S, int64_t t,
                  float lr, float beta1, float beta2, float eps)
{
    float bc1 = (float)(1.0 - pow((double)beta1, (double)t));
    float bc2 = (float)(1.0 - pow((double)beta2, (double)t));
    float one_m_b1 = 1.0f - beta1;
    float one_m_b2 = 1.0f - beta2;
    float step_size = lr / bc1;
    float sqrt_bc2 = sqrtf(bc2);
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < S; ++k) {
        float gk = g[k];
        float mk = beta1 * m[k] + one_m_b1 * gk;
        float vk = beta2 * v[k] + one_m_b2 * gk * gk;
        float denom = sqrtf(vk) / sqrt_bc2 + eps;
        p[k] = p[k] - step_size * (mk / denom);
        m[k] = mk;
        v[k] = vk;
    }
}

/* The same update evaluated in binary64 from the binary32 inputs (hyper-
 * parameters widened from their binary32 values); a second witness so that
 * neither evaluation order is privileged in the tolerance test. */
void orc_adam_f64(const float *p, const float *g, const float *m, const float *v, int64_t S,
                  int64_t t, float lr, float beta1, float beta2, float eps,
                  double *p_out, double *m_out, double *v_out)
{
    double b1 = beta1, b2 = beta2;
    double bc1 = 1.0 - pow(b1, (double)t);
    double bc2 = 1.0 - pow(b2, (double)t);
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < S; ++k) {
        double gk = g[k];
        double mk = b1 * (double)m[k] + (1.0 - b1) * gk;
        double vk = b2 * (double)v[k] + (1.0 - b2) * gk * gk;
        double denom = sqrt(vk) / sqrt(bc2) + (double)eps;
        p_out[k] = (double)p[k] - ((double)lr / bc1) * (mk / denom);
        m_out[k] = mk;
        v_out[k] = vk;
    }
}

/* number of threads the parallel loops use (reported with timings) */
#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
void orc_set_num_threads(int n) { omp_set_num_threads(n); }
#else
int orc_num_threads(void) { return 1; }
void orc_set_num_threads(int n) { (void)n; }
#endif
