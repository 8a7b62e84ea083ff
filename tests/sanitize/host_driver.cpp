// Host-code sanitizer driver (test infrastructure).  Built by
// tests/test_host_sanitizers.py with AddressSanitizer and
// UndefinedBehaviorSanitizer, together with (a) the CPU oracle and (b) the host
// side of libfsdp_flat: the layout planner, every entry point's argument
// validation and the batch object's bookkeeping.  No kernel is launched: every
// compute call below is one that must be rejected on the host, so the driver
// runs without a GPU.  All buffers are heap blocks of exactly the documented
// size, so that an overrun on either side is reported.
//
// Prints "ALL OK" and exits 0 when every check passed.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "fsdp_flat.h"

extern "C" {
int orc_layout(const int64_t*, const int32_t*, int32_t, int32_t, int64_t*, int64_t*, int64_t*, int64_t*);
void orc_flatten_pad(const float* const*, const int64_t*, int32_t, int64_t, float*);
void orc_chunk(const float*, int64_t, int32_t, float*);
void orc_cast_bf16(const float*, int64_t, uint16_t*);
void orc_cast_bf16_bits(uint32_t, int64_t, uint16_t*);
void orc_unshard_bf16(const float* const*, int32_t, int64_t, uint16_t*);
void orc_unshard_f32(const float* const*, int32_t, int64_t, float*);
void orc_gather_lp(const uint16_t* const*, int32_t, int64_t, uint16_t*);
void orc_reduce_slices_f32(const float* const*, int32_t, int64_t, float, float, float*);
void orc_reduce_slices_bf16(const uint16_t* const*, int32_t, int64_t, float, float, float*);
void orc_reduce_scatter_f32(const float* const*, int32_t, int64_t, int32_t, float, float, float*);
void orc_reduce_scatter_bf16(const uint16_t* const*, int32_t, int64_t, int32_t, float, float, float*);
void orc_reduce_full_f32(const float* const*, int32_t, int64_t, float, float, float*);
void orc_reduce_slices_hybrid_f32(const float* const*, int32_t, int32_t, int64_t, float, float, float*);
void orc_reduce_slices_hybrid_bf16(const uint16_t* const*, int32_t, int32_t, int64_t, float, float, float*);
void orc_accumulate_f32(float*, const float*, int64_t);
void orc_accumulate_bf16(float*, const uint16_t*, int64_t);
void orc_cast_f16(const float*, int64_t, uint16_t*);
void orc_cast_f16_bits(uint32_t, int64_t, uint16_t*);
void orc_upcast_f16(const uint16_t*, int64_t, float*);
void orc_unshard_f16(const float* const*, int32_t, int64_t, uint16_t*);
void orc_reduce_slices_f16(const uint16_t* const*, int32_t, int64_t, float, float, float*);
float orc_unscale_check(float*, int64_t, float);
float orc_found_inf_combine(const float*, int32_t);
void orc_scaler_update(float*, int32_t*, float, float, float, int32_t);
void orc_adam_f32(float*, const float*, float*, float*, int64_t, int64_t, float, float, float, float);
void orc_adam_f64(const float*, const float*, const float*, const float*, int64_t, int64_t, float, float, float,
                  float, double*, double*, double*);
}

static int g_fail = 0;
#define CHECK(cond)                                                             \
    do {                                                                        \
        if (!(cond)) {                                                          \
            std::printf("CHECK failed at line %d: %s\n", __LINE__, #cond);      \
            ++g_fail;                                                           \
        }                                                                       \
    } while (0)

static uint32_t g_rng = 12345u;
static uint32_t rnd() { g_rng = g_rng * 1664525u + 1013904223u; return g_rng >> 8; }
static float rndf() { return (static_cast<int>(rnd() % 2001) - 1000) * 1e-3f; }

// a fake, suitably aligned "device" pointer: validated by the library, never dereferenced on the host
static void* fake(uintptr_t i) { return reinterpret_cast<void*>(0x10000000ull + 0x1000ull * i); }

static void planner_checks()
{
    // agreement with the oracle's layout on random ragged shape lists
    for (int it = 0; it < 300; ++it) {
        const int32_t p = 1 + rnd() % 9, W = 1 + rnd() % 70;
        std::vector<int64_t> dims;
        std::vector<int32_t> nd(p);
        for (int32_t i = 0; i < p; ++i) {
            nd[i] = rnd() % 4;
            for (int32_t k = 0; k < nd[i]; ++k) dims.push_back(rnd() % 7 == 0 ? 0 : 1 + rnd() % 9);
        }
        std::vector<int64_t> off(p + 1);
        int64_t S = 0, P = 0, pad = 0;
        CHECK(orc_layout(dims.data(), nd.data(), p, W, off.data(), &S, &P, &pad) == 0);
        fsdp_layout_t* L = nullptr;
        const int rc = fsdp_layout_init(dims.empty() ? nullptr : dims.data(), nd.data(), p, W, &L);
        if (off[p] == 0) {
            CHECK(rc == FSDP_ERR_INVALID_ARG && L == nullptr);
            continue;
        }
        CHECK(rc == FSDP_OK && L != nullptr);
        if (!L) continue;
        int64_t N2, P2, S2, pad2;
        int32_t p2, W2;
        CHECK(fsdp_layout_info(L, &N2, &P2, &S2, &pad2, &p2, &W2) == FSDP_OK);
        CHECK(N2 == off[p] && P2 == P && S2 == S && pad2 == pad && p2 == p && W2 == W);
        CHECK(pad2 >= 0 && pad2 < W);
        for (int32_t i = 0; i < p; ++i) {
            int64_t o, n;
            CHECK(fsdp_layout_param(L, i, &o, &n) == FSDP_OK);
            CHECK(o == off[i] && n == off[i + 1] - off[i]);
            void* v = nullptr;
            CHECK(fsdp_view_ptr(L, fake(1), FSDP_BF16, i, &v) == FSDP_OK);
            CHECK(v == static_cast<char*>(fake(1)) + 2 * off[i]);
        }
        CHECK(fsdp_layout_param(L, p, nullptr, nullptr) == FSDP_ERR_RANK_RANGE);
        CHECK(fsdp_layout_param(L, -1, nullptr, nullptr) == FSDP_ERR_RANK_RANGE);
        fsdp_layout_destroy(L);
    }
    // error paths
    fsdp_layout_t* L = nullptr;
    int64_t d2[2] = {4, 3};
    int32_t n1[1] = {2};
    CHECK(fsdp_layout_init(d2, n1, 1, 4, nullptr) == FSDP_ERR_NULL_PTR);
    CHECK(fsdp_layout_init(d2, nullptr, 1, 4, &L) == FSDP_ERR_NULL_PTR);
    CHECK(fsdp_layout_init(nullptr, n1, 1, 4, &L) == FSDP_ERR_NULL_PTR);
    CHECK(fsdp_layout_init(d2, n1, 0, 4, &L) == FSDP_ERR_INVALID_ARG);
    CHECK(fsdp_layout_init(d2, n1, 1, 0, &L) == FSDP_ERR_INVALID_ARG);
    int64_t neg[2] = {4, -3};
    CHECK(fsdp_layout_init(neg, n1, 1, 4, &L) == FSDP_ERR_INVALID_ARG);
    int32_t nneg[1] = {-1};
    CHECK(fsdp_layout_init(d2, nneg, 1, 4, &L) == FSDP_ERR_INVALID_ARG);
    int64_t big[2] = {INT64_C(1) << 40, INT64_C(1) << 40};
    CHECK(fsdp_layout_init(big, n1, 1, 4, &L) == FSDP_ERR_OVERFLOW);
    int64_t big1[1] = {INT64_MAX / 4};
    int32_t one[1] = {1};
    CHECK(fsdp_layout_init(big1, one, 1, 3, &L) == FSDP_ERR_OVERFLOW);
    int64_t bigz[3] = {INT64_C(1) << 40, 0, INT64_C(1) << 40};   // a zero dim wins over the overflow
    int32_t n3[2] = {3, 1};
    int64_t bigz2[4] = {bigz[0], bigz[1], bigz[2], 5};
    CHECK(fsdp_layout_init(bigz2, n3, 2, 2, &L) == FSDP_OK);
    fsdp_layout_destroy(L);
    fsdp_layout_destroy(nullptr);
    CHECK(fsdp_layout_info(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == FSDP_ERR_NULL_PTR);
    for (int32_t W = 1; W <= 300; ++W) {
        float pre = 0, post = 0;
        CHECK(fsdp_default_divide_factors(W, &pre, &post) == FSDP_OK);
        CHECK(pre >= 1.0f && post >= 1.0f && pre * post == static_cast<float>(W));
    }
    float x;
    CHECK(fsdp_default_divide_factors(0, &x, &x) == FSDP_ERR_INVALID_ARG);
    CHECK(fsdp_default_divide_factors(8, nullptr, &x) == FSDP_ERR_NULL_PTR);
    CHECK(std::strcmp(fsdp_status_string(FSDP_ERR_BAD_DTYPE), "bad dtype") == 0);
    CHECK(fsdp_status_string(-99) != nullptr);
    {
        const int64_t d1[1] = {5};
        const int32_t n1[1] = {1};
        fsdp_layout_t* lw = nullptr;
        CHECK(fsdp_layout_init_ex(d1, n1, 1, 2, 9, &lw) == FSDP_ERR_INVALID_ARG && lw == nullptr);
        CHECK(fsdp_layout_init_ex(d1, n1, 1, 2, FSDP_WALK_DEEP, &lw) == FSDP_OK && lw != nullptr);
        fsdp_layout_destroy(lw);
    }
}

// every compute entry point with arguments it must reject before any launch
static void validation_checks()
{
    for (int32_t W : {1, 3, 8, 64, 65, 130}) {
        int64_t dims[1] = {1000 + W};
        int32_t nd[1] = {1};
        fsdp_layout_t* L = nullptr;
        CHECK(fsdp_layout_init(dims, nd, 1, W, &L) == FSDP_OK);
        std::vector<const void*> tab(W), bad(W);
        for (int32_t w = 0; w < W; ++w) tab[w] = bad[w] = fake(10 + w);
        bad[W - 1] = nullptr;
        std::vector<const void*> odd(tab);
        odd[0] = static_cast<const char*>(fake(5)) + 1;      // misaligned for every dtype
        auto ftab = reinterpret_cast<const float* const*>(tab.data());
        auto fbad = reinterpret_cast<const float* const*>(bad.data());
        auto fodd = reinterpret_cast<const float* const*>(odd.data());
        float* out = static_cast<float*>(fake(1));
        float *p = static_cast<float*>(fake(2)), *m = static_cast<float*>(fake(3)), *v = static_cast<float*>(fake(4));

        std::vector<float*> mtab(W), mbad(W);
        for (int32_t w = 0; w < W; ++w) mtab[w] = mbad[w] = static_cast<float*>(fake(10 + w));
        mbad[W - 1] = nullptr;
        const void* params[1] = {fake(6)};
        const void* nullparams[1] = {nullptr};
        CHECK(fsdp_flatten_shard(L, nullparams, mtab.data(), nullptr) == FSDP_ERR_NULL_PTR);
        CHECK(fsdp_flatten_shard(L, params, mbad.data(), nullptr) == FSDP_ERR_NULL_PTR);
        CHECK(fsdp_flatten_shard(nullptr, params, mtab.data(), nullptr) == FSDP_ERR_NULL_PTR);

        CHECK(fsdp_unshard(L, fbad, out, FSDP_BF16, nullptr) == FSDP_ERR_NULL_PTR);
        CHECK(fsdp_unshard(L, ftab, nullptr, FSDP_BF16, nullptr) == FSDP_ERR_NULL_PTR);
        CHECK(fsdp_unshard(L, ftab, out, static_cast<fsdp_dtype_t>(7), nullptr) == FSDP_ERR_BAD_DTYPE);
        CHECK(fsdp_unshard(L, fodd, out, FSDP_BF16, nullptr) == FSDP_ERR_INVALID_ARG);

        CHECK(fsdp_reduce_scatter_local(L, bad.data(), FSDP_F32, 0, 1.0f, 1.0f, out, nullptr) == FSDP_ERR_NULL_PTR);
        CHECK(fsdp_reduce_scatter_local(L, tab.data(), FSDP_F32, W, 1.0f, 1.0f, out, nullptr) == FSDP_ERR_RANK_RANGE);
        CHECK(fsdp_reduce_scatter_local(L, tab.data(), FSDP_F32, -1, 1.0f, 1.0f, out, nullptr) == FSDP_ERR_RANK_RANGE);
        CHECK(fsdp_reduce_scatter_local(L, tab.data(), FSDP_F32, 0, 0.0f, 1.0f, out, nullptr) == FSDP_ERR_INVALID_ARG);
        CHECK(fsdp_reduce_scatter_local(L, tab.data(), FSDP_F32, 0, 1.0f, -2.0f, out, nullptr) == FSDP_ERR_INVALID_ARG);
        CHECK(fsdp_reduce_scatter_local(L, tab.data(), static_cast<fsdp_dtype_t>(-1), 0, 1.0f, 1.0f, out, nullptr) ==
              FSDP_ERR_BAD_DTYPE);
        CHECK(fsdp_reduce_scatter_local(L, tab.data(), FSDP_F32, 0, 1.0f, 1.0f, nullptr, nullptr) == FSDP_ERR_NULL_PTR);
        CHECK(fsdp_reduce_scatter_local(L, odd.data(), FSDP_BF16, 0, 1.0f, 1.0f, out, nullptr) == FSDP_ERR_INVALID_ARG);

        CHECK(fsdp_shard_adam_step(L, p, out, m, v, 0, 1e-3f, 0.9f, 0.999f, 1e-8f, nullptr) == FSDP_ERR_INVALID_ARG);
        CHECK(fsdp_shard_adam_step(L, p, out, m, v, 1, 1e-3f, 1.0f, 0.999f, 1e-8f, nullptr) == FSDP_ERR_INVALID_ARG);
        CHECK(fsdp_shard_adam_step(L, p, out, m, v, 1, 1e-3f, 0.9f, -0.1f, 1e-8f, nullptr) == FSDP_ERR_INVALID_ARG);
        CHECK(fsdp_shard_adam_step(L, p, out, m, v, 1, 1e-3f, 0.9f, 0.999f, -1.0f, nullptr) == FSDP_ERR_INVALID_ARG);
        CHECK(fsdp_shard_adam_step(L, p, nullptr, m, v, 1, 1e-3f, 0.9f, 0.999f, 1e-8f, nullptr) == FSDP_ERR_NULL_PTR);

        CHECK(fsdp_reduce_scatter_adam_fused(L, bad.data(), FSDP_F32, 0, 1.0f, 1.0f, out, p, m, v, 1, 1e-3f, 0.9f, 0.999f,
                                             1e-8f, nullptr, nullptr) == FSDP_ERR_NULL_PTR);
        CHECK(fsdp_reduce_scatter_adam_fused(L, tab.data(), FSDP_F32, 0, 1.0f, 1.0f, out, p, m, v, 0, 1e-3f, 0.9f, 0.999f,
                                             1e-8f, nullptr, nullptr) == FSDP_ERR_INVALID_ARG);
        if (W > FSDP_MAX_RANKS_PER_LAUNCH) {
            // split launches carry the partial sum in the gradient shard: it may not be omitted
            CHECK(fsdp_reduce_scatter_adam_fused(L, tab.data(), FSDP_F32, 0, 1.0f, 1.0f, nullptr, p, m, v, 1, 1e-3f, 0.9f,
                                                 0.999f, 1e-8f, nullptr, nullptr) == FSDP_ERR_NULL_PTR);
            CHECK(fsdp_reduce_scatter_accumulate(L, tab.data(), FSDP_F32, 0, 1.0f, 1.0f, out, nullptr) ==
                  FSDP_ERR_INVALID_ARG);
        }
        CHECK(fsdp_reduce_scatter_hybrid(L, tab.data(), FSDP_F32, 0, 0, 1.0f, 1.0f, out, nullptr) == FSDP_ERR_INVALID_ARG);
        CHECK(fsdp_reduce_scatter_hybrid_adam_fused(L, tab.data(), FSDP_F32, 0, 0, 1.0f, 1.0f, out, p, m, v, 1, 1e-3f, 0.9f,
                                                    0.999f, 1e-8f, nullptr, nullptr) == FSDP_ERR_INVALID_ARG);
        CHECK(fsdp_reduce_scatter_hybrid_adam_fused(L, tab.data(), FSDP_F32, 1, 0, 1.0f, 1.0f, out, p, nullptr, v, 1, 1e-3f,
                                                    0.9f, 0.999f, 1e-8f, nullptr, nullptr) == FSDP_ERR_NULL_PTR);
        CHECK(fsdp_reduce_scatter_accumulate_adam_fused(L, tab.data(), FSDP_F32, 0, 1.0f, 1.0f, nullptr, p, m, v, 1, 1e-3f,
                                                        0.9f, 0.999f, 1e-8f, nullptr, nullptr) == FSDP_ERR_NULL_PTR);
        CHECK(fsdp_reduce_scatter_accumulate_adam_fused(L, tab.data(), FSDP_F32, 0, 1.0f, 1.0f, out, p, m, v, 0, 1e-3f, 0.9f,
                                                        0.999f, 1e-8f, nullptr, nullptr) == FSDP_ERR_INVALID_ARG);
        CHECK(fsdp_reduce_scatter_accumulate(L, bad.data(), FSDP_F32, 0, 1.0f, 1.0f, out, nullptr) == FSDP_ERR_NULL_PTR);
        CHECK(fsdp_grad_accumulate(L, nullptr, fake(9), FSDP_F32, nullptr) == FSDP_ERR_NULL_PTR);
        CHECK(fsdp_grad_accumulate(L, out, fake(9), static_cast<fsdp_dtype_t>(3), nullptr) == FSDP_ERR_BAD_DTYPE);
        CHECK(fsdp_cast_shard(L, nullptr, fake(9), FSDP_BF16, nullptr) == FSDP_ERR_NULL_PTR);
        CHECK(fsdp_cast_shard(L, out, fake(9), FSDP_F32, nullptr) == FSDP_ERR_BAD_DTYPE);
        CHECK(fsdp_unshard_lp(L, bad.data(), out, nullptr) == FSDP_ERR_NULL_PTR);
        CHECK(fsdp_reduce_scatter_unscale(L, tab.data(), FSDP_F16, 0, 1.0f, 1.0f, 1.0f, out, nullptr, nullptr) ==
              FSDP_ERR_NULL_PTR);
        CHECK(fsdp_found_inf_combine(nullptr, 4, nullptr) == FSDP_ERR_NULL_PTR);
        CHECK(fsdp_shard_adam_step_guarded(L, p, out, m, v, 1, 1e-3f, 0.9f, 0.999f, 1e-8f, nullptr, nullptr) ==
              FSDP_ERR_NULL_PTR);
        CHECK(fsdp_grad_scaler_update(nullptr, reinterpret_cast<int32_t*>(fake(7)), out, 2.0f, 0.5f, 100, nullptr) ==
              FSDP_ERR_NULL_PTR);

        // the batch object: record, grow, clear, record again, reject, destroy
        fsdp_batch_t* b = nullptr;
        CHECK(fsdp_batch_create(&b) == FSDP_OK && b != nullptr);
        for (int rep = 0; rep < 3; ++rep) {
            for (int i = 0; i < 40; ++i) {
                CHECK(fsdp_batch_add_unshard(b, L, ftab, fake(100 + i), FSDP_BF16) == FSDP_OK);
                CHECK(fsdp_batch_add_reduce_scatter_adam(b, L, tab.data(), i % 2 ? FSDP_BF16 : FSDP_F32, i % W, 1.0f,
                                                         static_cast<float>(W), i % 3 ? out : nullptr, p, m, v, 1e-3f,
                                                         0.9f, 0.999f, 1e-8f, nullptr) ==
                      ((i % 3 == 0 && W > FSDP_MAX_RANKS_PER_LAUNCH) ? FSDP_ERR_NULL_PTR : FSDP_OK));
            }
            CHECK(fsdp_batch_add_unshard_lp(b, L, tab.data(), fake(300)) == FSDP_OK);
            CHECK(fsdp_batch_add_unshard_lp(b, L, bad.data(), out) == FSDP_ERR_NULL_PTR);
            CHECK(fsdp_batch_add_unshard_lp(b, L, odd.data(), out) == FSDP_ERR_INVALID_ARG);
            CHECK(fsdp_batch_add_unshard_lp(b, L, tab.data(), nullptr) == FSDP_ERR_NULL_PTR);
            CHECK(fsdp_batch_add_unshard(b, L, fbad, out, FSDP_BF16) == FSDP_ERR_NULL_PTR);
            CHECK(fsdp_batch_add_unshard(b, L, ftab, out, static_cast<fsdp_dtype_t>(9)) == FSDP_ERR_BAD_DTYPE);
            CHECK(fsdp_batch_add_reduce_scatter_adam(b, L, tab.data(), FSDP_F32, W, 1.0f, 1.0f, out, p, m, v, 1e-3f, 0.9f,
                                                     0.999f, 1e-8f, nullptr) == FSDP_ERR_RANK_RANGE);
            CHECK(fsdp_batch_add_reduce_scatter_adam(b, L, tab.data(), FSDP_F32, 0, 1.0f, 1.0f, out, p, m, v, 1e-3f, 1.5f,
                                                     0.999f, 1e-8f, nullptr) == FSDP_ERR_INVALID_ARG);
            CHECK(fsdp_batch_launch(b, 0, nullptr) == FSDP_ERR_INVALID_ARG);
            // the recorded plan, read back launch by launch
            int32_t n_launches = -1;
            CHECK(fsdp_batch_launch_count(b, &n_launches) == FSDP_OK && n_launches > 0);
            for (int32_t i = 0; i < n_launches; ++i) {
                int32_t kernel = -1, nu = -1, ns = -1;
                int64_t wgs = -1;
                CHECK(fsdp_batch_launch_info(b, i, &kernel, &nu, &ns, &wgs) == FSDP_OK);
                CHECK(fsdp_kernel_name(kernel) != nullptr && nu >= 0 && ns >= 0 && nu + ns >= 1 && wgs >= 1);
                CHECK(fsdp_batch_launch_info(b, i, nullptr, nullptr, nullptr, nullptr) == FSDP_OK);
            }
            CHECK(fsdp_batch_launch_info(b, n_launches, nullptr, nullptr, nullptr, nullptr) == FSDP_ERR_RANK_RANGE);
            CHECK(fsdp_batch_launch_info(b, -1, nullptr, nullptr, nullptr, nullptr) == FSDP_ERR_RANK_RANGE);
            CHECK(fsdp_batch_launch_count(b, nullptr) == FSDP_ERR_NULL_PTR);
            CHECK(fsdp_batch_clear(b) == FSDP_OK);
            CHECK(fsdp_batch_launch_count(b, &n_launches) == FSDP_OK && n_launches == 0);
        }
        CHECK(fsdp_kernel_name(-1) == nullptr && fsdp_kernel_name(FSDP_KERNEL_GATHER_LP) != nullptr);
        CHECK(fsdp_batch_launch(b, 1, nullptr) == FSDP_OK);        // an empty batch launches nothing
        CHECK(fsdp_batch_launch(nullptr, 1, nullptr) == FSDP_ERR_NULL_PTR);
        CHECK(fsdp_batch_clear(nullptr) == FSDP_ERR_NULL_PTR);
        fsdp_batch_destroy(b);
        fsdp_batch_destroy(nullptr);
        fsdp_layout_destroy(L);
    }
}

template <class T>
static std::vector<const T*> ptrs(const std::vector<std::vector<T>>& v)
{
    std::vector<const T*> r;
    for (const auto& x : v) r.push_back(x.data());
    return r;
}

// the oracle on exactly sized heap buffers
static void oracle_checks()
{
    for (int32_t W : {1, 2, 3, 5, 8, 12}) {
        for (int64_t S : {int64_t{1}, int64_t{7}, int64_t{64}, int64_t{1001}}) {
            const int64_t P = S * W;
            // ragged parameters adding up to N in (P - W, P]
            const int64_t N = P - (W > 1 ? static_cast<int64_t>(rnd() % W) : 0);
            std::vector<std::vector<float>> params;
            std::vector<int64_t> numel;
            for (int64_t left = N; left > 0;) {
                const int64_t n = 1 + static_cast<int64_t>(rnd()) % left;
                params.emplace_back(n);
                for (auto& x : params.back()) x = rndf();
                numel.push_back(n);
                left -= n;
                if (rnd() % 4 == 0) { params.emplace_back(0); numel.push_back(0); }
            }
            std::vector<float> flat(P, 7.0f);
            auto pp = ptrs(params);
            orc_flatten_pad(pp.data(), numel.data(), static_cast<int32_t>(numel.size()), P, flat.data());
            for (int64_t k = N; k < P; ++k) CHECK(flat[k] == 0.0f);
            std::vector<std::vector<float>> shards(W, std::vector<float>(S));
            for (int32_t w = 0; w < W; ++w) orc_chunk(flat.data(), S, w, shards[w].data());
            auto sp = ptrs(shards);
            std::vector<uint16_t> lp(P), lp16(P), lp2(P);
            std::vector<float> f32(P), up(P);
            orc_unshard_bf16(sp.data(), W, S, lp.data());
            orc_unshard_f16(sp.data(), W, S, lp16.data());
            orc_unshard_f32(sp.data(), W, S, f32.data());
            CHECK(std::memcmp(f32.data(), flat.data(), P * 4) == 0);
            orc_cast_bf16(flat.data(), P, lp2.data());
            CHECK(std::memcmp(lp.data(), lp2.data(), P * 2) == 0);
            orc_cast_f16(flat.data(), P, lp2.data());
            CHECK(std::memcmp(lp16.data(), lp2.data(), P * 2) == 0);
            orc_upcast_f16(lp16.data(), P, up.data());
            std::vector<std::vector<uint16_t>> lps(W, std::vector<uint16_t>(S));
            for (int32_t w = 0; w < W; ++w) orc_cast_bf16(shards[w].data(), S, lps[w].data());
            auto lpp = ptrs(lps);
            orc_gather_lp(lpp.data(), W, S, lp2.data());
            CHECK(std::memcmp(lp.data(), lp2.data(), P * 2) == 0);

            // gradients of W ranks (P elements each), fp32 / bf16 / fp16
            std::vector<std::vector<float>> g(W, std::vector<float>(P));
            std::vector<std::vector<uint16_t>> gb(W, std::vector<uint16_t>(P)), gh(W, std::vector<uint16_t>(P));
            for (int32_t w = 0; w < W; ++w) {
                for (auto& x : g[w]) x = rndf();
                orc_cast_bf16(g[w].data(), P, gb[w].data());
                orc_cast_f16(g[w].data(), P, gh[w].data());
            }
            auto gp = ptrs(g);
            auto gbp = ptrs(gb);
            auto ghp = ptrs(gh);
            std::vector<float> full(P), out(S), acc(S, 0.0f), accP(P, 0.0f);
            const float pre = 2.0f, post = W / 2.0f;
            orc_reduce_full_f32(gp.data(), W, P, pre, post, full.data());
            for (int32_t r = 0; r < W; ++r) {
                orc_reduce_scatter_f32(gp.data(), W, S, r, pre, post, out.data());
                CHECK(std::memcmp(out.data(), full.data() + r * S, S * 4) == 0);
                orc_reduce_scatter_bf16(gbp.data(), W, S, r, pre, post, out.data());
                std::vector<const uint16_t*> sl(W);
                for (int32_t w = 0; w < W; ++w) sl[w] = gh[w].data() + r * S;
                orc_reduce_slices_f16(sl.data(), W, S, pre, post, out.data());
                for (int32_t w = 0; w < W; ++w) sl[w] = gb[w].data() + r * S;
                orc_reduce_slices_bf16(sl.data(), W, S, pre, post, out.data());
                orc_accumulate_f32(acc.data(), out.data(), S);
            }
            orc_accumulate_f32(accP.data(), g[0].data(), P);
            orc_accumulate_bf16(accP.data(), gb[W - 1].data(), P);
            for (int32_t G = 1; G <= W; ++G) {
                if (W % G) continue;
                const int32_t F = W / G;
                std::vector<const float*> sl(W);
                std::vector<const uint16_t*> slb(W);
                for (int32_t w = 0; w < W; ++w) { sl[w] = g[w].data(); slb[w] = gb[w].data(); }
                orc_reduce_slices_hybrid_f32(sl.data(), G, F, S, pre, post, out.data());
                orc_reduce_slices_hybrid_bf16(slb.data(), G, F, S, pre, post, out.data());
            }
            const float fi = orc_unscale_check(out.data(), S, 1.0f / 1024.0f);
            CHECK(fi == 0.0f);
            std::vector<float> flags(W, 0.0f);
            flags[W - 1] = 1.0f;
            CHECK(orc_found_inf_combine(flags.data(), W) == 1.0f);

            std::vector<float> pS(shards[0]), mS(S, 0.0f), vS(S, 0.0f);
            std::vector<double> dp(S), dm(S), dv(S);
            orc_adam_f64(pS.data(), out.data(), mS.data(), vS.data(), S, 1, 1e-3f, 0.9f, 0.999f, 1e-8f, dp.data(),
                         dm.data(), dv.data());
            orc_adam_f32(pS.data(), out.data(), mS.data(), vS.data(), S, 1, 1e-3f, 0.9f, 0.999f, 1e-8f);
            orc_adam_f32(pS.data(), out.data(), mS.data(), vS.data(), S, 2, 1e-3f, 0.9f, 0.999f, 1e-8f);
            for (int64_t k = 0; k < S; ++k) CHECK(pS[k] == pS[k]);
        }
    }
    std::vector<uint16_t> y(4096);
    orc_cast_bf16_bits(0x7F7FF000u, 4096, y.data());
    orc_cast_f16_bits(0x477FE000u, 4096, y.data());
    orc_cast_bf16_bits(0xFFFFF000u, 4096, y.data());     // wraps through the NaN range to +0
    float scale = 65536.0f;
    int32_t tracker = 0;
    for (int i = 0; i < 10; ++i) orc_scaler_update(&scale, &tracker, i == 4 ? 1.0f : 0.0f, 2.0f, 0.5f, 3);
    CHECK(scale > 0.0f);
}

int main()
{
    planner_checks();
    std::printf("planner done\n");
    validation_checks();
    std::printf("validation done\n");
    oracle_checks();
    std::printf("oracle done\n");
    if (g_fail) {
        std::printf("%d checks failed\n", g_fail);
        return 1;
    }
    std::printf("ALL OK\n");
    return 0;
}
