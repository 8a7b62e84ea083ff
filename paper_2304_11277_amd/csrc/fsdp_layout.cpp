// Host planner of libfsdp_flat: the flatten-concat-pad-chunk layout of one FSDP
// unit's FlatParameter (Sec. 3.2.1) and the zero-copy parameter views
// (Sec. 3.2.3).  No device is touched in this file.
#include <cmath>
#include <cstdint>
#include <limits>
#include <new>

#include "fsdp_internal.h"

namespace {
thread_local int g_last_hip_error = 0;

bool mul_overflow(int64_t a, int64_t b, int64_t* out) { return __builtin_mul_overflow(a, b, out); }
bool add_overflow(int64_t a, int64_t b, int64_t* out) { return __builtin_add_overflow(a, b, out); }
}  // namespace

namespace fsdp {
void set_last_hip_error(int e) { g_last_hip_error = e; }
}  // namespace fsdp

extern "C" {

int fsdp_last_hip_error(void) { return g_last_hip_error; }

const char* fsdp_status_string(int status)
{
    switch (status) {
        case FSDP_OK: return "ok";
        case FSDP_ERR_INVALID_ARG: return "invalid argument";
        case FSDP_ERR_NULL_PTR: return "null pointer";
        case FSDP_ERR_OVERFLOW: return "size overflows int64";
        case FSDP_ERR_OOM: return "host allocation failed";
        case FSDP_ERR_BAD_DTYPE: return "bad dtype";
        case FSDP_ERR_RANK_RANGE: return "rank or parameter index out of range";
        case FSDP_ERR_HIP: return "HIP launch error";
        default: return "unknown status";
    }
}

// Sec. 3.2.1: concatenate p flattened parameters, pad on the right to a
// multiple of the sharding factor, cut into W equal chunks.
int fsdp_layout_init(const int64_t* dims, const int32_t* ndims, int32_t num_params,
                     int32_t world_size, fsdp_layout_t** out)
{
    return fsdp_layout_init_ex(dims, ndims, num_params, world_size, FSDP_WALK_AUTO, out);
}

int fsdp_layout_init_ex(const int64_t* dims, const int32_t* ndims, int32_t num_params,
                        int32_t world_size, int32_t reduce_walk, fsdp_layout_t** out)
{
    if (!out) return FSDP_ERR_NULL_PTR;
    *out = nullptr;
    if (!ndims) return FSDP_ERR_NULL_PTR;
    if (num_params <= 0 || world_size <= 0) return FSDP_ERR_INVALID_ARG;
    if (reduce_walk != FSDP_WALK_AUTO && reduce_walk != FSDP_WALK_WIDE && reduce_walk != FSDP_WALK_DEEP &&
        reduce_walk != FSDP_WALK_HALF)
        return FSDP_ERR_INVALID_ARG;

    fsdp_layout* L = new (std::nothrow) fsdp_layout;
    if (!L) return FSDP_ERR_OOM;
    int rc = FSDP_OK;
    try {
        L->off.resize(static_cast<size_t>(num_params) + 1);
        L->numel.resize(static_cast<size_t>(num_params));
    } catch (const std::bad_alloc&) {
        delete L;
        return FSDP_ERR_OOM;
    }
    int64_t d = 0, acc = 0;
    for (int32_t i = 0; i < num_params && rc == FSDP_OK; ++i) {
        if (ndims[i] < 0) { rc = FSDP_ERR_INVALID_ARG; break; }
        if (ndims[i] > 0 && !dims) { rc = FSDP_ERR_NULL_PTR; break; }
        int64_t n = 1;
        bool zero = false;
        // A zero dim makes the numel 0 whatever the other dims are; look for it
        // first so that it cannot be reported as an overflow.
        for (int32_t k = 0; k < ndims[i]; ++k) {
            if (dims[d + k] < 0) { rc = FSDP_ERR_INVALID_ARG; break; }
            if (dims[d + k] == 0) zero = true;
        }
        if (rc != FSDP_OK) break;
        for (int32_t k = 0; k < ndims[i]; ++k) {
            if (zero) { n = 0; break; }
            if (mul_overflow(n, dims[d + k], &n)) { rc = FSDP_ERR_OVERFLOW; break; }
        }
        if (rc != FSDP_OK) break;
        d += ndims[i];
        L->off[i] = acc;
        L->numel[i] = n;
        if (add_overflow(acc, n, &acc)) { rc = FSDP_ERR_OVERFLOW; break; }
    }
    if (rc == FSDP_OK) {
        L->off[num_params] = acc;
        if (acc == 0) rc = FSDP_ERR_INVALID_ARG;      // nothing to shard
    }
    if (rc == FSDP_OK) {
        const int64_t W = world_size;
        int64_t tmp, P, bytes;
        // S = ceil(N / W) without forming N + W - 1 past int64
        int64_t S = acc / W + (acc % W != 0 ? 1 : 0);
        if (mul_overflow(S, W, &P) || mul_overflow(P, int64_t{4}, &bytes) ||
            add_overflow(bytes, int64_t{64}, &tmp)) {
            rc = FSDP_ERR_OVERFLOW;
        } else {
            L->num_params = num_params;
            L->world_size = world_size;
            L->N = acc;
            L->S = S;
            L->P = P;
            L->pad = P - acc;
            L->reduce_walk = reduce_walk;
        }
    }
    if (rc != FSDP_OK) {
        delete L;
        return rc;
    }
    *out = L;
    return FSDP_OK;
}

void fsdp_layout_destroy(fsdp_layout_t* layout) { delete layout; }

int fsdp_layout_info(const fsdp_layout_t* L, int64_t* numel, int64_t* padded, int64_t* shard,
                     int64_t* pad, int32_t* num_params, int32_t* world_size)
{
    if (!L) return FSDP_ERR_NULL_PTR;
    if (numel) *numel = L->N;
    if (padded) *padded = L->P;
    if (shard) *shard = L->S;
    if (pad) *pad = L->pad;
    if (num_params) *num_params = L->num_params;
    if (world_size) *world_size = L->world_size;
    return FSDP_OK;
}

int fsdp_layout_param(const fsdp_layout_t* L, int32_t i, int64_t* offset, int64_t* numel)
{
    if (!L) return FSDP_ERR_NULL_PTR;
    if (i < 0 || i >= L->num_params) return FSDP_ERR_RANK_RANGE;
    if (offset) *offset = L->off[i];
    if (numel) *numel = L->numel[i];
    return FSDP_OK;
}

// Sec. 3.2.3: parameter i is the view flat[off_i, off_i + n_i) of the unsharded
// FlatParameter; only an address is computed.
int fsdp_view_ptr(const fsdp_layout_t* L, void* flat_base, fsdp_dtype_t dtype, int32_t i, void** out)
{
    if (!L || !flat_base || !out) return FSDP_ERR_NULL_PTR;
    if (dtype != FSDP_F32 && dtype != FSDP_BF16 && dtype != FSDP_F16) return FSDP_ERR_BAD_DTYPE;
    if (i < 0 || i >= L->num_params) return FSDP_ERR_RANK_RANGE;
    const int64_t esize = dtype == FSDP_F32 ? 4 : 2;
    *out = static_cast<char*>(flat_base) + L->off[i] * esize;
    return FSDP_OK;
}

int fsdp_default_divide_factors(int32_t world_size, float* pre, float* post)
{
    if (!pre || !post) return FSDP_ERR_NULL_PTR;
    if (world_size <= 0) return FSDP_ERR_INVALID_ARG;
    const int64_t W = world_size;
    int64_t f = 1;
    while (W % (f * 2) == 0 && f * f < W) f *= 2;
    *pre = static_cast<float>(f);
    *post = static_cast<float>(W / f);
    return FSDP_OK;
}

}  // extern "C"
