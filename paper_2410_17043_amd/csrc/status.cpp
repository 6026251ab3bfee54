// Status strings and the thread-local error detail.
#include "common.h"

static thread_local char g_err[512] = "";

int moe_set_error(int status, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return status;
}

extern "C" const char* moe_last_error(void) { return g_err; }

extern "C" const char* moe_status_str(int status) {
    switch (status) {
        case MOE_OK: return "MOE_OK";
        case MOE_EINVAL: return "MOE_EINVAL";
        case MOE_ESHAPE: return "MOE_ESHAPE";
        case MOE_EDTYPE: return "MOE_EDTYPE";
        case MOE_EALIGN: return "MOE_EALIGN";
        case MOE_ENOMEM: return "MOE_ENOMEM";
        case MOE_EHIP: return "MOE_EHIP";
        case MOE_EINTERNAL: return "MOE_EINTERNAL";
        default: return "MOE_UNKNOWN";
    }
}

int moe_check_shape(const moe_shape* s) {
    if (!s) return moe_set_error(MOE_EINVAL, "shape is NULL");
    if (s->T <= 0 || s->H <= 0 || s->E <= 0 || s->k <= 0 || s->G <= 0)
        return moe_set_error(MOE_EINVAL, "T, H, E, k, G must be positive");
    if (s->dtype != MOE_F32 && s->dtype != MOE_BF16) return moe_set_error(MOE_EDTYPE, "unknown dtype %d", s->dtype);
    if (s->k > s->E || s->k > MOE_MAX_K) return moe_set_error(MOE_ESHAPE, "k=%d must be <= min(E, %d)", s->k, MOE_MAX_K);
    if (s->E > MOE_MAX_E || s->G > MOE_MAX_G) return moe_set_error(MOE_ESHAPE, "E <= %d and G <= %d required", MOE_MAX_E, MOE_MAX_G);
    if ((int64_t)s->T * s->k >= (int64_t)1 << 31) return moe_set_error(MOE_ESHAPE, "T*k must be below 2^31");
    if (((int64_t)s->H * elem_size(s->dtype)) % 16 != 0) return moe_set_error(MOE_EALIGN, "row size H*elem must be a multiple of 16 bytes");
    if (s->capacity < 0 || (s->renorm != 0 && s->renorm != 1)) return moe_set_error(MOE_EINVAL, "capacity >= 0 and renorm in {0,1} required");
    return MOE_OK;
}

extern "C" int moe_ctx_create(moe_ctx** out, const moe_shape* shape) {
    if (!out) return moe_set_error(MOE_EINVAL, "out is NULL");
    *out = nullptr;
    int rc = moe_check_shape(shape);
    if (rc != MOE_OK) return rc;
    moe_ctx* c = new (std::nothrow) moe_ctx();
    if (!c) return moe_set_error(MOE_ENOMEM, "host allocation failed");
    c->s = *shape;
    c->n_slots = shape->T * shape->k;
    c->n_blocks = (c->n_slots + MOE_SLOTS_PER_BLOCK - 1) / MOE_SLOTS_PER_BLOCK;
    c->block_hist = nullptr;
    c->rank_src = nullptr;
    c->reuse_ranks = false;
    size_t bytes = ((size_t)c->n_blocks * shape->E + shape->E + (size_t)c->n_slots) * sizeof(int32_t);
    hipError_t e = hipMalloc((void**)&c->block_hist, bytes);
    if (e != hipSuccess) {
        delete c;
        return moe_set_error(e == hipErrorOutOfMemory ? MOE_ENOMEM : MOE_EHIP, "hipMalloc(%zu): %s", bytes, hipGetErrorString(e));
    }
    c->raw_count = c->block_hist + (size_t)c->n_blocks * shape->E;
    c->slot_rank = c->raw_count + shape->E;
    *out = c;
    return MOE_OK;
}

extern "C" int moe_ctx_invalidate(moe_ctx* ctx) {
    if (!ctx) return moe_set_error(MOE_EINVAL, "moe_ctx_invalidate: ctx is NULL");
    ctx->rank_src = nullptr;
    return MOE_OK;
}

extern "C" int moe_ctx_set_rank_reuse(moe_ctx* ctx, int32_t enable) {
    if (!ctx) return moe_set_error(MOE_EINVAL, "moe_ctx_set_rank_reuse: ctx is NULL");
    ctx->reuse_ranks = enable != 0;
    ctx->rank_src = nullptr;
    return MOE_OK;
}

extern "C" int moe_ctx_destroy(moe_ctx* ctx) {
    if (!ctx) return MOE_OK;
    hipError_t e = hipFree(ctx->block_hist);
    delete ctx;
    if (e != hipSuccess) return moe_set_error(MOE_EHIP, "hipFree: %s", hipGetErrorString(e));
    return MOE_OK;
}
