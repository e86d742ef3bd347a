// C-ABI entry points of libals: argument validation, context and workspace management, and the
// epoch / loss glue.  All arithmetic of the method lives in the kernel translation units.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "als_internal.h"

namespace als {

static thread_local char static_error[256] = "";  // message of the last failed context-free call of this thread

als_status fail(als_ctx *ctx, als_status st, const std::string &msg) {
    if (ctx) ctx->last_error = msg;
    else snprintf(static_error, sizeof(static_error), "%s", msg.c_str());
    return st;
}

als_status ensure(als_ctx *ctx, DevBuf &b, size_t bytes) {
    if (bytes <= b.bytes) return ALS_OK;
    if (b.p) {
        ALS_HIP(ctx, hipFree(b.p));  // hipFree waits for work that may still use the old buffer
        b.p = nullptr;
        b.bytes = 0;
    }
    size_t want = bytes + bytes / 8 + 256;
    hipError_t e = hipMalloc(&b.p, want);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        b.p = nullptr;
        return fail(ctx, ALS_ENOMEM, "workspace allocation of " + std::to_string(want) + " bytes failed");
    }
    b.bytes = want;
    return ALS_OK;
}

void timer_begin(als_ctx *ctx, int slot, hipStream_t s) {
    if (!ctx->timing) return;
    Timer t;
    if (!ctx->free_timers.empty()) {
        t = ctx->free_timers.back();
        ctx->free_timers.pop_back();
    } else {
        if (hipEventCreate(&t.e0) != hipSuccess || hipEventCreate(&t.e1) != hipSuccess) return;
    }
    t.slot = slot;
    (void)hipEventRecord(t.e0, s);
    ctx->timers.push_back(t);
}

void timer_end(als_ctx *ctx, hipStream_t s) {
    if (!ctx->timing || ctx->timers.empty()) return;
    (void)hipEventRecord(ctx->timers.back().e1, s);
}

static void timers_reset(als_ctx *ctx) {
    for (auto &t : ctx->timers) ctx->free_timers.push_back(t);
    ctx->timers.clear();
    for (double &v : ctx->timing_ms) v = 0.0;
}

static bool d_supported(int d) { return d == 16 || d == 32 || d == 64 || d == 128; }

static als_status check_table(als_ctx *ctx, const als_table *t, const char *name) {
    if (!t) return fail(ctx, ALS_EINVAL, std::string(name) + " is null");
    if (!d_supported(t->d)) return fail(ctx, ALS_EDTYPE, std::string(name) + ": d must be 16, 32, 64 or 128");
    if (t->dtype != ALS_F32 && t->dtype != ALS_BF16) return fail(ctx, ALS_EDTYPE, std::string(name) + ": unknown dtype");
    if (t->rows < 0) return fail(ctx, ALS_EINVAL, std::string(name) + ": negative row count");
    if (t->ld < t->d) return fail(ctx, ALS_ESHAPE, std::string(name) + ": ld < d");
    if (t->ld > INT32_MAX) return fail(ctx, ALS_ESHAPE, std::string(name) + ": ld does not fit 31 bits");
    size_t es = t->dtype == ALS_F32 ? 4 : 2;
    if ((t->ld * es) % 16 != 0 || ((uintptr_t)t->data % 16) != 0)
        return fail(ctx, ALS_ESHAPE, std::string(name) + ": rows must be 16-byte aligned");
    if (t->rows > 0 && !t->data) return fail(ctx, ALS_EINVAL, std::string(name) + ": data is null");
    return ALS_OK;
}

static als_status check_csr_args(als_ctx *ctx, const als_csr *y, const char *name) {
    if (!y) return fail(ctx, ALS_EINVAL, std::string(name) + " is null");
    if (y->rows < 0 || y->cols < 0 || y->nnz < 0) return fail(ctx, ALS_EINVAL, std::string(name) + ": negative size");
    if (y->cols > INT32_MAX) return fail(ctx, ALS_ESHAPE, std::string(name) + ": cols exceeds int32 column ids");
    if (!y->indptr) return fail(ctx, ALS_EINVAL, std::string(name) + ": indptr is null");
    if (y->nnz > 0 && !y->indices) return fail(ctx, ALS_EINVAL, std::string(name) + ": indices is null");
    return ALS_OK;
}

static als_status check_params(als_ctx *ctx, const als_params *p) {
    if (!p) return fail(ctx, ALS_EINVAL, "params is null");
    if (!(p->alpha >= 0.0f)) return fail(ctx, ALS_EINVAL, "alpha must be >= 0");
    if (!(p->lambda > 0.0f)) return fail(ctx, ALS_ENOTSPD, "lambda must be > 0");
    if (p->path < 0 || p->path > 2) return fail(ctx, ALS_EINVAL, "unknown path");
    if (p->dual_max_k < 0 || p->dual_max_k > 128) return fail(ctx, ALS_EINVAL, "dual_max_k must be in [0, 128]");
    if (p->split_nnz < 0) return fail(ctx, ALS_EINVAL, "split_nnz must be >= 0");
    if (p->solver < 0 || p->solver > 2) return fail(ctx, ALS_EINVAL, "unknown solver");
    if (p->cg_max_iters < 0 || !(p->cg_tol >= 0.0f)) return fail(ctx, ALS_EINVAL, "bad CG parameters");
    return ALS_OK;
}

static bool overlaps(const als_table *a, const als_table *b) {
    if (a->rows == 0 || b->rows == 0) return false;
    auto span = [](const als_table *t) {
        size_t es = t->dtype == ALS_F32 ? 4 : 2;
        return (size_t)((t->rows - 1) * t->ld + t->d) * es;
    };
    uintptr_t a0 = (uintptr_t)a->data, a1 = a0 + span(a);
    uintptr_t b0 = (uintptr_t)b->data, b1 = b0 + span(b);
    return a0 < b1 && b0 < a1;
}

static als_status check_solve_args(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                                   const als_params *prm, const als_table *X, int64_t r0, int64_t r1) {
    als_status st;
    if ((st = check_csr_args(ctx, Y, "Y")) != ALS_OK) return st;
    if ((st = check_table(ctx, V, "V")) != ALS_OK) return st;
    if ((st = check_table(ctx, X, "X")) != ALS_OK) return st;
    if ((st = check_params(ctx, prm)) != ALS_OK) return st;
    if (!G) return fail(ctx, ALS_EINVAL, "G is null");
    if (V->d != X->d) return fail(ctx, ALS_ESHAPE, "V and X differ in d");
    if (V->dtype != X->dtype) return fail(ctx, ALS_EDTYPE, "V and X differ in dtype");
    if (Y->cols != V->rows) return fail(ctx, ALS_ESHAPE, "Y->cols != V->rows");
    if (Y->rows != X->rows) return fail(ctx, ALS_ESHAPE, "Y->rows != X->rows");
    if (r0 < 0 || r1 < r0 || r1 > Y->rows) return fail(ctx, ALS_EINVAL, "row range outside [0, rows]");
    if (overlaps(V, X)) return fail(ctx, ALS_EALIAS, "X overlaps V");
    return ALS_OK;
}

}  // namespace als

using namespace als;

extern "C" {

als_status als_create(als_ctx **out, int device) {
    if (!out) return ALS_EINVAL;
    *out = nullptr;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) {
        (void)hipGetLastError();
        return ALS_EHIP;
    }
    if (hipSetDevice(device) != hipSuccess) return ALS_EHIP;
    als_ctx *ctx = new (std::nothrow) als_ctx();
    if (!ctx) return ALS_ENOMEM;
    ctx->device = device;
    (void)gramian_static_setup(device);  // address of this GPU's static workspace, for als_gramian_static
    als_status st = ensure(ctx, ctx->small, SM_BYTES);
    if (st == ALS_OK) st = ensure(ctx, ctx->gram_w, 128 * 128 * sizeof(float));
    if (st == ALS_OK) st = ensure(ctx, ctx->gram_h, 128 * 128 * sizeof(float));
    if (st == ALS_OK && hipHostMalloc((void **)&ctx->host_counters, 16 * sizeof(int32_t)) != hipSuccess) st = ALS_ENOMEM;
    if (st == ALS_OK && hipHostMalloc((void **)&ctx->host_scalar, 2 * sizeof(double)) != hipSuccess) st = ALS_ENOMEM;
    if (st == ALS_OK && hipMemset(ctx->small.p, 0, ctx->small.bytes) != hipSuccess) st = ALS_EHIP;
    if (st == ALS_OK && hipHostMalloc((void **)&ctx->hint_counts, N_HINTS * HINT_INTS * sizeof(int32_t),
                                      hipHostMallocMapped) != hipSuccess)
        st = ALS_ENOMEM;
    if (st == ALS_OK) memset(ctx->hint_counts, 0, N_HINTS * HINT_INTS * sizeof(int32_t));
    if (st == ALS_OK && hipHostGetDevicePointer((void **)&ctx->hint_counts_dev, ctx->hint_counts, 0) != hipSuccess)
        st = ALS_EHIP;
    hipDeviceProp_t prop;
    if (st == ALS_OK && hipGetDeviceProperties(&prop, device) == hipSuccess && prop.multiProcessorCount > 0)
        ctx->num_cu = prop.multiProcessorCount;
    if (st != ALS_OK) {
        als_destroy(ctx);
        return st;
    }
    *out = ctx;
    return ALS_OK;
}

als_status als_destroy(als_ctx *ctx) {
    if (!ctx) return ALS_OK;
    (void)hipSetDevice(ctx->device);
    (void)hipDeviceSynchronize();
    DevBuf *bufs[] = {&ctx->gram_partials, &ctx->lists, &ctx->seg_partials, &ctx->ztable, &ctx->rtable, &ctx->small,
                      &ctx->loss_partials, &ctx->topk_partials, &ctx->gram_w, &ctx->gram_h};
    for (DevBuf *b : bufs)
        if (b->p) (void)hipFree(b->p);
    if (ctx->hint_counts) (void)hipHostFree(ctx->hint_counts);
    if (ctx->host_counters) (void)hipHostFree(ctx->host_counters);
    if (ctx->host_scalar) (void)hipHostFree(ctx->host_scalar);
    for (auto &t : ctx->timers) { (void)hipEventDestroy(t.e0); (void)hipEventDestroy(t.e1); }
    for (auto &t : ctx->free_timers) { (void)hipEventDestroy(t.e0); (void)hipEventDestroy(t.e1); }
    delete ctx;
    return ALS_OK;
}

als_status als_gramian(als_ctx *ctx, const als_table *V, float *G, void *stream) {
    if (!ctx) return ALS_EINVAL;
    als_status st = check_table(ctx, V, "V");
    if (st != ALS_OK) return st;
    if (!G) return fail(ctx, ALS_EINVAL, "G is null");
    timers_reset(ctx);
    return launch_gramian(ctx, V, G, (hipStream_t)stream);
}

als_status als_gramian_static(int device, const als_table *V, float *G, void *stream) {
    int ndev = 0, cur = -1;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev || hipGetDevice(&cur) != hipSuccess) {
        (void)hipGetLastError();
        return fail(nullptr, ALS_EHIP, "als_gramian_static: no such device");
    }
    if (cur != device) return fail(nullptr, ALS_EINVAL, "als_gramian_static: `device` must be the calling thread's current device");
    als_status st = check_table(nullptr, V, "V");
    if (st != ALS_OK) return st;
    if (!G) return fail(nullptr, ALS_EINVAL, "G is null");
    if (V->rows > ALS_GRAMIAN_STATIC_MAX_ROWS)
        return fail(nullptr, ALS_ESHAPE, "als_gramian_static: V has " + std::to_string(V->rows) + " rows, the static workspace holds the partial sums of at most " +
                                             std::to_string((long long)ALS_GRAMIAN_STATIC_MAX_ROWS) + " (use als_gramian)");
    st = launch_gramian_static(device, V, G, (hipStream_t)stream);
    if (st != ALS_OK) return fail(nullptr, st, "als_gramian_static: launch failed");
    return ALS_OK;
}

const char *als_static_last_error(void) { return static_error; }

als_status als_solve_rows(als_ctx *ctx, const als_csr *Y, const als_table *V, const float *G,
                          const als_params *prm, als_table *X, int64_t r0, int64_t r1, void *stream) {
    if (!ctx) return ALS_EINVAL;
    als_status st = check_solve_args(ctx, Y, V, G, prm, X, r0, r1);
    if (st != ALS_OK) return st;
    timers_reset(ctx);
    if (r1 == r0) return ALS_OK;
    return launch_solve_rows(ctx, Y, V, G, prm, X, r0, r1, (hipStream_t)stream);
}

als_status als_epoch(als_ctx *ctx, const als_csr *Y, const als_csr *Yt, als_table *W, als_table *H,
                     const als_params *prm, void *stream) {
    if (!ctx) return ALS_EINVAL;
    float *GH = (float *)ctx->gram_h.p, *GW = (float *)ctx->gram_w.p;
    // validate both halves before anything is launched, so an error leaves W and H untouched
    als_status st = check_solve_args(ctx, Y, H, GH, prm, W, 0, Y ? Y->rows : 0);
    if (st != ALS_OK) return st;
    st = check_solve_args(ctx, Yt, W, GW, prm, H, 0, Yt ? Yt->rows : 0);
    if (st != ALS_OK) return st;
    if (Yt->rows != Y->cols || Yt->cols != Y->rows || Yt->nnz != Y->nnz)
        return fail(ctx, ALS_ESHAPE, "Yt is not shaped as the transpose of Y");
    timers_reset(ctx);
    hipStream_t s = (hipStream_t)stream;
    if ((st = launch_gramian(ctx, H, GH, s)) != ALS_OK) return st;
    if (Y->rows > 0 && (st = launch_solve_rows(ctx, Y, H, GH, prm, W, 0, Y->rows, s)) != ALS_OK) return st;
    if ((st = launch_gramian(ctx, W, GW, s)) != ALS_OK) return st;
    if (Yt->rows > 0 && (st = launch_solve_rows(ctx, Yt, W, GW, prm, H, 0, Yt->rows, s)) != ALS_OK) return st;
    return ALS_OK;
}

als_status als_status_sync(als_ctx *ctx, void *stream) {
    if (!ctx) return ALS_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    int32_t *flag = (int32_t *)((char *)ctx->small.p + SM_COUNTERS) + 2;
    ALS_HIP(ctx, hipMemcpyAsync(ctx->host_counters + 2, flag, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    ALS_HIP(ctx, hipStreamSynchronize(s));
    if (ctx->host_counters[2] != 0) {
        ALS_HIP(ctx, hipMemsetAsync(flag, 0, sizeof(int32_t), s));
        if (ctx->host_counters[2] & 2)
            return fail(ctx, ALS_EINVAL, "CSR structure inconsistent with its nnz: rows were dropped (run als_check_csr)");
        return fail(ctx, ALS_ENOTSPD, "a non-positive pivot was met while factorising a row system");
    }
    return ALS_OK;
}

als_status als_loss(als_ctx *ctx, const als_csr *Y, const als_table *W, const als_table *H,
                    const als_params *prm, double *loss_host, void *stream) {
    if (!ctx) return ALS_EINVAL;
    als_status st;
    if ((st = check_csr_args(ctx, Y, "Y")) != ALS_OK) return st;
    if ((st = check_table(ctx, W, "W")) != ALS_OK) return st;
    if ((st = check_table(ctx, H, "H")) != ALS_OK) return st;
    if ((st = check_params(ctx, prm)) != ALS_OK) return st;
    if (!loss_host) return fail(ctx, ALS_EINVAL, "loss_host is null");
    if (W->d != H->d) return fail(ctx, ALS_ESHAPE, "W and H differ in d");
    if (W->dtype != H->dtype) return fail(ctx, ALS_EDTYPE, "W and H differ in dtype");
    if (Y->rows != W->rows || Y->cols != H->rows) return fail(ctx, ALS_ESHAPE, "Y does not fit W and H");
    timers_reset(ctx);
    hipStream_t s = (hipStream_t)stream;
    float *GH = (float *)ctx->gram_h.p, *GW = (float *)ctx->gram_w.p;
    if ((st = launch_gramian(ctx, H, GH, s)) != ALS_OK) return st;
    if ((st = launch_gramian(ctx, W, GW, s)) != ALS_OK) return st;
    double *out_dev = (double *)((char *)ctx->small.p + SM_LOSS);
    if ((st = launch_loss(ctx, Y, W, H, GW, GH, prm, out_dev, s)) != ALS_OK) return st;
    ALS_HIP(ctx, hipMemcpyAsync(ctx->host_scalar, out_dev, sizeof(double), hipMemcpyDeviceToHost, s));
    if ((st = als_status_sync(ctx, stream)) != ALS_OK) return st;
    *loss_host = ctx->host_scalar[0];
    return ALS_OK;
}

als_status als_topk(als_ctx *ctx, const als_table *Q, const als_table *H, const als_csr *exclude, int32_t k,
                    int32_t *ids, float *scores, void *stream) {
    if (!ctx) return ALS_EINVAL;
    als_status st;
    if ((st = check_table(ctx, Q, "Q")) != ALS_OK) return st;
    if ((st = check_table(ctx, H, "H")) != ALS_OK) return st;
    if (Q->d != H->d) return fail(ctx, ALS_ESHAPE, "Q and H differ in d");
    if (Q->dtype != H->dtype) return fail(ctx, ALS_EDTYPE, "Q and H differ in dtype");
    if (k < 1 || k > ALS_TOPK_MAX_K) return fail(ctx, ALS_EINVAL, "k must be in [1, ALS_TOPK_MAX_K]");
    if (H->rows > INT32_MAX) return fail(ctx, ALS_ESHAPE, "item ids must fit int32");
    if (!ids || !scores) return fail(ctx, ALS_EINVAL, "ids or scores is null");
    if (exclude) {
        if ((st = check_csr_args(ctx, exclude, "exclude")) != ALS_OK) return st;
        if (exclude->rows != Q->rows || exclude->cols != H->rows)
            return fail(ctx, ALS_ESHAPE, "exclude must have one row per query and one column per item");
    }
    if (Q->rows == 0) return ALS_OK;
    return launch_topk(ctx, Q, H, exclude, k, ids, scores, (hipStream_t)stream);
}

als_status als_check_csr(als_ctx *ctx, const als_csr *Y, void *stream) {
    if (!ctx) return ALS_EINVAL;
    als_status st = check_csr_args(ctx, Y, "Y");
    if (st != ALS_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    int32_t *flag = (int32_t *)((char *)ctx->small.p + SM_COUNTERS) + 4;
    ALS_HIP(ctx, hipMemsetAsync(flag, 0, sizeof(int32_t), s));
    if ((st = launch_check_csr(ctx, Y, flag, s)) != ALS_OK) return st;
    ALS_HIP(ctx, hipMemcpyAsync(ctx->host_counters + 4, flag, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    ALS_HIP(ctx, hipStreamSynchronize(s));
    if (ctx->host_counters[4] != 0) return fail(ctx, ALS_EINVAL, "CSR structure is invalid (indptr order or column id range)");
    return ALS_OK;
}

als_status als_copy_probe(als_ctx *ctx, const void *src, void *dst, int64_t bytes, void *stream) {
    if (!ctx) return ALS_EINVAL;
    if (!src || !dst || bytes < 0 || bytes % 16 != 0 || ((uintptr_t)src % 16) || ((uintptr_t)dst % 16))
        return fail(ctx, ALS_EINVAL, "copy probe needs 16-byte aligned buffers and a size that is a multiple of 16");
    return launch_copy_probe(ctx, src, dst, bytes, (hipStream_t)stream);
}

als_status als_set_timing(als_ctx *ctx, int enabled) {
    if (!ctx) return ALS_EINVAL;
    ctx->timing = enabled != 0;
    return ALS_OK;
}

als_status als_get_timing(als_ctx *ctx, double *ms_host) {
    if (!ctx || !ms_host) return ALS_EINVAL;
    for (double &v : ctx->timing_ms) v = 0.0;
    for (auto &t : ctx->timers) {
        ALS_HIP(ctx, hipEventSynchronize(t.e1));
        float ms = 0.f;
        ALS_HIP(ctx, hipEventElapsedTime(&ms, t.e0, t.e1));
        ctx->timing_ms[t.slot] += ms;
        ctx->timing_ms[T_COUNT + t.slot] += 1.0;
    }
    for (int i = 0; i < 2 * T_COUNT; ++i) ms_host[i] = ctx->timing_ms[i];
    return ALS_OK;
}

const char *als_strerror(als_status st) {
    switch (st) {
        case ALS_OK: return "ok";
        case ALS_EINVAL: return "invalid argument";
        case ALS_ESHAPE: return "shape mismatch";
        case ALS_EDTYPE: return "unsupported dtype or dimension";
        case ALS_EALIAS: return "output overlaps input";
        case ALS_ENOTSPD: return "system not positive definite";
        case ALS_ENOMEM: return "out of memory";
        case ALS_EHIP: return "HIP runtime error";
    }
    return "unknown status";
}

const char *als_last_error(const als_ctx *ctx) { return ctx ? ctx->last_error.c_str() : ""; }

}  // extern "C"
