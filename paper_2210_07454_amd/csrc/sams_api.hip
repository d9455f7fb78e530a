// The extern "C" entry points declared in include/sams.h: argument validation, context life cycle,
// optional per-kernel timing, and the calls into the per-stage enqueue functions.
#include <stdlib.h>
#include <string.h>
#include <mutex>
#include <new>

#include "sams_ctx.h"

namespace sams {

int g_last_hip_error = 0;
Tunables g_tun = {0, 0, 0, 0, 0, 1024, 0, 0, 1, 0, 16, 0, 0, 2};
static std::mutex g_tun_mutex;      // sams_configure against the copy sams_create takes

static const char *const kKernelNames[KID_COUNT] = {
    "k_fill_u32", "k_hash_dump", "k_tail_x", "k_tail_zero_e", "k_head", "k_sketch_atomic", "k_reduce",
    "k_estimate", "k_sel_init", "k_sel_hist", "k_sel_pick", "k_sel_count", "k_sel_scan", "k_sel_write",
    "k_gather", "k_plan_build", "k_bin_scatter", "k_bin_accumulate", "k_sketch_lds", "k_bin_lookup",
    "k_bin_collect", "k_est_median", "k_head_scatter", "k_refine_map", "k_head_pa", "k_head_sparse_v", "k_sel_small"};

const char *kernel_name(int kid) { return (kid >= 0 && kid < KID_COUNT) ? kKernelNames[kid] : ""; }

__global__ void k_fill_u32(uint32_t *p, int64_t n, uint32_t val)
{
    int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    int64_t st = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += st) p[i] = val;
}

__global__ void k_hash_dump(HashParams hp, int64_t d, int32_t *bucket, int8_t *sign)
{
    int64_t l = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (l >= d) return;
    for (int j = 0; j < hp.r; ++j) {
        bucket[(int64_t)j * d + l] = (int32_t)bucket_of(hp, j, (uint32_t)l);
        sign[(int64_t)j * d + l] = sign_neg(hp, j, (uint32_t)l) ? (int8_t)-1 : (int8_t)1;
    }
}

int enqueue_fill_u32(sams_ctx *ctx, uint32_t *p, int64_t n, uint32_t val)
{
    SAMS_LAUNCH(ctx, KID_FILL, k_fill_u32, grid_for(n, 256 * 4, 1 << 16), 256, p, n, val);
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

int enqueue_hash_dump(sams_ctx *ctx, int32_t *bucket, int8_t *sign)
{
    SAMS_LAUNCH(ctx, KID_HASH_DUMP, k_hash_dump, grid_for(ctx->d, 256), 256, ctx->hp, ctx->d, bucket, sign);
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

// folds the finished event pairs into the per-kernel totals (synchronises the stream)
static int prof_drain(sams_ctx *ctx)
{
    if (ctx->prof_used == 0) return SAMS_OK;
    SAMS_HIP(hipStreamSynchronize(ctx->stream));
    for (int s = 0; s < ctx->prof_used; ++s) {
        float ms = 0.f;
        SAMS_HIP(hipEventElapsedTime(&ms, ctx->prof[s].a, ctx->prof[s].b));
        ctx->prof_ms[ctx->prof[s].kid] += ms;
        ctx->prof_n[ctx->prof[s].kid] += 1;
    }
    ctx->prof_used = 0;
    return SAMS_OK;
}

}  // namespace sams

using namespace sams;

extern "C" {

int sams_last_hip_error(void) { return g_last_hip_error; }

int sams_create(sams_ctx **out, int64_t d, int32_t n, int32_t r, int64_t c, int64_t k,
                const uint32_t *hash_host, void *hip_stream)
{
    if (!out) return SAMS_EINVAL;
    *out = nullptr;
    if (!hash_host) return SAMS_EINVAL;
    if (d < 1 || d >= (int64_t)kP31 || n < 1 || n > kMaxWorkers || r < 1 || r > SAMS_MAX_ROWS || c < 1 ||
        c >= (int64_t)kP31 || k < 1 || k > d)
        return SAMS_EINVAL;
    for (int j = 0; j < r; ++j) {
        const uint32_t *h = hash_host + 4 * j;
        if (h[0] < 1 || h[0] >= kP31 || h[1] >= kP31 || h[2] < 1 || h[2] >= kP31 || h[3] >= kP31)
            return SAMS_EINVAL;
    }
    sams_ctx *ctx = new (std::nothrow) sams_ctx;
    if (!ctx) return SAMS_ENOMEM;
    memset(ctx, 0, sizeof(*ctx));
    ctx->d = d; ctx->n = n; ctx->r = r; ctx->c = c; ctx->k = k;
    ctx->stream = (hipStream_t)hip_stream;
    ctx->prof_only = -1;
    {
        std::lock_guard<std::mutex> lock(g_tun_mutex);
        ctx->tun = g_tun;                                            // every later call reads this copy only
    }
    ctx->hp.r = r;
    ctx->hp.modc = make_modc((uint32_t)c);
    for (int j = 0; j < r; ++j) {
        ctx->hp.row[j].ah = hash_host[4 * j + 0];
        ctx->hp.row[j].bh = hash_host[4 * j + 1];
        ctx->hp.row[j].as = hash_host[4 * j + 2];
        ctx->hp.row[j].bs = hash_host[4 * j + 3];
    }
    ctx->ntile = (d + kSelTile - 1) / kSelTile;
    const int64_t words = (d + 31) / 32;
    struct { void **p; int64_t bytes; } allocs[] = {
        {(void **)&ctx->est, d * 4},
        {(void **)&ctx->bitmap, words * 4},
        {(void **)&ctx->hist, kHistBins * 4},
        {(void **)&ctx->sel, (int64_t)sizeof(SelState)},
        {(void **)&ctx->cnt, 2 * ctx->ntile * 4},
        {(void **)&ctx->base, 2 * ctx->ntile * 4},
    };
    for (auto &a : allocs) {
        hipError_t e = hipMalloc(a.p, (size_t)a.bytes);
        if (e != hipSuccess) {
            g_last_hip_error = (int)e;
            (void)hipGetLastError();
            sams_destroy(ctx);
            return SAMS_ENOMEM;
        }
        ctx->scratch_bytes += a.bytes;
    }
    void *static_scratch = nullptr;
    if (ctx->tun.fuse_head == 2 && ctx->tun.sketch_path != 1) {      // the per-worker fused head compacts g on I_{t-1}
        struct { void **p; int64_t bytes; } extra[] = {{(void **)&ctx->wordrank, words * 4}, {(void **)&ctx->gsel, (int64_t)n * k * 4}};
        for (auto &a : extra) {
            hipError_t e = hipMalloc(a.p, (size_t)a.bytes);
            if (e != hipSuccess) {
                g_last_hip_error = (int)e;
                (void)hipGetLastError();
                sams_destroy(ctx);
                return SAMS_ENOMEM;
            }
            ctx->scratch_bytes += a.bytes;
        }
    }
    int rc = static_scratch_ptr(&static_scratch);                    // resolved here so that topk_refine_static never has to
    if (rc == SAMS_OK) rc = enqueue_fill_u32(ctx, ctx->bitmap, words, 0u);
    if (rc == SAMS_OK && ctx->tun.sketch_path != 1) rc = plan_create(ctx, ctx->tun);
    if (rc != SAMS_OK) {
        sams_destroy(ctx);
        return rc;
    }
    *out = ctx;
    return SAMS_OK;
}

int sams_destroy(sams_ctx *ctx)
{
    if (!ctx) return SAMS_OK;
    int rc = SAMS_OK;
    hipError_t e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) { g_last_hip_error = (int)e; rc = SAMS_EHIP; }
    void *ptrs[] = {ctx->est, ctx->bitmap, ctx->wordrank, ctx->gsel, ctx->hist, ctx->sel, ctx->cnt, ctx->base};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    plan_destroy(ctx);
    if (ctx->prof) {
        for (int s = 0; s < kProfPool; ++s) {
            if (ctx->prof[s].a) (void)hipEventDestroy(ctx->prof[s].a);
            if (ctx->prof[s].b) (void)hipEventDestroy(ctx->prof[s].b);
        }
        free(ctx->prof);
    }
    delete ctx;
    return rc;
}

int sams_configure(const char *key, int value)
{
    if (!key) return SAMS_EINVAL;
    std::lock_guard<std::mutex> lock(g_tun_mutex);
    if (!strcmp(key, "tile_log2")) {
        if (value != 0 && (value < 6 || value > 14)) return SAMS_EINVAL;
        g_tun.tile_log2 = value;
    } else if (!strcmp(key, "win_log2")) {
        if (value != 0 && (value < 4 || value > 15)) return SAMS_EINVAL;
        g_tun.win_log2 = value;
    } else if (!strcmp(key, "chunk_log2")) {
        if (value != 0 && (value < 6 || value > 11)) return SAMS_EINVAL;
        g_tun.chunk_log2 = value;
    } else if (!strcmp(key, "acc_threads")) {
        if (value != 0 && value != 256 && value != 512 && value != 1024) return SAMS_EINVAL;
        g_tun.acc_threads = value;
    } else if (!strcmp(key, "scatter_threads")) {
        if (value != 256 && value != 512 && value != 1024) return SAMS_EINVAL;
        g_tun.scatter_threads = value;
    } else if (!strcmp(key, "estimate_path")) {
        if (value < 0 || value > 2) return SAMS_EINVAL;
        g_tun.estimate_path = value;
    } else if (!strcmp(key, "fuse_head")) {
        if (value < 0 || value > 2) return SAMS_EINVAL;
        g_tun.fuse_head = value;
    } else if (!strcmp(key, "fuse_median")) {
        if (value < 0 || value > 1) return SAMS_EINVAL;
        g_tun.fuse_median = value;
    } else if (!strcmp(key, "stage_rows")) {
        if (value < 0 || value > SAMS_MAX_ROWS) return SAMS_EINVAL;
        g_tun.stage_rows = value;
    } else if (!strcmp(key, "run_pad")) {
        if (value != 4 && value != 8 && value != 16 && value != 32) return SAMS_EINVAL;
        g_tun.run_pad = value;
    } else if (!strcmp(key, "stage_interleave")) {
        if (value < 0 || value > 1) return SAMS_EINVAL;
        g_tun.stage_interleave = value;
    } else if (!strcmp(key, "stage_spread")) {
        if (value < 0 || value > 1) return SAMS_EINVAL;
        g_tun.stage_spread = value;
    } else if (!strcmp(key, "acc_wide")) {
        if (value < 0 || value > 2) return SAMS_EINVAL;
        g_tun.acc_wide = value;
    } else if (!strcmp(key, "sketch_path")) {
        if (value < 0 || value > 3) return SAMS_EINVAL;
        g_tun.sketch_path = value;
    } else {
        return SAMS_EINVAL;
    }
    return SAMS_OK;
}

int sams_sketch_mode(const sams_ctx *ctx) { return ctx ? ctx->plan.mode : -1; }

int sams_accumulate_variant(const sams_ctx *ctx)
{
    return (ctx && ctx->plan.mode == PLAN_BINNED) ? ctx->plan.acc_variant : -1;
}

int64_t sams_record_rows(const sams_ctx *ctx)
{
    return (ctx && ctx->plan.mode == PLAN_BINNED) ? (int64_t)ctx->plan.rec_mask : -1;
}

int64_t sams_scratch_bytes(const sams_ctx *ctx) { return ctx ? ctx->scratch_bytes : 0; }

int64_t sams_precondition_device_memory(double fraction)
{
    if (!(fraction > 0.0) || fraction > 1.0) return SAMS_EINVAL;
    size_t free_b = 0, total_b = 0;
    hipError_t e = hipMemGetInfo(&free_b, &total_b);
    if (e != hipSuccess) { g_last_hip_error = (int)e; return SAMS_EHIP; }
    const size_t block = (size_t)1 << 30;
    const size_t want = (size_t)((double)free_b * fraction) / block;
    void **held = (void **)malloc((want + 1) * sizeof(void *));
    if (!held) return SAMS_ENOMEM;
    size_t got = 0;
    while (got < want) {
        if (hipMalloc(&held[got], block) != hipSuccess) {
            (void)hipGetLastError();                                 // out of memory: what could be had has been had
            break;
        }
        ++got;
    }
    e = hipDeviceSynchronize();
    for (size_t q = 0; q < got; ++q) (void)hipFree(held[q]);
    free(held);
    if (e != hipSuccess) { g_last_hip_error = (int)e; return SAMS_EHIP; }
    return (int64_t)got;
}

int sams_profile_kernels(void) { return KID_COUNT; }

const char *sams_profile_name(int kernel) { return kernel_name(kernel); }

int sams_profile_enable(sams_ctx *ctx, int on)
{
    if (!ctx) return SAMS_EINVAL;
    if (on) {
        if (!ctx->prof) {
            ctx->prof = (ProfRec *)calloc(kProfPool, sizeof(ProfRec));
            if (!ctx->prof) return SAMS_ENOMEM;
            for (int s = 0; s < kProfPool; ++s) {
                hipError_t e = hipEventCreate(&ctx->prof[s].a);
                if (e == hipSuccess) e = hipEventCreate(&ctx->prof[s].b);
                if (e != hipSuccess) {                               // all or nothing: a later call starts over
                    for (int q = 0; q <= s; ++q) {
                        if (ctx->prof[q].a) (void)hipEventDestroy(ctx->prof[q].a);
                        if (ctx->prof[q].b) (void)hipEventDestroy(ctx->prof[q].b);
                    }
                    free(ctx->prof);
                    ctx->prof = nullptr;
                    g_last_hip_error = (int)e;
                    (void)hipGetLastError();
                    return SAMS_EHIP;
                }
            }
        }
        SAMS_TRY(prof_drain(ctx));
        for (int q = 0; q < KID_COUNT; ++q) { ctx->prof_ms[q] = 0.0; ctx->prof_n[q] = 0; }
        ctx->prof_on = 1;
    } else {
        ctx->prof_on = 0;
    }
    return SAMS_OK;
}

int sams_profile_only(sams_ctx *ctx, int kernel)
{
    if (!ctx || kernel < -1 || kernel >= KID_COUNT) return SAMS_EINVAL;
    ctx->prof_only = kernel;
    return SAMS_OK;
}

int sams_profile_read(sams_ctx *ctx, double *total_ms, int64_t *launches)
{
    if (!ctx || !total_ms || !launches) return SAMS_EINVAL;
    SAMS_TRY(prof_drain(ctx));
    for (int q = 0; q < KID_COUNT; ++q) { total_ms[q] = ctx->prof_ms[q]; launches[q] = ctx->prof_n[q]; }
    return SAMS_OK;
}

int sams_hash_dump(sams_ctx *ctx, int32_t *bucket, int8_t *sign)
{
    if (!ctx || !bucket || !sign) return SAMS_EINVAL;
    return enqueue_hash_dump(ctx, bucket, sign);
}

int sketch_accumulate(sams_ctx *ctx, const float *u, float *S_workers)
{
    if (!ctx || !u || !S_workers || !aligned16(u) || !aligned16(S_workers)) return SAMS_EINVAL;
    return enqueue_sketch(ctx, u, S_workers);
}

int sketch_reduce(sams_ctx *ctx, const float *S_workers, float *S_mean)
{
    if (!ctx || !S_workers || !S_mean || !aligned16(S_workers) || !aligned16(S_mean)) return SAMS_EINVAL;
    return enqueue_reduce(ctx, S_workers, S_mean);
}

int unsketch_estimates(sams_ctx *ctx, const float *S_mean, const float *vhat, float *est)
{
    if (!ctx || !S_mean || !est || !aligned16(S_mean) || !aligned16(est) || !aligned16(vhat))
        return SAMS_EINVAL;
    return enqueue_estimate(ctx, S_mean, vhat, est, nullptr, nullptr);
}

int unsketch_topk(sams_ctx *ctx, const float *S_mean, const float *vhat, int32_t *idx, float *est_sel)
{
    if (!ctx || !S_mean || !idx || !aligned16(S_mean) || !aligned16(idx) || !aligned16(vhat) ||
        !aligned16(est_sel))
        return SAMS_EINVAL;
    // the selection's state is reset first, so that the estimate kernel can already take the first histogram
    const SelScratch sc = ctx_sel_scratch(ctx);
    const bool passes = select_uses_passes(ctx->d);
    bool hist0_done = false;
    if (passes) SAMS_TRY(enqueue_select_begin(ctx, ctx->stream, sc, ctx->k));
    SAMS_TRY(enqueue_estimate(ctx, S_mean, vhat, ctx->est, passes ? sc.hist : nullptr, &hist0_done));
    return enqueue_select(ctx, ctx->stream, sc, ctx->est, ctx->d, ctx->k, idx, est_sel, passes, hist0_done);
}

int topk_refine(sams_ctx *ctx, const int32_t *idx_in, const float *delta_in, int64_t k_out, int32_t *idx_out,
                float *delta_out)
{
    if (!ctx || !idx_in || !delta_in || !idx_out || !delta_out || k_out < 1 || k_out > ctx->k) return SAMS_EINVAL;
    if (!aligned16(idx_in) || !aligned16(delta_in) || !aligned16(idx_out) || !aligned16(delta_out)) return SAMS_EINVAL;
    // the estimate scratch is free at this point: it holds the positions among the candidates
    return enqueue_refine(ctx, ctx->stream, ctx_sel_scratch(ctx), reinterpret_cast<int32_t *>(ctx->est), idx_in, delta_in,
                          ctx->k, k_out, idx_out, delta_out);
}

int gather_topk(sams_ctx *ctx, const float *u, const float *vhat, const int32_t *idx, float *U_workers,
                float *delta)
{
    if (!ctx || !u || !idx || !U_workers || !delta || !aligned16(u) || !aligned16(vhat) ||
        !aligned16(idx) || !aligned16(U_workers) || !aligned16(delta))
        return SAMS_EINVAL;
    return enqueue_gather(ctx, u, vhat, idx, U_workers, delta);
}

int amsgrad_ef_update(sams_ctx *ctx, const float *g_next, float *m, float *e_u, float *v, float *vhat,
                      float *x, const int32_t *idx, const float *delta, int64_t k_sel, float beta1,
                      float beta2, float lr, float ef_ratio)
{
    if (!ctx || !m || !e_u || !v || !vhat || !x) return SAMS_EINVAL;
    if (k_sel < 0 || k_sel > ctx->k || (k_sel > 0 && (!idx || !delta))) return SAMS_EINVAL;
    if (!aligned16(g_next) || !aligned16(m) || !aligned16(e_u) || !aligned16(v) || !aligned16(vhat) ||
        !aligned16(x) || !aligned16(idx) || !aligned16(delta))
        return SAMS_EINVAL;
    ctx->plan.staged_u = nullptr;                                    // e_u is about to change
    SAMS_TRY(enqueue_tail(ctx, e_u, x, idx, delta, k_sel, lr, g_next == nullptr));
    if (g_next) {
        if (head_can_fuse(ctx))
            SAMS_TRY(enqueue_head_scatter(ctx, g_next, m, e_u, v, vhat, beta1, beta2, ef_ratio, false, idx, k_sel));
        else
            SAMS_TRY(enqueue_head(ctx, g_next, m, e_u, v, vhat, beta1, beta2, ef_ratio));
    }
    return SAMS_OK;
}

int amsgrad_ef_update_pa(sams_ctx *ctx, const float *g_next, float *m, float *e_u, float *v_workers,
                         float *vhat_workers, float *x, const int32_t *idx, const float *delta, int64_t k_sel,
                         float beta1, float beta2, float lr, float ef_ratio)
{
    if (!ctx || !m || !e_u || !v_workers || !vhat_workers || !x) return SAMS_EINVAL;
    if (k_sel < 0 || k_sel > ctx->k || (k_sel > 0 && (!idx || !delta))) return SAMS_EINVAL;
    if (!aligned16(g_next) || !aligned16(m) || !aligned16(e_u) || !aligned16(v_workers) ||
        !aligned16(vhat_workers) || !aligned16(x) || !aligned16(idx) || !aligned16(delta))
        return SAMS_EINVAL;
    ctx->plan.staged_u = nullptr;                                    // e_u is about to change
    SAMS_TRY(enqueue_tail(ctx, e_u, x, idx, delta, k_sel, lr, g_next == nullptr));
    if (g_next) {
        if (head_can_fuse(ctx))
            SAMS_TRY(enqueue_head_scatter(ctx, g_next, m, e_u, v_workers, vhat_workers, beta1, beta2, ef_ratio, true, idx, k_sel));
        else
            SAMS_TRY(enqueue_head_pa(ctx, g_next, m, e_u, v_workers, vhat_workers, beta1, beta2, ef_ratio));
    }
    return SAMS_OK;
}

}  // extern "C"
