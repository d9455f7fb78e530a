// Stage 1 of the pipeline declared in sams.h: Count Sketch accumulation (Sec. II-C update rule).
#include "sams_ctx.h"

// Every formula below is evaluated as separate IEEE-754 binary32 operations, rounded to nearest:
// no fused multiply-add is formed (here and with -ffp-contract=off on the command line), and
// x / y and sqrtf(x) are the correctly rounded ones (hipcc's default; never build this file with
// -ffast-math or -fno-hip-fp32-correctly-rounded-divide-sqrt).
#pragma clang fp contract(off)

namespace sams {
// ------------------------------------------------------------------------------------------
// stage 1: Count Sketch accumulation (Sec. II-C)
// ------------------------------------------------------------------------------------------
// One thread per coordinate: the r bucket/sign hashes are evaluated once and reused by all workers.
__global__ void __launch_bounds__(256)
k_sketch_atomic(const float *__restrict__ u, float *__restrict__ S, HashParams hp, int32_t n,
                int64_t d, int64_t c)
{
    int64_t l = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (l >= d) return;
    const int r = hp.r;
    for (int j = 0; j < r; ++j) {
        uint32_t b = bucket_of(hp, j, (uint32_t)l);
        bool neg = sign_neg(hp, j, (uint32_t)l);
        for (int32_t i = 0; i < n; ++i) {
            float val = u[(int64_t)i * d + l];
            atomicAdd(&S[((int64_t)i * r + j) * c + b], neg ? -val : val);
        }
    }
}

int enqueue_sketch(sams_ctx *ctx, const float *u, float *S_workers)
{
    if (ctx->plan.mode != PLAN_ATOMIC) return enqueue_sketch_planned(ctx, u, S_workers);
    const int64_t cells = (int64_t)ctx->n * ctx->r * ctx->c;
    SAMS_TRY(enqueue_fill_u32(ctx, (uint32_t *)S_workers, cells, 0u));
    SAMS_LAUNCH(ctx, KID_SKETCH_ATOMIC, k_sketch_atomic, grid_for(ctx->d, 256), 256, u, S_workers,
                ctx->hp, ctx->n, ctx->d, ctx->c);
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

}  // namespace sams
