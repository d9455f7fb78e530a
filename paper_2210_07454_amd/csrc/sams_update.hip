// Stage 5 (AMSGrad update with error feedback: tail and head of Alg. 2), stage 2 (mean of the worker
// sketches) and stage 4 (exact values of the selected coordinates) of the pipeline declared in sams.h.
#include "sams_ctx.h"

// Every formula below is evaluated as separate IEEE-754 binary32 operations, rounded to nearest:
// no fused multiply-add is formed (here and with -ffp-contract=off on the command line), and
// x / y and sqrtf(x) are the correctly rounded ones (hipcc's default; never build this file with
// -ffast-math or -fno-hip-fp32-correctly-rounded-divide-sqrt).
#pragma clang fp contract(off)

namespace sams {
// ------------------------------------------------------------------------------------------
// stage 5: tail (finish iteration t) and head (start iteration t+1) of Alg. 2
// ------------------------------------------------------------------------------------------
// x[idx[q]] -= lr * delta[q]; mark idx[q] in the bitmap (I_t for the next head).  wordrank != null: idx is ascending
// (as amsgrad_ef_update requires), so the rank of the first coordinate of every bitmap word that has one is its q
__global__ void k_tail_x(const int32_t *__restrict__ idx, const float *__restrict__ delta, int64_t k,
                         float lr, float *__restrict__ x, uint32_t *__restrict__ bitmap, uint32_t *__restrict__ wordrank)
{
    int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q >= k) return;
    uint32_t l = (uint32_t)idx[q];
    x[l] = (x[l] - (lr * delta[q]));
    atomicOr(&bitmap[l >> 5], 1u << (l & 31));
    if (wordrank && (q == 0 || ((uint32_t)idx[q - 1] >> 5) != (l >> 5))) wordrank[l >> 5] = (uint32_t)q;
}

// e[i][idx[q]] = 0 (only needed when no head follows; otherwise the head reads the bitmap)
__global__ void k_tail_zero_e(const int32_t *__restrict__ idx, int64_t k, int32_t n, int64_t d,
                              float *__restrict__ e)
{
    int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q >= k) return;
    int64_t l = idx[q];
    for (int32_t i = 0; i < n; ++i) e[(int64_t)i * d + l] = 0.0f;
}

// Dense head.  One thread owns VEC consecutive coordinates and walks the n workers, so that the
// worker sum of g needed for h (only on I_t) comes for free and in ascending worker order.
template <int VEC>
__global__ void __launch_bounds__(256)
k_head(const float *__restrict__ g, float *__restrict__ m, float *__restrict__ e,
       float *__restrict__ v, float *__restrict__ vhat, const uint32_t *__restrict__ bitmap,
       int32_t n, int64_t d, float beta1, float omb1, float beta2, float omb2, float rho)
{
    int64_t l0 = (blockIdx.x * (int64_t)blockDim.x + threadIdx.x) * VEC;
    if (l0 >= d) return;
    uint32_t selbits;
    if (VEC == 4) {
        selbits = (bitmap[l0 >> 5] >> (l0 & 31)) & 0xFu;
    } else {
        selbits = (bitmap[l0 >> 5] >> (l0 & 31)) & 1u;
    }
    float gs[VEC];
    for (int32_t i = 0; i < n; ++i) {
        int64_t off = (int64_t)i * d + l0;
        float gv[VEC], mv[VEC], ev[VEC];
        if (VEC == 4) {
            float4 a = *reinterpret_cast<const float4 *>(g + off);
            float4 b = *reinterpret_cast<const float4 *>(m + off);
            float4 cc = *reinterpret_cast<const float4 *>(e + off);
            gv[0] = a.x; gv[1] = a.y; gv[2] = a.z; gv[3] = a.w;
            mv[0] = b.x; mv[1] = b.y; mv[2] = b.z; mv[3] = b.w;
            ev[0] = cc.x; ev[1] = cc.y; ev[2] = cc.z; ev[3] = cc.w;
        } else {
            gv[0] = g[off]; mv[0] = m[off]; ev[0] = e[off];
        }
#pragma unroll
        for (int t = 0; t < VEC; ++t) {
            float mm = ((beta1 * mv[t]) + (omb1 * gv[t]));
            float ein = ((selbits >> t) & 1u) ? 0.0f : ev[t];       // e_t is zero on I_t
            mv[t] = mm;
            ev[t] = (mm + (rho * ein));
            gs[t] = (i == 0) ? gv[t] : (gs[t] + gv[t]);
        }
        if (VEC == 4) {
            *reinterpret_cast<float4 *>(m + off) = make_float4(mv[0], mv[1], mv[2], mv[3]);
            *reinterpret_cast<float4 *>(e + off) = make_float4(ev[0], ev[1], ev[2], ev[3]);
        } else {
            m[off] = mv[0]; e[off] = ev[0];
        }
    }
    float fn = (float)n;
#pragma unroll
    for (int t = 0; t < VEC; ++t) {
        float h = ((selbits >> t) & 1u) ? (gs[t] / fn) : 0.0f;
        float vv = (beta2 * v[l0 + t]) + (omb2 * (h * h));
        v[l0 + t] = vv;
        if (vv > vhat[l0 + t]) vhat[l0 + t] = vv;
    }
}

// ------------------------------------------------------------------------------------------
// stage 2: mean of the worker sketches (Alg. 2, master)
// ------------------------------------------------------------------------------------------
// VEC = 4: four consecutive cells per thread with 16-byte loads (needs r*c to be a multiple of 4, so that
// every worker's table starts on a 16-byte boundary)
__device__ __forceinline__ float4 ld4_stream(const float *p)
{
    typedef float vec4f __attribute__((ext_vector_type(4)));
    const vec4f t = __builtin_nontemporal_load(reinterpret_cast<const vec4f *>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}

template <int VEC>
__global__ void __launch_bounds__(256)
k_reduce(const float *__restrict__ S_w, float *__restrict__ S_mean, int32_t n, int64_t rc)
{
    int64_t t = (blockIdx.x * (int64_t)blockDim.x + threadIdx.x) * VEC;
    const int64_t st = (int64_t)gridDim.x * blockDim.x * VEC;
    const float fn = (float)n;
    for (; t < rc; t += st) {
        if constexpr (VEC == 4) {
            float4 acc = ld4_stream(S_w + t);                        // every table is read once: streaming loads
            for (int32_t i0 = 1; i0 < n; i0 += 8) {                  // eight tables' loads in flight, added in worker order
                float4 b[8];
#pragma unroll
                for (int z = 0; z < 8; ++z) {
                    const int32_t i = (i0 + z < n) ? (i0 + z) : (n - 1);
                    b[z] = ld4_stream(S_w + (int64_t)i * rc + t);
                }
#pragma unroll
                for (int z = 0; z < 8; ++z) {
                    if (i0 + z < n) {
                        acc.x = (acc.x + b[z].x);
                        acc.y = (acc.y + b[z].y);
                        acc.z = (acc.z + b[z].z);
                        acc.w = (acc.w + b[z].w);
                    }
                }
            }
            *reinterpret_cast<float4 *>(S_mean + t) = make_float4((acc.x / fn), (acc.y / fn), (acc.z / fn), (acc.w / fn));
        } else {
            float acc = S_w[t];
            for (int32_t i = 1; i < n; ++i) acc = (acc + S_w[(int64_t)i * rc + t]);
            S_mean[t] = (acc / fn);
        }
    }
}

// ------------------------------------------------------------------------------------------
// stage 4: exact values of the selected coordinates (second round, Sec. III-A)
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_gather(const float *__restrict__ u, const float *__restrict__ vhat, const int32_t *__restrict__ idx,
         int64_t k, int32_t n, int64_t d, float *__restrict__ U_w, float *__restrict__ delta)
{
    int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q >= k) return;
    int64_t l = idx[q];
    float acc = 0.0f;
    // eight workers' values are fetched before the first is used (with many workers and few coordinates the
    // kernel is a chain of memory latencies otherwise); they are still added in worker order
    for (int32_t i0 = 0; i0 < n; i0 += 8) {
        float val[8];
#pragma unroll
        for (int z = 0; z < 8; ++z) {
            const int32_t i = (i0 + z < n) ? (i0 + z) : (n - 1);
            val[z] = u[(int64_t)i * d + l];
        }
#pragma unroll
        for (int z = 0; z < 8; ++z) {
            if (i0 + z < n) {
                U_w[(int64_t)(i0 + z) * k + q] = val[z];
                acc = (i0 + z == 0) ? val[z] : (acc + val[z]);
            }
        }
    }
    float mean = (acc / (float)n);
    delta[q] = vhat ? (mean / sqrtf(vhat[l])) : mean;
}

// The same for many workers: 32 lanes share a coordinate and fetch its n values side by side; they meet in LDS
// and one lane adds them in worker order.  With n in the tens and k in the hundreds the one-thread-per-
// coordinate kernel is a chain of n memory latencies on a handful of compute units.
__global__ void __launch_bounds__(256)
k_gather_wide(const float *__restrict__ u, const float *__restrict__ vhat, const int32_t *__restrict__ idx,
              int64_t k, int32_t n, int64_t d, float *__restrict__ U_w, float *__restrict__ delta)
{
    __shared__ float vals[kWideCoords * kMaxWorkers];
    const int ql = threadIdx.x >> 5, wl = threadIdx.x & 31;
    const int64_t q = blockIdx.x * (int64_t)kWideCoords + ql;
    const int64_t l = q < k ? idx[q] : 0;
    if (q < k) {
        for (int32_t i = wl; i < n; i += 32) {
            const float val = u[(int64_t)i * d + l];
            U_w[(int64_t)i * k + q] = val;
            vals[ql * n + i] = val;
        }
    }
    __syncthreads();
    if (q < k && wl == 0) {
        float acc = vals[ql * n];
        for (int32_t i = 1; i < n; ++i) acc = (acc + vals[ql * n + i]);
        const float mean = (acc / (float)n);
        delta[q] = vhat ? (mean / sqrtf(vhat[l])) : mean;
    }
}

// Head of Alg. 1 (parameter averaging): per-worker second moments, u = m / sqrt(vhat) + rho * e.
// Purely elementwise over the n*d entries; e is taken as zero on the recorded index set (bitmap over d).
template <int VEC>
__global__ void __launch_bounds__(256)
k_head_pa(const float *__restrict__ g, float *__restrict__ m, float *__restrict__ e, float *__restrict__ vw,
          float *__restrict__ vhw, const uint32_t *__restrict__ bitmap, int64_t d, float beta1, float omb1,
          float beta2, float omb2, float rho)
{
    const int64_t l0 = (blockIdx.x * (int64_t)blockDim.x + threadIdx.x) * VEC;
    if (l0 >= d) return;
    const int64_t off = (int64_t)blockIdx.y * d + l0;
    const uint32_t selbits = (bitmap[l0 >> 5] >> (l0 & 31)) & (VEC == 4 ? 0xFu : 1u);
    float gv[VEC], mv[VEC], ev[VEC], vv[VEC], vh[VEC];
    if (VEC == 4) {
        const float4 a = *reinterpret_cast<const float4 *>(g + off), b = *reinterpret_cast<const float4 *>(m + off),
                     cc = *reinterpret_cast<const float4 *>(e + off), p = *reinterpret_cast<const float4 *>(vw + off),
                     q = *reinterpret_cast<const float4 *>(vhw + off);
        gv[0] = a.x; gv[1] = a.y; gv[2] = a.z; gv[3] = a.w;
        mv[0] = b.x; mv[1] = b.y; mv[2] = b.z; mv[3] = b.w;
        ev[0] = cc.x; ev[1] = cc.y; ev[2] = cc.z; ev[3] = cc.w;
        vv[0] = p.x; vv[1] = p.y; vv[2] = p.z; vv[3] = p.w;
        vh[0] = q.x; vh[1] = q.y; vh[2] = q.z; vh[3] = q.w;
    } else {
        gv[0] = g[off]; mv[0] = m[off]; ev[0] = e[off]; vv[0] = vw[off]; vh[0] = vhw[off];
    }
#pragma unroll
    for (int t = 0; t < VEC; ++t) {
        const float mm = (beta1 * mv[t]) + (omb1 * gv[t]);
        const float v2 = (beta2 * vv[t]) + (omb2 * (gv[t] * gv[t]));
        const float ein = ((selbits >> t) & 1u) ? 0.0f : ev[t];
        mv[t] = mm;
        vv[t] = v2;
        if (v2 > vh[t]) vh[t] = v2;
        ev[t] = (mm / sqrtf(vh[t])) + (rho * ein);
    }
    if (VEC == 4) {
        *reinterpret_cast<float4 *>(m + off) = make_float4(mv[0], mv[1], mv[2], mv[3]);
        *reinterpret_cast<float4 *>(e + off) = make_float4(ev[0], ev[1], ev[2], ev[3]);
        *reinterpret_cast<float4 *>(vw + off) = make_float4(vv[0], vv[1], vv[2], vv[3]);
        *reinterpret_cast<float4 *>(vhw + off) = make_float4(vh[0], vh[1], vh[2], vh[3]);
    } else {
        m[off] = mv[0]; e[off] = ev[0]; vw[off] = vv[0]; vhw[off] = vh[0];
    }
}

int enqueue_head_pa(sams_ctx *ctx, const float *g, float *m, float *e_u, float *v_w, float *vhat_w, float beta1,
                    float beta2, float rho)
{
    const int64_t d = ctx->d;
    const float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
    if ((d & 3) == 0) {
        ProfScope ps(ctx, KID_HEAD_PA);
        hipLaunchKernelGGL(k_head_pa<4>, dim3((unsigned)grid_for(d / 4, 256), (unsigned)ctx->n), dim3(256), 0,
                           ctx->stream, g, m, e_u, v_w, vhat_w, ctx->bitmap, d, beta1, omb1, beta2, omb2, rho);
    } else {
        ProfScope ps(ctx, KID_HEAD_PA);
        hipLaunchKernelGGL(k_head_pa<1>, dim3((unsigned)grid_for(d, 256), (unsigned)ctx->n), dim3(256), 0,
                           ctx->stream, g, m, e_u, v_w, vhat_w, ctx->bitmap, d, beta1, omb1, beta2, omb2, rho);
    }
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

int enqueue_tail(sams_ctx *ctx, float *e_u, float *x, const int32_t *idx, const float *delta,
                 int64_t k_sel, float lr, bool zero_e)
{
    const int64_t words = (ctx->d + 31) / 32;
    SAMS_TRY(enqueue_fill_u32(ctx, ctx->bitmap, words, 0u));
    if (k_sel > 0) {
        SAMS_LAUNCH(ctx, KID_TAIL_X, k_tail_x, grid_for(k_sel, 256), 256, idx, delta, k_sel, lr, x,
                    ctx->bitmap, ctx->wordrank);
        if (zero_e)
            SAMS_LAUNCH(ctx, KID_TAIL_ZERO_E, k_tail_zero_e, grid_for(k_sel, 256), 256, idx, k_sel,
                        ctx->n, ctx->d, e_u);
    }
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

int enqueue_head(sams_ctx *ctx, const float *g, float *m, float *e_u, float *v, float *vhat,
                 float beta1, float beta2, float rho)
{
    const int64_t d = ctx->d;
    const float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
    if ((d & 3) == 0) {
        SAMS_LAUNCH(ctx, KID_HEAD, (k_head<4>), grid_for(d / 4, 256), 256, g, m, e_u, v, vhat,
                    ctx->bitmap, ctx->n, d, beta1, omb1, beta2, omb2, rho);
    } else {
        SAMS_LAUNCH(ctx, KID_HEAD, (k_head<1>), grid_for(d, 256), 256, g, m, e_u, v, vhat, ctx->bitmap,
                    ctx->n, d, beta1, omb1, beta2, omb2, rho);
    }
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

int enqueue_reduce(sams_ctx *ctx, const float *S_workers, float *S_mean)
{
    const int64_t rc = (int64_t)ctx->r * ctx->c;
    if ((rc & 3) == 0)
        SAMS_LAUNCH(ctx, KID_REDUCE, k_reduce<4>, grid_for(rc / 4, 256, 1 << 16), 256, S_workers, S_mean, ctx->n, rc);
    else
        SAMS_LAUNCH(ctx, KID_REDUCE, k_reduce<1>, grid_for(rc, 256, 1 << 16), 256, S_workers, S_mean, ctx->n, rc);
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

int enqueue_gather(sams_ctx *ctx, const float *u, const float *vhat, const int32_t *idx,
                   float *U_workers, float *delta)
{
    if (ctx->n >= kWideMinWorkers)
        SAMS_LAUNCH(ctx, KID_GATHER, k_gather_wide, (unsigned)((ctx->k + kWideCoords - 1) / kWideCoords), 256, u, vhat,
                    idx, ctx->k, ctx->n, ctx->d, U_workers, delta);
    else
        SAMS_LAUNCH(ctx, KID_GATHER, k_gather, grid_for(ctx->k, 256), 256, u, vhat, idx, ctx->k, ctx->n,
                    ctx->d, U_workers, delta);
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

}  // namespace sams
