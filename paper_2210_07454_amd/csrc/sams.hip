// MI355X (gfx950) implementation of the C ABI declared in include/sams.h: the per-step
// compression-plus-update pipeline of SketchedAMSGrad with gradient averaging (Alg. 2 of
// arXiv 2210.07454).  Build with -ffp-contract=off: the update formulas are evaluated as
// separate IEEE multiplies and adds, in the order sams.h writes them.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <new>

#include "../../include/sams.h"
#include "sams_hash.h"

// Every formula below is evaluated as separate IEEE-754 binary32 operations, rounded to nearest:
// no fused multiply-add is formed (here and with -ffp-contract=off on the command line), and
// x / y and sqrtf(x) are the correctly rounded ones (hipcc's default; never build this file with
// -ffast-math or -fno-hip-fp32-correctly-rounded-divide-sqrt).
#pragma clang fp contract(off)

namespace sams {

static int g_last_hip_error = 0;

#define SAMS_HIP(expr)                                  \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) {                         \
            g_last_hip_error = (int)e_;                 \
            return SAMS_EHIP;                           \
        }                                               \
    } while (0)

constexpr int kWave = 64;
constexpr int kSelTile = 2048;      // coordinates one wavefront compacts in the selection
constexpr int kHistBins = 2048;     // first radix digit: 11 bits, then 10 and 10
constexpr int kSelPasses = 3;

// device-resident state of the radix selection (no host round trip inside a step)
struct SelState {
    uint32_t prefix;   // key bits decided so far (top bits of the k-th largest |est| pattern)
    uint32_t k_rem;    // how many keys to take among those matching the prefix
    uint32_t tau;      // final: the 31-bit pattern of the k-th largest |est|
    uint32_t k_eq;     // final: how many coordinates with |est| == tau are selected (smallest indices)
};

}  // namespace sams

struct sams_ctx {
    int64_t d, c, k;
    int32_t n, r;
    hipStream_t stream;
    sams::HashParams hp;
    // scratch
    float *est;              // [d]
    uint32_t *bitmap;        // [ceil(d/32)]  bit l set <=> l in the most recent index set
    uint32_t *hist;          // [kHistBins]
    sams::SelState *sel;     // [1]
    uint32_t *cnt;           // [2][ntile]  per-wavefront-tile counts: greater, equal
    uint32_t *base;          // [2][ntile]  exclusive prefix: selected before, equal before
    int64_t ntile;
    int64_t scratch_bytes;
};

namespace sams {

// ------------------------------------------------------------------------------------------
// small utilities
// ------------------------------------------------------------------------------------------
__global__ void k_fill_u32(uint32_t *p, int64_t n, uint32_t val)
{
    int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    int64_t st = (int64_t)gridDim.x * blockDim.x;
    for (; i < n; i += st) p[i] = val;
}

static inline int grid_for(int64_t work, int block, int64_t cap = (int64_t)1 << 20)
{
    int64_t g = (work + block - 1) / block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
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

// ------------------------------------------------------------------------------------------
// stage 5: tail (finish iteration t) and head (start iteration t+1) of Alg. 2
// ------------------------------------------------------------------------------------------
// x[idx[q]] -= lr * delta[q]; mark idx[q] in the bitmap (I_t for the next head)
__global__ void k_tail_x(const int32_t *__restrict__ idx, const float *__restrict__ delta, int64_t k,
                         float lr, float *__restrict__ x, uint32_t *__restrict__ bitmap)
{
    int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q >= k) return;
    uint32_t l = (uint32_t)idx[q];
    x[l] = (x[l] - (lr * delta[q]));
    atomicOr(&bitmap[l >> 5], 1u << (l & 31));
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

// ------------------------------------------------------------------------------------------
// stage 2: mean of the worker sketches (Alg. 2, master)
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_reduce(const float *__restrict__ S_w, float *__restrict__ S_mean, int32_t n, int64_t rc)
{
    int64_t t = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    int64_t st = (int64_t)gridDim.x * blockDim.x;
    float fn = (float)n;
    for (; t < rc; t += st) {
        float acc = S_w[t];
        for (int32_t i = 1; i < n; ++i) acc = (acc + S_w[(int64_t)i * rc + t]);
        S_mean[t] = (acc / fn);
    }
}

// ------------------------------------------------------------------------------------------
// stage 3a: per-coordinate estimates (Sec. II-C median, Alg. 3 scaling)
// ------------------------------------------------------------------------------------------
template <int R>
__device__ __forceinline__ float median_of(float (&a)[R])
{
    // odd-even transposition network: R rounds sort R values; compile-time unrolled
#pragma unroll
    for (int round = 0; round < R; ++round) {
#pragma unroll
        for (int p = (round & 1); p + 1 < R; p += 2) {
            float lo = a[p + 1] < a[p] ? a[p + 1] : a[p];
            float hi = a[p + 1] < a[p] ? a[p] : a[p + 1];
            a[p] = lo;
            a[p + 1] = hi;
        }
    }
    return a[(R - 1) / 2];
}

template <int R>
__global__ void __launch_bounds__(256)
k_estimate(const float *__restrict__ S, const float *__restrict__ vhat, float *__restrict__ est,
           HashParams hp, int64_t d, int64_t c)
{
    int64_t l = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (l >= d) return;
    float a[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        uint32_t b = bucket_of(hp, j, (uint32_t)l);
        float q = S[(int64_t)j * c + b];
        a[j] = sign_neg(hp, j, (uint32_t)l) ? -q : q;
    }
    float med = median_of<R>(a);
    est[l] = vhat ? (med / sqrtf(vhat[l])) : med;
}

// ------------------------------------------------------------------------------------------
// stage 3b: exact top-k of |est| by radix selection on the 31-bit magnitude pattern
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t mag_key(float x) { return __float_as_uint(x) & 0x7fffffffu; }

__device__ __forceinline__ int sel_shift(int pass) { return pass == 0 ? 20 : (pass == 1 ? 10 : 0); }
__device__ __forceinline__ int sel_width(int pass) { return pass == 0 ? 11 : 10; }

__global__ void k_sel_init(SelState *st, uint32_t k, uint32_t *hist)
{
    for (int t = threadIdx.x; t < kHistBins; t += blockDim.x) hist[t] = 0;
    if (threadIdx.x == 0) {
        st->prefix = 0;
        st->k_rem = k;
        st->tau = 0;
        st->k_eq = 0;
    }
}

// histogram of the current digit over the keys whose higher digits equal the prefix
__global__ void __launch_bounds__(256)
k_sel_hist(const float *__restrict__ est, int64_t d, int pass, const SelState *__restrict__ st,
           uint32_t *__restrict__ hist)
{
    __shared__ uint32_t lh[kHistBins];
    for (int t = threadIdx.x; t < kHistBins; t += blockDim.x) lh[t] = 0;
    __syncthreads();
    const int shift = sel_shift(pass), width = sel_width(pass);
    const uint32_t prefix = st->prefix;
    const uint32_t dmask = (1u << width) - 1u;
    int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < d; i += stride) {
        uint32_t key = mag_key(est[i]);
        if ((key >> (shift + width)) == prefix) atomicAdd(&lh[(key >> shift) & dmask], 1u);
    }
    __syncthreads();
    for (int t = threadIdx.x; t < kHistBins; t += blockDim.x)
        if (lh[t]) atomicAdd(&hist[t], lh[t]);
}

// choose the digit in which the k_rem-th largest key lies; clear the histogram for the next pass
__global__ void k_sel_pick(SelState *st, uint32_t *hist, int pass)
{
    __shared__ uint32_t lh[kHistBins];
    const int nb = 1 << sel_width(pass);
    for (int t = threadIdx.x; t < kHistBins; t += blockDim.x) {
        lh[t] = hist[t];
        hist[t] = 0;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t k_rem = st->k_rem, cum = 0;
        int b = nb - 1;
        for (; b > 0; --b) {
            if (cum + lh[b] >= k_rem) break;
            cum += lh[b];
        }
        uint32_t prefix = (st->prefix << sel_width(pass)) | (uint32_t)b;
        st->prefix = prefix;
        st->k_rem = k_rem - cum;
        if (pass == kSelPasses - 1) {
            st->tau = prefix;
            st->k_eq = k_rem - cum;
        }
    }
}

// per wavefront tile of kSelTile consecutive coordinates: how many keys exceed tau, how many equal it
__global__ void __launch_bounds__(256)
k_sel_count(const float *__restrict__ est, int64_t d, const SelState *__restrict__ st,
            uint32_t *__restrict__ cnt_gt, uint32_t *__restrict__ cnt_eq, int64_t ntile)
{
    const int lane = threadIdx.x & (kWave - 1);
    int64_t tile = blockIdx.x * (int64_t)(blockDim.x / kWave) + (threadIdx.x / kWave);
    if (tile >= ntile) return;
    const uint32_t tau = st->tau;
    int64_t base = tile * kSelTile;
    uint32_t ngt = 0, neq = 0;
    for (int s = 0; s < kSelTile; s += kWave) {
        int64_t l = base + s + lane;
        uint32_t key = l < d ? mag_key(est[l]) : 0u;
        bool gt = l < d && key > tau, eq = l < d && key == tau;
        ngt += (uint32_t)__popcll(__ballot(gt));
        neq += (uint32_t)__popcll(__ballot(eq));
    }
    if (lane == 0) {
        cnt_gt[tile] = ngt;
        cnt_eq[tile] = neq;
    }
}

// single block: exclusive prefixes over the tiles.  eq_base = equal keys before the tile;
// sel_base = selected coordinates before the tile, where a tile contributes all its greater keys
// and as many of its equal keys as are still wanted (k_eq counted from the smallest index).
__global__ void __launch_bounds__(1024)
k_sel_scan(const uint32_t *__restrict__ cnt_gt, const uint32_t *__restrict__ cnt_eq, int64_t ntile,
           const SelState *__restrict__ st, uint32_t *__restrict__ sel_base,
           uint32_t *__restrict__ eq_base)
{
    __shared__ uint32_t part[1024];
    const int T = blockDim.x, t = threadIdx.x;
    const int64_t per = (ntile + T - 1) / T;
    const int64_t lo = (int64_t)t * per, hi = lo + per < ntile ? lo + per : ntile;
    const uint32_t k_eq = st->k_eq;
    // pass A: equal counts
    uint32_t s = 0;
    for (int64_t q = lo; q < hi; ++q) s += cnt_eq[q];
    part[t] = s;
    __syncthreads();
    if (t == 0) {
        uint32_t run = 0;
        for (int q = 0; q < T; ++q) { uint32_t x = part[q]; part[q] = run; run += x; }
    }
    __syncthreads();
    uint32_t run = part[t];
    __syncthreads();
    uint32_t s2 = 0;
    for (int64_t q = lo; q < hi; ++q) {
        eq_base[q] = run;
        uint32_t want = run < k_eq ? k_eq - run : 0u;
        uint32_t ce = cnt_eq[q];
        s2 += cnt_gt[q] + (ce < want ? ce : want);
        run += ce;
    }
    // pass B: selected counts
    part[t] = s2;
    __syncthreads();
    if (t == 0) {
        uint32_t r2 = 0;
        for (int q = 0; q < T; ++q) { uint32_t x = part[q]; part[q] = r2; r2 += x; }
    }
    __syncthreads();
    uint32_t run2 = part[t];
    for (int64_t q = lo; q < hi; ++q) {
        sel_base[q] = run2;
        uint32_t eb = eq_base[q];
        uint32_t want = eb < k_eq ? k_eq - eb : 0u;
        uint32_t ce = cnt_eq[q];
        run2 += cnt_gt[q] + (ce < want ? ce : want);
    }
}

// ordered compaction: every wavefront walks its tile in index order and writes the selected
// coordinates (key > tau, or key == tau and among the first k_eq such coordinates) at their rank
__global__ void __launch_bounds__(256)
k_sel_write(const float *__restrict__ est, int64_t d, const SelState *__restrict__ st,
            const uint32_t *__restrict__ sel_base, const uint32_t *__restrict__ eq_base,
            int64_t ntile, int64_t k, int32_t *__restrict__ idx, float *__restrict__ est_sel)
{
    const int lane = threadIdx.x & (kWave - 1);
    int64_t tile = blockIdx.x * (int64_t)(blockDim.x / kWave) + (threadIdx.x / kWave);
    if (tile >= ntile) return;
    const uint32_t tau = st->tau, k_eq = st->k_eq;
    int64_t base = tile * kSelTile;
    uint32_t out = sel_base[tile], eqr = eq_base[tile];
    const uint64_t below = ((uint64_t)1 << lane) - 1;
    for (int s = 0; s < kSelTile; s += kWave) {
        int64_t l = base + s + lane;
        float val = l < d ? est[l] : 0.0f;
        uint32_t key = mag_key(val);
        bool gt = l < d && key > tau, eq = l < d && key == tau;
        uint64_t meq = __ballot(eq);
        bool take = gt || (eq && eqr + (uint32_t)__popcll(meq & below) < k_eq);
        uint64_t msel = __ballot(take);
        if (take) {
            int64_t pos = (int64_t)out + __popcll(msel & below);
            if (pos < k) {
                idx[pos] = (int32_t)l;
                if (est_sel) est_sel[pos] = val;
            }
        }
        out += (uint32_t)__popcll(msel);
        eqr += (uint32_t)__popcll(meq);
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
    for (int32_t i = 0; i < n; ++i) {
        float val = u[(int64_t)i * d + l];
        U_w[(int64_t)i * k + q] = val;
        acc = (i == 0) ? val : (acc + val);
    }
    float mean = (acc / (float)n);
    delta[q] = vhat ? (mean / sqrtf(vhat[l])) : mean;
}

static inline bool aligned16(const void *p) { return (((uintptr_t)p) & 15u) == 0; }

static int launch_estimate(sams_ctx *ctx, const float *S_mean, const float *vhat, float *est)
{
    const int block = 256;
    const int grid = grid_for(ctx->d, block, (int64_t)1 << 30);
    switch (ctx->r) {
#define SAMS_CASE(R)                                                                               \
    case R:                                                                                        \
        hipLaunchKernelGGL(k_estimate<R>, dim3(grid), dim3(block), 0, ctx->stream, S_mean, vhat,   \
                           est, ctx->hp, ctx->d, ctx->c);                                          \
        break;
        SAMS_CASE(1) SAMS_CASE(2) SAMS_CASE(3) SAMS_CASE(4) SAMS_CASE(5) SAMS_CASE(6) SAMS_CASE(7)
        SAMS_CASE(8) SAMS_CASE(9) SAMS_CASE(10) SAMS_CASE(11) SAMS_CASE(12) SAMS_CASE(13)
        SAMS_CASE(14) SAMS_CASE(15) SAMS_CASE(16)
#undef SAMS_CASE
    default:
        return SAMS_EINVAL;
    }
    SAMS_HIP(hipGetLastError());
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
    if (d < 1 || d >= (int64_t)kP31 || n < 1 || n > 1024 || r < 1 || r > SAMS_MAX_ROWS || c < 1 ||
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
    hipLaunchKernelGGL(k_fill_u32, dim3(grid_for(words, 256, 4096)), dim3(256), 0, ctx->stream,
                       ctx->bitmap, words, 0u);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        sams_destroy(ctx);
        return SAMS_EHIP;
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
    void *ptrs[] = {ctx->est, ctx->bitmap, ctx->hist, ctx->sel, ctx->cnt, ctx->base};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    delete ctx;
    return rc;
}

int64_t sams_scratch_bytes(const sams_ctx *ctx) { return ctx ? ctx->scratch_bytes : 0; }

int sams_hash_dump(sams_ctx *ctx, int32_t *bucket, int8_t *sign)
{
    if (!ctx || !bucket || !sign) return SAMS_EINVAL;
    hipLaunchKernelGGL(k_hash_dump, dim3(grid_for(ctx->d, 256, (int64_t)1 << 30)), dim3(256), 0,
                       ctx->stream, ctx->hp, ctx->d, bucket, sign);
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

int sketch_accumulate(sams_ctx *ctx, const float *u, float *S_workers)
{
    if (!ctx || !u || !S_workers || !aligned16(u) || !aligned16(S_workers)) return SAMS_EINVAL;
    const int64_t cells = (int64_t)ctx->n * ctx->r * ctx->c;
    hipLaunchKernelGGL(k_fill_u32, dim3(grid_for(cells, 256, 1 << 16)), dim3(256), 0, ctx->stream,
                       (uint32_t *)S_workers, cells, 0u);
    SAMS_HIP(hipGetLastError());
    hipLaunchKernelGGL(k_sketch_atomic, dim3(grid_for(ctx->d, 256, (int64_t)1 << 30)), dim3(256), 0,
                       ctx->stream, u, S_workers, ctx->hp, ctx->n, ctx->d, ctx->c);
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

int sketch_reduce(sams_ctx *ctx, const float *S_workers, float *S_mean)
{
    if (!ctx || !S_workers || !S_mean || !aligned16(S_workers) || !aligned16(S_mean)) return SAMS_EINVAL;
    const int64_t rc = (int64_t)ctx->r * ctx->c;
    hipLaunchKernelGGL(k_reduce, dim3(grid_for(rc, 256, 1 << 16)), dim3(256), 0, ctx->stream,
                       S_workers, S_mean, ctx->n, rc);
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

int unsketch_estimates(sams_ctx *ctx, const float *S_mean, const float *vhat, float *est)
{
    if (!ctx || !S_mean || !est || !aligned16(S_mean) || !aligned16(est) || !aligned16(vhat))
        return SAMS_EINVAL;
    return launch_estimate(ctx, S_mean, vhat, est);
}

int unsketch_topk(sams_ctx *ctx, const float *S_mean, const float *vhat, int32_t *idx, float *est_sel)
{
    if (!ctx || !S_mean || !idx || !aligned16(S_mean) || !aligned16(idx) || !aligned16(vhat) ||
        !aligned16(est_sel))
        return SAMS_EINVAL;
    int rc = launch_estimate(ctx, S_mean, vhat, ctx->est);
    if (rc != SAMS_OK) return rc;
    hipStream_t s = ctx->stream;
    const int64_t d = ctx->d, nt = ctx->ntile;
    uint32_t *cnt_gt = ctx->cnt, *cnt_eq = ctx->cnt + nt;
    uint32_t *sel_base = ctx->base, *eq_base = ctx->base + nt;
    hipLaunchKernelGGL(k_sel_init, dim3(1), dim3(256), 0, s, ctx->sel, (uint32_t)ctx->k, ctx->hist);
    for (int pass = 0; pass < kSelPasses; ++pass) {
        hipLaunchKernelGGL(k_sel_hist, dim3(grid_for(d, 256 * 16, 4096)), dim3(256), 0, s, ctx->est, d,
                           pass, ctx->sel, ctx->hist);
        hipLaunchKernelGGL(k_sel_pick, dim3(1), dim3(256), 0, s, ctx->sel, ctx->hist, pass);
    }
    const int waves_per_block = 256 / kWave;
    const int tgrid = (int)((nt + waves_per_block - 1) / waves_per_block);
    hipLaunchKernelGGL(k_sel_count, dim3(tgrid), dim3(256), 0, s, ctx->est, d, ctx->sel, cnt_gt, cnt_eq, nt);
    hipLaunchKernelGGL(k_sel_scan, dim3(1), dim3(1024), 0, s, cnt_gt, cnt_eq, nt, ctx->sel, sel_base,
                       eq_base);
    hipLaunchKernelGGL(k_sel_write, dim3(tgrid), dim3(256), 0, s, ctx->est, d, ctx->sel, sel_base, eq_base,
                       nt, ctx->k, idx, est_sel);
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

int gather_topk(sams_ctx *ctx, const float *u, const float *vhat, const int32_t *idx, float *U_workers,
                float *delta)
{
    if (!ctx || !u || !idx || !U_workers || !delta || !aligned16(u) || !aligned16(vhat) ||
        !aligned16(idx) || !aligned16(U_workers) || !aligned16(delta))
        return SAMS_EINVAL;
    hipLaunchKernelGGL(k_gather, dim3(grid_for(ctx->k, 256, (int64_t)1 << 30)), dim3(256), 0, ctx->stream,
                       u, vhat, idx, ctx->k, ctx->n, ctx->d, U_workers, delta);
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
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
    hipStream_t s = ctx->stream;
    const int64_t d = ctx->d, words = (d + 31) / 32;
    // tail of iteration t
    hipLaunchKernelGGL(k_fill_u32, dim3(grid_for(words, 256, 4096)), dim3(256), 0, s, ctx->bitmap, words, 0u);
    if (k_sel > 0) {
        hipLaunchKernelGGL(k_tail_x, dim3(grid_for(k_sel, 256, (int64_t)1 << 30)), dim3(256), 0, s, idx,
                           delta, k_sel, lr, x, ctx->bitmap);
        if (!g_next)
            hipLaunchKernelGGL(k_tail_zero_e, dim3(grid_for(k_sel, 256, (int64_t)1 << 30)), dim3(256), 0,
                               s, idx, k_sel, ctx->n, d, e_u);
    }
    SAMS_HIP(hipGetLastError());
    // head of iteration t+1
    if (g_next) {
        const float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
        if ((d & 3) == 0) {
            hipLaunchKernelGGL(k_head<4>, dim3(grid_for(d / 4, 256, (int64_t)1 << 30)), dim3(256), 0, s,
                               g_next, m, e_u, v, vhat, ctx->bitmap, ctx->n, d, beta1, omb1, beta2, omb2,
                               ef_ratio);
        } else {
            hipLaunchKernelGGL(k_head<1>, dim3(grid_for(d, 256, (int64_t)1 << 30)), dim3(256), 0, s,
                               g_next, m, e_u, v, vhat, ctx->bitmap, ctx->n, d, beta1, omb1, beta2, omb2,
                               ef_ratio);
        }
        SAMS_HIP(hipGetLastError());
    }
    return SAMS_OK;
}

}  // extern "C"
