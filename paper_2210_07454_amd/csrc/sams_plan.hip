// Binned Count Sketch accumulation (stage 1 of sams.h; Sec. II-C update rule) for tables that do not
// fit in LDS.
//
// The bucket hash sends consecutive coordinates to buckets spread over the whole row, so a direct
// implementation is one uncoalesced read-modify-write per (worker, row, coordinate).  Because the
// hashes never change, the permutation "coordinate order -> bucket order" is fixed, and it is worked
// out once, at context creation (the plan):
//   * coordinates are cut into tiles of L = 2^tile_log2; a row's buckets into windows ("bins") of
//     W = 2^win_log2 buckets that fit in LDS;
//   * inside every (row, tile) the coordinates are sorted by (bin, coordinate).  src[row][tile*L+p]
//     names the coordinate (and its sign) that sorted position p takes, wlow[...] its bucket inside
//     the window, and bst[row][bin][tile] the first sorted position of each bin.
// Per step, pass 1 (k_bin_scatter) streams each worker's vector through LDS once and writes, for every
// row, the signed values in sorted order (fully coalesced stores); pass 2 (k_bin_accumulate) gives one
// workgroup per (worker, row, bin): it reads that bin's short runs from every tile (coalesced), adds
// them into its LDS window with LDS atomics, and writes the finished window once.  No global atomics,
// no zero-fill of the output, and every table cell is written exactly once.
#include "sams_ctx.h"

#pragma clang fp contract(off)

namespace sams {

constexpr int kPlanThreads = 1024;
constexpr int kScatterThreads = 256;
constexpr int kAccThreads = 1024;
constexpr int kNumXcd = 8;

// ------------------------------------------------------------------------------------------
// plan construction: one workgroup per (row, tile); bitonic sort of L keys in LDS
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kPlanThreads)
k_plan_build(HashParams hp, int64_t d, int tile_log2, int win_log2, int64_t nbins, int64_t ntile,
             int64_t dpad, uint16_t *__restrict__ src, uint16_t *__restrict__ wlow,
             uint16_t *__restrict__ bst)
{
    extern __shared__ uint32_t keys[];
    const int L = 1 << tile_log2;
    const int64_t tile = blockIdx.x;
    const int j = blockIdx.y;
    const int64_t l0 = tile << tile_log2;
    for (int p = threadIdx.x; p < L; p += blockDim.x) {
        int64_t l = l0 + p;
        uint32_t key = 0xffffffffu;                                 // beyond d: sorts last
        if (l < d) {
            uint32_t bin = bucket_of(hp, j, (uint32_t)l) >> win_log2;
            key = (bin << tile_log2) | (uint32_t)p;
        }
        keys[p] = key;
    }
    __syncthreads();
    for (int k = 2; k <= L; k <<= 1) {
        for (int jj = k >> 1; jj > 0; jj >>= 1) {
            for (int t = threadIdx.x; t < L; t += blockDim.x) {
                int other = t ^ jj;
                if (other > t) {
                    uint32_t a = keys[t], b = keys[other];
                    bool up = (t & k) == 0;
                    if ((a > b) == up) {
                        keys[t] = b;
                        keys[other] = a;
                    }
                }
            }
            __syncthreads();
        }
    }
    const uint32_t lmask = (uint32_t)L - 1u, wmask = (1u << win_log2) - 1u;
    for (int p = threadIdx.x; p < L; p += blockDim.x) {
        uint32_t key = keys[p];
        uint16_t s = 0, w = 0;
        if (key != 0xffffffffu) {
            uint32_t loc = key & lmask;
            uint32_t l = (uint32_t)(l0 + loc);
            s = (uint16_t)(loc | (sign_neg(hp, j, l) ? 0x8000u : 0u));
            w = (uint16_t)(bucket_of(hp, j, l) & wmask);
        }
        src[(int64_t)j * dpad + l0 + p] = s;
        wlow[(int64_t)j * dpad + l0 + p] = w;
    }
    // first sorted position of every bin (bin == nbins: one past the last real coordinate)
    for (int64_t b = threadIdx.x; b <= nbins; b += blockDim.x) {
        uint32_t want = (uint32_t)b << tile_log2;                   // smallest key of bin b
        int lo = 0, hi = L;
        while (lo < hi) {
            int mid = (lo + hi) >> 1;
            uint32_t key = keys[mid];
            bool less = key != 0xffffffffu && key < want;
            if (b == nbins) less = key != 0xffffffffu;
            if (less) lo = mid + 1; else hi = mid;
        }
        bst[((int64_t)j * (nbins + 1) + b) * ntile + tile] = (uint16_t)lo;
    }
}

// ------------------------------------------------------------------------------------------
// pass 1: per tile, every worker's values into per-row sorted order
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kScatterThreads)
k_bin_scatter(const float *__restrict__ u, const uint16_t *__restrict__ src, float *__restrict__ stg,
              int32_t n, int32_t r, int64_t d, int tile_log2, int64_t dpad)
{
    extern __shared__ float tilebuf[];
    const int L = 1 << tile_log2;
    const int64_t l0 = (int64_t)blockIdx.x << tile_log2;
    const bool vec = (d & 3) == 0;
    for (int32_t i = 0; i < n; ++i) {
        const float *ui = u + (int64_t)i * d;
        if (vec) {
            for (int p = threadIdx.x * 4; p < L; p += blockDim.x * 4) {
                float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
                if (l0 + p < d) q = *reinterpret_cast<const float4 *>(ui + l0 + p);
                *reinterpret_cast<float4 *>(tilebuf + p) = q;
            }
        } else {
            for (int p = threadIdx.x; p < L; p += blockDim.x) tilebuf[p] = (l0 + p < d) ? ui[l0 + p] : 0.f;
        }
        __syncthreads();
        for (int32_t j = 0; j < r; ++j) {
            const uint16_t *sj = src + (int64_t)j * dpad + l0;
            float *oj = stg + ((int64_t)i * r + j) * dpad + l0;
            for (int p = threadIdx.x * 4; p < L; p += blockDim.x * 4) {
                uint2 packed = *reinterpret_cast<const uint2 *>(sj + p);
                uint32_t s0 = packed.x & 0xffffu, s1 = packed.x >> 16, s2 = packed.y & 0xffffu,
                         s3 = packed.y >> 16;
                float4 o;
                o.x = tilebuf[s0 & 0x7fffu]; o.x = (s0 & 0x8000u) ? -o.x : o.x;
                o.y = tilebuf[s1 & 0x7fffu]; o.y = (s1 & 0x8000u) ? -o.y : o.y;
                o.z = tilebuf[s2 & 0x7fffu]; o.z = (s2 & 0x8000u) ? -o.z : o.z;
                o.w = tilebuf[s3 & 0x7fffu]; o.w = (s3 & 0x8000u) ? -o.w : o.w;
                *reinterpret_cast<float4 *>(oj + p) = o;
            }
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------
// pass 2: per (worker, row, bin), add the bin's runs of every tile into an LDS window
// ------------------------------------------------------------------------------------------
// Workgroup ids are dealt round-robin to the 8 XCDs; the mapping below places the n workers of one
// (row, bin) on the same XCD in consecutive slots, so that the shared wlow/bst metadata is read from
// HBM once and then served by that XCD's L2.
__global__ void __launch_bounds__(kAccThreads)
k_bin_accumulate(const float *__restrict__ stg, const uint16_t *__restrict__ wlow,
                 const uint16_t *__restrict__ bst, float *__restrict__ S, int32_t n, int32_t r, int64_t c,
                 int win_log2, int64_t nbins, int64_t ntile, int tile_log2, int64_t dpad)
{
    extern __shared__ float win[];
    const int W = 1 << win_log2;
    const int64_t id = blockIdx.x;
    const int64_t slot = id / kNumXcd;
    const int64_t group = (id % kNumXcd) + kNumXcd * (slot / n);     // (row, bin) index
    const int32_t i = (int32_t)(slot % n);
    if (group >= (int64_t)r * nbins) return;
    const int32_t j = (int32_t)(group / nbins);
    const int64_t bin = group % nbins;
    for (int t = threadIdx.x; t < W; t += blockDim.x) win[t] = 0.f;
    __syncthreads();
    const uint16_t *st0 = bst + ((int64_t)j * (nbins + 1) + bin) * ntile;
    const uint16_t *st1 = st0 + ntile;
    const float *vbase = stg + ((int64_t)i * r + j) * dpad;
    const uint16_t *wbase = wlow + (int64_t)j * dpad;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave, nwave = blockDim.x / kWave;
    for (int64_t t0 = (int64_t)wave * kWave; t0 < ntile; t0 += (int64_t)nwave * kWave) {
        // each lane fetches the run bounds of one tile; the wavefront then walks the 64 runs together
        const int64_t tl = t0 + lane;
        int a_l = 0, b_l = 0;
        if (tl < ntile) { a_l = st0[tl]; b_l = st1[tl]; }
        const int cnt = (ntile - t0) < kWave ? (int)(ntile - t0) : kWave;
        for (int q = 0; q < cnt; q += 4) {
            float v[4];
            uint32_t w[4];
            bool ok[4];
            int rest = 0;
#pragma unroll
            for (int z = 0; z < 4; ++z) {
                const int a = __shfl(a_l, (q + z) & (kWave - 1)), b = __shfl(b_l, (q + z) & (kWave - 1));
                const int pos = a + lane;
                ok[z] = (q + z < cnt) && pos < b;
                const int64_t off = ((t0 + q + z) << tile_log2) + pos;
                v[z] = ok[z] ? vbase[off] : 0.f;
                w[z] = ok[z] ? wbase[off] : 0u;
                rest |= (q + z < cnt) && (a + kWave < b);
            }
#pragma unroll
            for (int z = 0; z < 4; ++z)
                if (ok[z]) atomicAdd(&win[w[z]], v[z]);
            if (__any(rest)) {                                       // runs longer than one wavefront
                for (int z = 0; z < 4 && q + z < cnt; ++z) {
                    const int a = __shfl(a_l, q + z), b = __shfl(b_l, q + z);
                    for (int pos = a + kWave + lane; pos < b; pos += kWave) {
                        const int64_t off = ((t0 + q + z) << tile_log2) + pos;
                        atomicAdd(&win[wbase[off]], vbase[off]);
                    }
                }
            }
        }
    }
    __syncthreads();
    const int64_t b0 = bin << win_log2;
    float *out = S + ((int64_t)i * r + j) * c + b0;
    const int64_t lim = (c - b0) < W ? (c - b0) : W;
    for (int t = threadIdx.x; t < lim; t += blockDim.x) out[t] = win[t];
}

// ------------------------------------------------------------------------------------------
// small tables: the whole row fits in LDS; accumulate there, then add the partial rows to memory
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_sketch_lds(const float *__restrict__ u, float *__restrict__ S, HashParams hp, int32_t n, int64_t d,
             int64_t c, int64_t chunk)
{
    extern __shared__ float row[];
    const int32_t i = blockIdx.z, j = blockIdx.y;
    for (int t = threadIdx.x; t < c; t += blockDim.x) row[t] = 0.f;
    __syncthreads();
    const int64_t lo = blockIdx.x * chunk, hi = (lo + chunk) < d ? (lo + chunk) : d;
    const float *ui = u + (int64_t)i * d;
    for (int64_t l = lo + threadIdx.x; l < hi; l += blockDim.x) {
        float val = ui[l];
        uint32_t b = bucket_of(hp, j, (uint32_t)l);
        atomicAdd(&row[b], sign_neg(hp, j, (uint32_t)l) ? -val : val);
    }
    __syncthreads();
    float *out = S + ((int64_t)i * hp.r + j) * c;
    for (int t = threadIdx.x; t < c; t += blockDim.x) {
        float val = row[t];
        if (val != 0.f) atomicAdd(&out[t], val);
    }
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
int plan_create(sams_ctx *ctx, int tile_log2, int win_log2)
{
    Plan &pl = ctx->plan;
    pl.win_log2 = win_log2;
    pl.tile_log2 = tile_log2;
    const int64_t W = (int64_t)1 << win_log2, L = (int64_t)1 << tile_log2;
    pl.nbins = (ctx->c + W - 1) / W;
    pl.mode = pl.nbins <= 1 ? PLAN_LDS_ROW : PLAN_BINNED;
    if (pl.mode == PLAN_LDS_ROW) {
        SAMS_HIP(hipFuncSetAttribute((const void *)k_sketch_lds, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)(W * 4)));
        return SAMS_OK;
    }
    if ((pl.nbins << tile_log2) >= ((int64_t)1 << 32) - 1) return SAMS_EINVAL;   // sort key must fit 32 bits
    pl.ntile = (ctx->d + L - 1) / L;
    pl.dpad = pl.ntile * L;
    const int64_t r = ctx->r, n = ctx->n;
    struct { void **p; int64_t bytes; } allocs[] = {
        {(void **)&pl.src, r * pl.dpad * 2},
        {(void **)&pl.wlow, r * pl.dpad * 2},
        {(void **)&pl.bst, r * (pl.nbins + 1) * pl.ntile * 2},
        {(void **)&pl.stg, n * r * pl.dpad * 4},
    };
    for (auto &a : allocs) {
        hipError_t e = hipMalloc(a.p, (size_t)a.bytes);
        if (e != hipSuccess) {
            g_last_hip_error = (int)e;
            (void)hipGetLastError();
            return SAMS_ENOMEM;
        }
        ctx->scratch_bytes += a.bytes;
    }
    SAMS_HIP(hipFuncSetAttribute((const void *)k_plan_build, hipFuncAttributeMaxDynamicSharedMemorySize,
                                 (int)(L * 4)));
    SAMS_HIP(hipFuncSetAttribute((const void *)k_bin_scatter, hipFuncAttributeMaxDynamicSharedMemorySize,
                                 (int)(L * 4)));
    SAMS_HIP(hipFuncSetAttribute((const void *)k_bin_accumulate,
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)(W * 4)));
    {
        ProfScope ps(ctx, KID_PLAN_BUILD);
        hipLaunchKernelGGL(k_plan_build, dim3((unsigned)pl.ntile, (unsigned)r), dim3(kPlanThreads),
                           (size_t)(L * 4), ctx->stream, ctx->hp, ctx->d, tile_log2, win_log2, pl.nbins,
                           pl.ntile, pl.dpad, pl.src, pl.wlow, pl.bst);
    }
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

void plan_destroy(sams_ctx *ctx)
{
    Plan &pl = ctx->plan;
    void *ptrs[] = {pl.src, pl.wlow, pl.bst, pl.stg};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    pl.src = pl.wlow = pl.bst = nullptr;
    pl.stg = nullptr;
}

int enqueue_sketch_planned(sams_ctx *ctx, const float *u, float *S_workers)
{
    Plan &pl = ctx->plan;
    if (pl.mode == PLAN_LDS_ROW) {
        const int64_t cells = (int64_t)ctx->n * ctx->r * ctx->c;
        SAMS_TRY(enqueue_fill_u32(ctx, (uint32_t *)S_workers, cells, 0u));
        // enough chunks to fill the chip, few enough that the final global adds stay negligible
        int64_t nchunk = 2048 / ((int64_t)ctx->n * ctx->r);
        if (nchunk < 1) nchunk = 1;
        const int64_t maxchunk = (ctx->d + 4095) / 4096;
        if (nchunk > maxchunk) nchunk = maxchunk;
        const int64_t chunk = (ctx->d + nchunk - 1) / nchunk;
        ProfScope ps(ctx, KID_SKETCH_LDS);
        hipLaunchKernelGGL(k_sketch_lds, dim3((unsigned)nchunk, (unsigned)ctx->r, (unsigned)ctx->n),
                           dim3(256), (size_t)(ctx->c * 4), ctx->stream, u, S_workers, ctx->hp, ctx->n,
                           ctx->d, ctx->c, chunk);
        SAMS_HIP(hipGetLastError());
        return SAMS_OK;
    }
    const int64_t L = (int64_t)1 << pl.tile_log2, W = (int64_t)1 << pl.win_log2;
    {
        ProfScope ps(ctx, KID_BIN_SCATTER);
        hipLaunchKernelGGL(k_bin_scatter, dim3((unsigned)pl.ntile), dim3(kScatterThreads), (size_t)(L * 4),
                           ctx->stream, u, pl.src, pl.stg, ctx->n, ctx->r, ctx->d, pl.tile_log2, pl.dpad);
    }
    SAMS_HIP(hipGetLastError());
    {
        const int64_t groups = (int64_t)ctx->r * pl.nbins;
        const int64_t gpad = (groups + kNumXcd - 1) / kNumXcd * kNumXcd;
        ProfScope ps(ctx, KID_BIN_ACCUMULATE);
        hipLaunchKernelGGL(k_bin_accumulate, dim3((unsigned)(gpad * ctx->n)), dim3(kAccThreads),
                           (size_t)(W * 4), ctx->stream, pl.stg, pl.wlow, pl.bst, S_workers, ctx->n, ctx->r,
                           ctx->c, pl.win_log2, pl.nbins, pl.ntile, pl.tile_log2, pl.dpad);
    }
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

}  // namespace sams
