// Internal header of the HIP library: the context, error plumbing, launch/timing helpers and the
// declarations of the per-stage enqueue functions (one .hip file per stage group).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sams.h"
#include "sams_hash.h"

namespace sams {

extern int g_last_hip_error;

#define SAMS_HIP(expr)                                  \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) {                         \
            ::sams::g_last_hip_error = (int)e_;         \
            return SAMS_EHIP;                           \
        }                                               \
    } while (0)

#define SAMS_TRY(expr)                                  \
    do {                                                \
        int rc_ = (expr);                               \
        if (rc_ != SAMS_OK) return rc_;                 \
    } while (0)

constexpr int kWave = 64;
constexpr int kSelTile = 8192;      // coordinates one wavefront compacts in the selection
constexpr int kHistBins = 2048;     // first radix digit: 11 bits, then 10 and 10
constexpr int kSelPasses = 3;
constexpr int kSelSmallSeg = 4096;   // keys per wavefront of the one-workgroup selection ...
constexpr int kSelSmallMax = 16 * kSelSmallSeg;   // ... which handles up to this many keys

// device-resident state of the radix selection (no host round trip inside a step)
struct SelState {
    uint32_t prefix;   // key bits decided so far (top bits of the k-th largest |est| pattern)
    uint32_t k_rem;    // how many keys to take among those matching the prefix
    uint32_t tau;      // final: the 31-bit pattern of the k-th largest |est|
    uint32_t k_eq;     // final: how many coordinates with |est| == tau are selected (smallest indices)
};

// kernels, for the optional per-kernel timing (sams_profile_*)
enum KernelId {
    KID_FILL = 0, KID_HASH_DUMP, KID_TAIL_X, KID_TAIL_ZERO_E, KID_HEAD, KID_SKETCH_ATOMIC, KID_REDUCE,
    KID_ESTIMATE, KID_SEL_INIT, KID_SEL_HIST, KID_SEL_PICK, KID_SEL_COUNT, KID_SEL_SCAN, KID_SEL_WRITE,
    KID_GATHER, KID_PLAN_BUILD, KID_BIN_SCATTER, KID_BIN_ACCUMULATE, KID_SKETCH_LDS, KID_BIN_LOOKUP,
    KID_BIN_COLLECT, KID_EST_MEDIAN, KID_HEAD_SCATTER, KID_REFINE_MAP, KID_HEAD_PA, KID_HEAD_SPARSE_V, KID_SEL_SMALL, KID_COUNT
};
const char *kernel_name(int kid);

constexpr int kMaxWorkers = 1024;     // n accepted by sams_create
constexpr int kWideCoords = 8;        // coordinates per workgroup of the 32-lanes-per-coordinate sparse kernels
constexpr int kWideMinWorkers = 16;   // ... which are used from this many workers on
constexpr int kProfPool = 8192;   // event pairs kept for one profiling window

struct ProfRec {
    hipEvent_t a, b;
    int kid;
};

// how sketch_accumulate is carried out for this context (chosen at creation from c and the tunables)
enum PlanMode { PLAN_ATOMIC = 0, PLAN_LDS_ROW = 1, PLAN_BINNED = 2 };

// static permutation "coordinate order -> bucket order" of the binned path (see sams_plan.hip)
struct Plan {
    int mode;
    int acc_variant;    // pass 2 of the rows that read meta words: 0 = 4-byte loads, 1 = 16-byte loads; 2 = no such row (all rows read chunk records)
    uint32_t rec_mask;  // bit j set: row j reads chunk records in pass 2 (k_bin_accumulate_r)
    int win_log2, tile_log2, chunk_log2, acc_threads, run_pad, grp_log2, stage_rows, stage_ilv, acc_wide;
    int64_t nbins, ntile, dpad, rowlen;
    uint16_t *srcp;     // [r][rowlen]      slot -> coordinate inside its tile (bits 0-14) and sign (bit 15), or padding
    uint32_t *dst16;    // [r][rowlen >> grp_log2]  stream position of each group of 2^grp_log2 slots (16, or the run padding if smaller)
    uint32_t *pbase;    // [r][ntile+1]     first slot of each tile
    uint32_t *binbase;  // [r][nbins+1]     start of each bin in the row stream (multiples of the chunk)
    uint32_t *meta;     // [r][rowlen]          per stream position: bucket in window, chain link, flags (absent with acc_variant 2)
    uint32_t *rec;      // [r][rowlen/4096][2560] chunk records of acc_variant 2: 4096 16-bit codes, 512 chain entries
    uint16_t *wlow;     // [r][rowlen]          per stream position: bucket in window only (what the recovery reads)
    void *stg_chunks;   // staging mapped from physical chunks picked all over device memory (stage_spread): their handles, else null
    int64_t stg_nchunks, stg_va_bytes;
    float *stg;         // n * stage_rows * rowlen floats: per-step staging, signed values at their stream positions
                        //                      ([stage_rows][rowlen/32][n][32], or [n][stage_rows][rowlen] without stage_ilv)
    const float *staged_u;  // vector whose sorted copy the staging holds (set by a fused head), else null
    float *rowest;      // [r][d]               per-step: signed row estimates in coordinate order (stage 3);
                        //                      absent when the median is fused (fused_median)
    bool fused_median;  // stage 3 keeps the row estimates in registers (decided when the plan is built)
};

// tunables: sams_configure edits the process-wide set, sams_create copies it into the context, and every
// later call on that context reads only its own copy
struct Tunables {
    int tile_log2;     // coordinates per tile of the binned path (0 = chosen from d)
    int win_log2;      // buckets per LDS window
    int chunk_log2;    // stream positions between two barriers of the accumulate kernel
    int acc_threads;   // workgroup size of the accumulate kernel
    int sketch_path;   // 0 = choose from c and d, 1 = global atomics, 2 = ordered (binned) always, 3 = LDS atomics when c fits a window
    int scatter_threads;  // workgroup size of the scatter kernel
    int estimate_path;    // stage 3: 0 = through the plan when there is one, unless table and vector are small; 1 = direct gathers from the table; 2 = through the plan
    int fuse_head;        // 1, 2 = amsgrad_ef_update also stages u for the next sketch_accumulate (2: a workgroup per worker)
    int fuse_median;      // 1 = recovery keeps the row estimates in registers where the shape allows, 0 = through memory
    int stage_rows;       // rows staged at once (0 = all r): bounds the staging buffer at n*stage_rows*rowlen floats
    int run_pad;          // runs are padded to a multiple of this many stream positions (4, 8, 16 or 32)
    int stage_interleave; // 1 = the workers' staged copies are interleaved in pieces of 32 stream positions
    int stage_spread;     // 1 = a staging buffer of 2 GiB or more is mapped from 1 GiB chunks picked at even distances over all free device memory
    int acc_wide;         // accumulate kernel where its shape allows (1024 threads, 2048-position chunks): 1 = 16-byte loads,
                          // 2 = 16-byte loads and compact chunk records instead of meta words (falls back to 1 when a chunk has too many chains)
};
extern Tunables g_tun;

// scratch of one radix selection (enqueue_select): the context's, or the static one of topk_refine_static
struct SelScratch {
    uint32_t *hist;          // [kHistBins]
    SelState *sel;           // [1]
    uint32_t *cnt;           // [2][ntile_cap]  per-wavefront-tile counts: greater, equal
    uint32_t *base;          // [2][ntile_cap]  exclusive prefix: selected before, equal before
    int64_t ntile_cap;       // tiles of kSelTile keys the arrays have room for
};

}  // namespace sams

struct sams_ctx {
    int64_t d, c, k;
    int32_t n, r;
    hipStream_t stream;
    sams::HashParams hp;
    // scratch (device)
    float *est;              // [d]
    uint32_t *bitmap;        // [ceil(d/32)]  bit l set <=> l in the most recent index set
    uint32_t *wordrank;      // [ceil(d/32)]  for a bitmap word with a bit set: the rank (position in idx) of its first set bit;
                             //               with gsel, only where the head is fused per worker (fuse_head = 2), else null
    float *gsel;             // [n][k]        g of every worker at the coordinates of the most recent index set, by rank
    uint32_t *hist;          // [kHistBins]
    sams::SelState *sel;     // [1]
    uint32_t *cnt;           // [2][ntile]  per-wavefront-tile counts: greater, equal
    uint32_t *base;          // [2][ntile]  exclusive prefix: selected before, equal before
    int64_t ntile;
    int64_t scratch_bytes;
    sams::Plan plan;
    sams::Tunables tun;      // the tunables as they were when the context was created
    // per-kernel timing (host)
    int prof_on;
    int prof_only;           // kernel id the timing is restricted to, -1 = every kernel
    int prof_used;
    sams::ProfRec *prof;     // [kProfPool], events created on first enable
    double prof_ms[sams::KID_COUNT];
    int64_t prof_n[sams::KID_COUNT];
};

namespace sams {

static inline int grid_for(int64_t work, int block, int64_t cap = (int64_t)1 << 30)
{
    int64_t g = (work + block - 1) / block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

static inline bool aligned16(const void *p) { return (((uintptr_t)p) & 15u) == 0; }

// Brackets one kernel launch with a HIP event pair on the context's stream while profiling is on.
struct ProfScope {
    sams_ctx *ctx;
    int slot;
    ProfScope(sams_ctx *c, int kid) : ctx(c), slot(-1)
    {
        if (c && c->prof_on && (c->prof_only < 0 || c->prof_only == kid) && c->prof_used < kProfPool) {
            slot = c->prof_used++;
            c->prof[slot].kid = kid;
            (void)hipEventRecord(c->prof[slot].a, c->stream);
        }
    }
    ~ProfScope()
    {
        if (slot >= 0) (void)hipEventRecord(ctx->prof[slot].b, ctx->stream);
    }
};

// SAMS_LAUNCH(ctx, KID_X, (kernel<..>), grid, block, args...)
#define SAMS_LAUNCH(ctx, kid, kernel, grid, block, ...)                                          \
    do {                                                                                         \
        ::sams::ProfScope ps_((ctx), (kid));                                                     \
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(block), 0, (ctx)->stream, __VA_ARGS__);      \
    } while (0)
// the same on a given stream, for code that also runs without a context (ctx may be null: no timing then)
#define SAMS_LAUNCH_ON(ctx, stream, kid, kernel, grid, block, ...)                               \
    do {                                                                                         \
        ::sams::ProfScope ps_((ctx), (kid));                                                     \
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(block), 0, (stream), __VA_ARGS__);           \
    } while (0)

// median of R row estimates (Sec. II-C); for an even R the lower middle element
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

// exclusive prefix sum over the 1024 threads of a block (part: at least 16 words of LDS; all threads call it):
// a shuffle scan inside every wavefront, then the 16 wavefront totals through LDS
__device__ __forceinline__ uint32_t block_exclusive_scan_1024(uint32_t val, uint32_t *part)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    uint32_t incl = val;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t x = __shfl_up(incl, off);
        if (lane >= off) incl += x;
    }
    if (lane == kWave - 1) part[wave] = incl;
    __syncthreads();
    uint32_t before = 0;
#pragma unroll
    for (int q = 0; q < 1024 / kWave; ++q) before += q < wave ? part[q] : 0u;
    __syncthreads();
    return before + incl - val;
}

// ---- enqueue functions (all asynchronous on ctx->stream; return SAMS_OK or SAMS_EHIP) ----
int enqueue_fill_u32(sams_ctx *ctx, uint32_t *p, int64_t n, uint32_t val);
int enqueue_hash_dump(sams_ctx *ctx, int32_t *bucket, int8_t *sign);
// sams_update.hip
int enqueue_tail(sams_ctx *ctx, float *e_u, float *x, const int32_t *idx, const float *delta,
                 int64_t k_sel, float lr, bool zero_e);
int enqueue_head(sams_ctx *ctx, const float *g, float *m, float *e_u, float *v, float *vhat,
                 float beta1, float beta2, float rho);
int enqueue_head_pa(sams_ctx *ctx, const float *g, float *m, float *e_u, float *v_w, float *vhat_w, float beta1,
                    float beta2, float rho);
int enqueue_reduce(sams_ctx *ctx, const float *S_workers, float *S_mean);
int enqueue_gather(sams_ctx *ctx, const float *u, const float *vhat, const int32_t *idx,
                   float *U_workers, float *delta);
// sams_sketch.hip
int enqueue_sketch(sams_ctx *ctx, const float *u, float *S_workers);
// sams_plan.hip
int plan_create(sams_ctx *ctx, const Tunables &tun);
void plan_destroy(sams_ctx *ctx);
int enqueue_sketch_planned(sams_ctx *ctx, const float *u, float *S_workers);
int enqueue_row_estimates_planned(sams_ctx *ctx, const float *S_mean, float *rowest);
// whole recovery through the plan when the fused collect+median kernel applies; *done says whether it ran
int enqueue_estimates_planned_fused(sams_ctx *ctx, const float *S_mean, const float *vhat, float *est, bool *done,
                                    uint32_t *hist);   // hist: null, or where to add the first-digit histogram of |est|
bool head_can_fuse(const sams_ctx *ctx);
// wordrank and gsel exist for this context (sams_create decides): the per-worker fused head then leaves the
// gradients of the selected coordinates in gsel and the second moments on I_{t-1} need no gathers
bool head_compacts_g(const sams_ctx *ctx);
int enqueue_head_scatter(sams_ctx *ctx, const float *g, float *m, float *e_u, float *v, float *vhat,
                         float beta1, float beta2, float rho, bool pa,   // pa: v, vhat are [n][d] (Alg. 1)
                         const int32_t *idx_prev, int64_t k_prev);       // I_{t-1}, as handed to the tail
// sams_select.hip
int enqueue_estimate(sams_ctx *ctx, const float *S_mean, const float *vhat, float *est, uint32_t *hist, bool *hist_done);
bool select_uses_passes(int64_t len);
int enqueue_select_begin(sams_ctx *ctx, hipStream_t stream, const SelScratch &sc, int64_t k);
// ctx may be null (no per-kernel timing); the work goes to `stream`, the scratch is the caller's
int enqueue_select(sams_ctx *ctx, hipStream_t stream, const SelScratch &sc, const float *keys, int64_t len, int64_t k,
                   int32_t *idx, float *val_sel, bool begun, bool hist0_done);
int enqueue_refine(sams_ctx *ctx, hipStream_t stream, const SelScratch &sc, int32_t *pos, const int32_t *idx_in,
                   const float *delta_in, int64_t k_in, int64_t k_out, int32_t *idx_out, float *delta_out);
SelScratch ctx_sel_scratch(const sams_ctx *ctx);
// sams_noalloc.hip: device address of the static scratch of topk_refine_static on the current device
int static_scratch_ptr(void **out);

}  // namespace sams
