// Binned, order-preserving Count Sketch accumulation (stage 1 of sams.h; Sec. II-C update rule) for
// tables that do not fit in LDS.
//
// The bucket hash sends consecutive coordinates to buckets spread over the whole row, so a direct
// implementation is one uncoalesced read-modify-write per (worker, row, coordinate).  Because the
// hashes never change, the permutation "coordinate order -> bucket order" is fixed, and it is worked
// out once, at context creation (the plan):
//   * coordinates are cut into tiles of L = 2^tile_log2; a row's buckets into windows ("bins") of
//     W = 2^win_log2 buckets that fit in LDS;
//   * every row owns a "stream": bin after bin, and inside a bin tile after tile, the coordinates that
//     fall into that bin in ascending order.  The piece of one (tile, bin) is a "run"; runs are padded
//     to a multiple of the run padding (4, 8, 16 or 32 elements) and bins to a whole number of chunks;
//   * seen from a tile, its padded runs laid one after the other are its "slots": srcp[row][slot]
//     names the coordinate (and its sign) a slot takes its value from (or marks padding), and
//     dst16[row][slot / G] says where in the row stream that group of G slots goes (G = the run padding,
//     at most 16);
//   * meta[row][pos] describes stream position pos: the bucket inside the window, and -- per chunk of
//     CH consecutive positions -- a chain linking the positions that hit the same bucket.
// Per step, pass 1 (k_bin_scatter) streams each worker's vector through LDS once and writes, for every
// row, the signed values to their stream positions (whole-sector stores); pass 2 (k_bin_accumulate)
// gives one workgroup per (worker, row, bin): it reads the bin's stream chunk by chunk (contiguous) and
// adds into its LDS window.  Inside a chunk the first position of every chain adds the whole chain, in
// stream order, with plain loads and stores: no two threads touch the same bucket between two barriers,
// so there are no atomics anywhere, every table cell is written exactly once, and the terms of a bucket
// are added in ascending coordinate order -- the same order as a sequential loop over the coordinates.
#include <stdlib.h>

#include "sams_ctx.h"

#pragma clang fp contract(off)

namespace sams {

constexpr int kPlanThreads = 1024;
constexpr int kNumXcd = 8;
constexpr int kScatterBatch = 4;             // groups of 4 slots whose metadata a scatter thread loads ahead
constexpr int kAccDepth = 8;                // chunks in flight per workgroup of the accumulate kernel
constexpr int kFusedThreads = 1024;          // kernels whose threads own the same 4-coordinate groups throughout
constexpr int kFusedIters = 4;              // tiles of at most 2^14 coordinates = 4 float4 per thread
constexpr int kMaxLdsBytes = 160 * 1024;      // LDS of one compute unit; the dynamic-LDS cap of every kernel here
constexpr int64_t kOrderedSingleBinMaxD = (int64_t)1 << 22;     // largest d sketched in order when c fits one window

constexpr uint16_t kSrcPad = 0x7fffu;          // slot source meaning "padding": tiles hold at most 2^14 coordinates
constexpr uint32_t kMetaNextShift = 15;
constexpr uint32_t kMetaHasNext = 1u << 26;
constexpr uint32_t kMetaNotFirst = 1u << 27;   // padding, or a position some earlier position adds
constexpr uint32_t kMetaPad = 1u << 28;        // padding (always together with kMetaNotFirst)
// Chunk records: the compact form of the meta words that k_bin_accumulate_r reads, one record per 4096 stream
// positions.  A record is 4096 16-bit codes followed by kRecChains chain entries.  Within a chunk, a position whose
// bucket no other position shares has its bucket as code (< 0x8000); the positions that share a bucket form a
// chain and carry 0x8000 | rank, the ranks of a chain being consecutive in stream order; padding carries
// 0x8000 | (a rank in the dummy range above kRecRanks).  Entry e describes chain e: bucket (bits 0-14), rank of its
// first position (bits 15-24), number of positions (bits 25-31; 0 = unused entry).
constexpr int kRecChunk = 4096;
constexpr int kRecCodeWords = kRecChunk / 2;
constexpr int kRecChains = 512;                // chains a chunk may have
constexpr int kRecRanks = 1024;                // chain positions a chunk may have
constexpr int kRecPadRanks = 256;              // dummy ranks of the padding positions
constexpr int kRecMaxChain = 127;              // positions one chain may have
constexpr int kRecWords = kRecCodeWords + kRecChains;
constexpr uint32_t kCodeChain = 0x8000u, kCodeRankMask = 0x7ffu;
constexpr int kRecDepth = 6;                   // chunks in flight per workgroup of k_bin_accumulate_r (even; 4, 6 and 8 time alike)

// streaming accesses: data touched once per step should not push the shared metadata out of L2.
// One 16-byte nontemporal instruction each (the pointers are 16-byte aligned, as float4 requires).
typedef float vec4f __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_stream(float4 *p, const float4 &v)
{
    vec4f t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<vec4f *>(p));
}
__device__ __forceinline__ float4 load_stream(const float4 *p)
{
    const vec4f t = __builtin_nontemporal_load(reinterpret_cast<const vec4f *>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}

// Rows [j0, j0 + rj) of the r rows are handled by one launch; their staging is stg[n][sr][rowlen] with
// row j at slot j - j0 (sr = rows the staging buffer was sized for, r in total).  With ilv set the layout is
// stg[sr][rowlen / 32][n][32] instead: the workers' copies of the same 32 stream positions (one 128-byte line
// each) lie next to each other, so that the workgroups of the n workers, which run side by side in both passes,
// write and read one contiguous region per (row, bin) instead of n regions rowlen apart.
struct RowGroup {
    int32_t j0, rj, sr, r, ilv;
};
constexpr int kIlvLog2 = 5;

// the rows (absolute numbers, all inside the row group at hand) one launch of an accumulate kernel handles
struct RowSel {
    int32_t cnt;
    int8_t row[SAMS_MAX_ROWS];
};

// start of worker i's copy of staged row jj, and the offset of stream position p from there
__device__ __forceinline__ int64_t stage_row(const RowGroup &rg, int32_t n, int64_t rowlen, int32_t i, int32_t jj)
{
    return rg.ilv ? (int64_t)jj * n * rowlen + ((int64_t)i << kIlvLog2) : ((int64_t)i * rg.sr + jj) * rowlen;
}
__device__ __forceinline__ int64_t stage_pos(const RowGroup &rg, int32_t n, uint32_t p)
{
    return rg.ilv ? ((int64_t)(p >> kIlvLog2) * n << kIlvLog2) + (p & ((1u << kIlvLog2) - 1u)) : (int64_t)p;
}

typedef uint32_t vec2u __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint2 load_stream2(const uint2 *p)
{
    const vec2u t = __builtin_nontemporal_load(reinterpret_cast<const vec2u *>(p));
    return make_uint2(t.x, t.y);
}

__host__ __device__ __forceinline__ int pad_run(int len, int pad) { return (len + pad - 1) & ~(pad - 1); }

// ------------------------------------------------------------------------------------------
// plan step 1: one workgroup per (row, tile); bitonic sort of the tile's coordinates by (bin, coordinate)
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kPlanThreads)
k_plan_sort(HashParams hp, int64_t d, int tile_log2, int win_log2, int64_t nbins, int64_t ntile,
            int64_t dpad, uint16_t *__restrict__ src, uint16_t *__restrict__ bst)
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
    const uint32_t lmask = (uint32_t)L - 1u;
    for (int p = threadIdx.x; p < L; p += blockDim.x) {
        uint32_t key = keys[p];
        uint16_t s = 0;
        if (key != 0xffffffffu) {
            uint32_t loc = key & lmask;
            s = (uint16_t)(loc | (sign_neg(hp, j, (uint32_t)(l0 + loc)) ? 0x8000u : 0u));
        }
        src[(int64_t)j * dpad + l0 + p] = s;
    }
    // first sorted position of every bin (bin == nbins: one past the last real coordinate)
    for (int64_t b = threadIdx.x; b <= nbins; b += blockDim.x) {
        uint32_t want = (uint32_t)b << tile_log2;                   // smallest key of bin b
        int lo = 0, hi = L;
        while (lo < hi) {
            int mid = (lo + hi) >> 1;
            uint32_t key = keys[mid];
            bool less = (b == nbins) ? (key != 0xffffffffu) : (key != 0xffffffffu && key < want);
            if (less) lo = mid + 1; else hi = mid;
        }
        bst[((int64_t)j * ntile + tile) * (nbins + 1) + b] = (uint16_t)lo;
    }
}

// ------------------------------------------------------------------------------------------
// plan step 2: per (row, bin), exclusive prefix over the tiles of the padded run lengths
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_plan_runlen(const uint16_t *__restrict__ bst, int pad, int64_t nbins, int64_t ntile, uint32_t *__restrict__ off,
              uint32_t *__restrict__ total)
{
    __shared__ uint32_t part[256];
    const int64_t bin = blockIdx.x;
    const int j = blockIdx.y;
    const int T = blockDim.x, t = threadIdx.x;
    const int64_t per = (ntile + T - 1) / T;
    const int64_t lo = (int64_t)t * per, hi = (lo + per) < ntile ? (lo + per) : ntile;
    const uint16_t *b0 = bst + (int64_t)j * ntile * (nbins + 1) + bin;
    uint32_t s = 0;
    for (int64_t q = lo; q < hi; ++q) {
        const uint16_t *e = b0 + q * (nbins + 1);
        s += (uint32_t)pad_run((int)e[1] - (int)e[0], pad);
    }
    part[t] = s;
    __syncthreads();
    if (t == 0) {
        uint32_t run = 0;
        for (int q = 0; q < T; ++q) { uint32_t x = part[q]; part[q] = run; run += x; }
        total[(int64_t)j * nbins + bin] = run;
    }
    __syncthreads();
    uint32_t run = part[t];
    uint32_t *o = off + ((int64_t)j * nbins + bin) * ntile;
    for (int64_t q = lo; q < hi; ++q) {
        const uint16_t *e = b0 + q * (nbins + 1);
        o[q] = run;
        run += (uint32_t)pad_run((int)e[1] - (int)e[0], pad);
    }
}

// ------------------------------------------------------------------------------------------
// plan step 3a: per (row, tile), the padded length of the tile's slots
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_plan_tilelen(const uint16_t *__restrict__ bst, int pad, int64_t nbins, int64_t ntile, uint32_t *__restrict__ tilelen)
{
    __shared__ uint32_t part[256];
    const int64_t tile = blockIdx.x;
    const int j = blockIdx.y;
    const uint16_t *bt = bst + ((int64_t)j * ntile + tile) * (nbins + 1);
    uint32_t s = 0;
    for (int64_t b = threadIdx.x; b < nbins; b += blockDim.x) s += (uint32_t)pad_run((int)bt[b + 1] - (int)bt[b], pad);
    part[threadIdx.x] = s;
    __syncthreads();
    for (int h = 128; h > 0; h >>= 1) {
        if ((int)threadIdx.x < h) part[threadIdx.x] += part[threadIdx.x + h];
        __syncthreads();
    }
    if (threadIdx.x == 0) tilelen[(int64_t)j * ntile + tile] = part[0];
}

// ------------------------------------------------------------------------------------------
// plan step 3b: per (row, tile): the source of every slot, the stream position of every group of G
// slots, and the bucket of every stream position
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_plan_place(HashParams hp, int pad, int gl, int tile_log2, int win_log2, int64_t nbins, int64_t ntile, int64_t dpad,
             int64_t rowlen, const uint16_t *__restrict__ src, const uint16_t *__restrict__ bst,
             const uint32_t *__restrict__ off, const uint32_t *__restrict__ binbase,
             const uint32_t *__restrict__ pbase, uint16_t *__restrict__ srcp, uint32_t *__restrict__ dst16,
             uint32_t *__restrict__ meta, uint16_t *__restrict__ wlow)
{
    extern __shared__ uint32_t pst[];                               // [nbins + 1] padded prefix inside the tile
    __shared__ uint32_t part[256];
    const int64_t tile = blockIdx.x;
    const int j = blockIdx.y;
    const int64_t l0 = tile << tile_log2;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave, nwave = blockDim.x / kWave;
    const uint32_t wmask = (1u << win_log2) - 1u;
    const uint16_t *bt = bst + ((int64_t)j * ntile + tile) * (nbins + 1);
    const uint16_t *sj = src + (int64_t)j * dpad + l0;
    // exclusive prefix of the padded run lengths over the bins (blocked two-level scan)
    const int T = blockDim.x, t = threadIdx.x;
    const int64_t per = (nbins + T - 1) / T;
    const int64_t lo = (int64_t)t * per, hi = (lo + per) < nbins ? (lo + per) : nbins;
    uint32_t sum = 0;
    for (int64_t b = lo; b < hi; ++b) sum += (uint32_t)pad_run((int)bt[b + 1] - (int)bt[b], pad);
    part[t] = sum;
    __syncthreads();
    if (t == 0) {
        uint32_t run = 0;
        for (int q = 0; q < T; ++q) { uint32_t x = part[q]; part[q] = run; run += x; }
    }
    __syncthreads();
    uint32_t run = part[t];
    for (int64_t b = lo; b < hi; ++b) {
        pst[b] = run;
        run += (uint32_t)pad_run((int)bt[b + 1] - (int)bt[b], pad);
    }
    __syncthreads();
    const uint32_t p0 = pbase[(int64_t)j * (ntile + 1) + tile];
    for (int64_t bin = wave; bin < nbins; bin += nwave) {
        const int a = bt[bin], len = (int)bt[bin + 1] - a, plen = pad_run(len, pad);
        const uint32_t start = binbase[(int64_t)j * (nbins + 1) + bin] + off[((int64_t)j * nbins + bin) * ntile + tile];
        const uint32_t po = p0 + pst[bin];
        for (int s = lane; s < plen; s += kWave) {
            uint16_t sv = kSrcPad;
            if (s < len) {
                sv = sj[a + s];
                uint32_t wl = bucket_of(hp, j, (uint32_t)(l0 + (sv & 0x7fffu))) & wmask;
                meta[(int64_t)j * rowlen + start + s] = wl;
                wlow[(int64_t)j * rowlen + start + s] = (uint16_t)wl;
            }
            srcp[(int64_t)j * rowlen + po + s] = sv;
            if ((s & ((1 << gl) - 1)) == 0) dst16[((int64_t)j * rowlen + po + s) >> gl] = start + (uint32_t)s;
        }
    }
}

// ------------------------------------------------------------------------------------------
// plan step 4: per (row, chunk), chain the positions that share a bucket
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kPlanThreads)
k_plan_chain(int chunk_log2, int64_t rowlen, uint32_t *__restrict__ meta)
{
    extern __shared__ uint32_t keys[];
    const int CH = 1 << chunk_log2;
    uint32_t *m = meta + (int64_t)blockIdx.y * rowlen + ((int64_t)blockIdx.x << chunk_log2);
    for (int p = threadIdx.x; p < CH; p += blockDim.x) {
        uint32_t w = m[p];
        keys[p] = (w & kMetaNotFirst) ? 0xffffffffu : ((w << chunk_log2) | (uint32_t)p);
    }
    __syncthreads();
    for (int k = 2; k <= CH; k <<= 1) {
        for (int jj = k >> 1; jj > 0; jj >>= 1) {
            for (int t = threadIdx.x; t < CH; t += blockDim.x) {
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
    const uint32_t pmask = (uint32_t)CH - 1u;
    for (int s = threadIdx.x; s < CH; s += blockDim.x) {
        uint32_t key = keys[s];
        if (key == 0xffffffffu) continue;                            // padding keeps its kMetaNotFirst word
        uint32_t wl = key >> chunk_log2, pos = key & pmask;
        uint32_t word = wl;
        if (s > 0 && (keys[s - 1] >> chunk_log2) == wl) word |= kMetaNotFirst;
        if (s + 1 < CH && keys[s + 1] != 0xffffffffu && (keys[s + 1] >> chunk_log2) == wl)
            word |= kMetaHasNext | ((keys[s + 1] & pmask) << kMetaNextShift);
        m[pos] = word;
    }
}

// ------------------------------------------------------------------------------------------
// plan step 4' (instead of step 4 where it applies): the chunk records of k_bin_accumulate_r
// ------------------------------------------------------------------------------------------
// One workgroup per (row, chunk of 4096 positions): sorts the chunk's positions by (bucket, position), finds the
// groups that share a bucket and writes the record.  `over` is set when a chunk does not fit the record format
// (too many chains or chain positions, or too long a chain), per row (over[row]): such rows keep their meta words.
__global__ void __launch_bounds__(kPlanThreads)
k_plan_records(const uint32_t *__restrict__ meta, uint32_t *__restrict__ rec, int64_t rowlen, uint32_t *__restrict__ over)
{
    __shared__ uint32_t keys[kRecChunk];
    __shared__ uint32_t part[16];
    __shared__ uint32_t nchains;
    const int t = threadIdx.x;
    const int64_t nchunk = rowlen / kRecChunk;
    const uint32_t *m = meta + (int64_t)blockIdx.y * rowlen + (int64_t)blockIdx.x * kRecChunk;
    uint32_t *rc = rec + ((int64_t)blockIdx.y * nchunk + blockIdx.x) * kRecWords;
    uint16_t *codes = reinterpret_cast<uint16_t *>(rc);
    for (int p = t; p < kRecChunk; p += kPlanThreads) {
        const uint32_t w = m[p];
        const bool pad = (w & kMetaPad) != 0;
        keys[p] = pad ? 0xffffffffu : (((w & 0x7fffu) << 12) | (uint32_t)p);
        if (pad) codes[p] = (uint16_t)(kCodeChain | (uint32_t)kRecRanks | ((uint32_t)p & (kRecPadRanks - 1)));
    }
    __syncthreads();
    for (int k = 2; k <= kRecChunk; k <<= 1) {
        for (int jj = k >> 1; jj > 0; jj >>= 1) {
            for (int q = t; q < kRecChunk; q += kPlanThreads) {
                const int other = q ^ jj;
                if (other > q) {
                    const uint32_t a = keys[q], b = keys[other];
                    const bool up = (q & k) == 0;
                    if ((a > b) == up) {
                        keys[q] = b;
                        keys[other] = a;
                    }
                }
            }
            __syncthreads();
        }
    }
    // thread t looks at the sorted elements 4t .. 4t+3
    bool inchain[4], cstart[4];
    uint32_t n_in = 0, n_cs = 0;
#pragma unroll
    for (int z = 0; z < 4; ++z) {
        const int s0 = 4 * t + z;
        const uint32_t key = keys[s0];
        const bool valid = key != 0xffffffffu;
        const uint32_t b = key >> 12;
        const bool prev_same = valid && s0 > 0 && (keys[s0 - 1] >> 12) == b;
        const bool next_same = valid && s0 + 1 < kRecChunk && keys[s0 + 1] != 0xffffffffu && (keys[s0 + 1] >> 12) == b;
        inchain[z] = prev_same || next_same;
        cstart[z] = !prev_same && next_same;
        n_in += inchain[z] ? 1u : 0u;
        n_cs += cstart[z] ? 1u : 0u;
    }
    uint32_t rank = block_exclusive_scan_1024(n_in, part);
    uint32_t e = block_exclusive_scan_1024(n_cs, part);
    bool too_long = false;
#pragma unroll
    for (int z = 0; z < 4; ++z) {
        const int s0 = 4 * t + z;
        const uint32_t key = keys[s0];
        if (key == 0xffffffffu) continue;
        const uint32_t b = key >> 12, pos = key & 0xfffu;
        codes[pos] = (uint16_t)(inchain[z] ? (kCodeChain | (rank & kCodeRankMask)) : b);
        if (cstart[z]) {
            uint32_t len = 1;
            while (s0 + (int)len < kRecChunk && keys[s0 + len] != 0xffffffffu && (keys[s0 + len] >> 12) == b &&
                   len <= (uint32_t)kRecMaxChain)
                ++len;
            if (len > (uint32_t)kRecMaxChain) too_long = true;
            if (e < (uint32_t)kRecChains && rank < (uint32_t)kRecRanks)
                rc[kRecCodeWords + e] = b | (rank << 15) | ((len & 127u) << 25);
            ++e;
        }
        if (inchain[z]) ++rank;
    }
    if (t == kPlanThreads - 1) {
        nchains = e;
        if (e > (uint32_t)kRecChains || rank > (uint32_t)kRecRanks) atomicOr(over + blockIdx.y, 1u);
    }
    if (too_long) atomicOr(over + blockIdx.y, 1u);
    __syncthreads();
    for (uint32_t q = nchains + (uint32_t)t; q < (uint32_t)kRecChains; q += kPlanThreads) rc[kRecCodeWords + q] = 0u;   // unused entries
}

// ------------------------------------------------------------------------------------------
// pass 1: per tile, every worker's values to their positions in the row streams
// ------------------------------------------------------------------------------------------
// One workgroup per (tile, worker).  Workgroup ids are dealt round-robin to the 8 XCDs; consecutive tiles are
// given to the same XCD so that neighbouring runs of a bin are written through one L2, and the n workers of
// a tile sit there in consecutive slots so that the tile's plan metadata crosses the fabric once and comes
// from that L2 for the other workers.  A thread owns 4 consecutive slots (always inside
// one group of G >= 4 slots, hence one run): one 8-byte load of their sources, one 4-byte load of the group's
// stream position, 4 LDS reads and one 16-byte store -- nothing depends on another global load.
__global__ void __launch_bounds__(1024)
k_bin_scatter(const float *__restrict__ u, const uint16_t *__restrict__ srcp, const uint32_t *__restrict__ dst16,
              const uint32_t *__restrict__ pbase, float *__restrict__ stg, int32_t n, RowGroup rg, int64_t d,
              int tile_log2, int64_t ntile, int64_t rowlen, int gl)
{
    extern __shared__ float tilebuf[];
    const int L = 1 << tile_log2;
    const int64_t per = (ntile + kNumXcd - 1) / kNumXcd;
    const int64_t slot = blockIdx.x / kNumXcd;
    const int32_t i = (int32_t)(slot % n);
    const int64_t tile = (int64_t)(blockIdx.x % kNumXcd) * per + slot / n;
    if (tile >= ntile) return;
    const int64_t l0 = tile << tile_log2;
    const bool vec = (d & 3) == 0;
    {
        const float *ui = u + (int64_t)i * d;
        if (vec) {
            for (int p = threadIdx.x * 4; p < L; p += blockDim.x * 4) {
                float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
                if (l0 + p < d) q = load_stream(reinterpret_cast<const float4 *>(ui + l0 + p));
                *reinterpret_cast<float4 *>(tilebuf + p) = q;
            }
        } else {
            for (int p = threadIdx.x; p < L; p += blockDim.x) tilebuf[p] = (l0 + p < d) ? ui[l0 + p] : 0.f;
        }
        __syncthreads();
        for (int32_t j = rg.j0; j < rg.j0 + rg.rj; ++j) {
            const uint32_t o0 = pbase[(int64_t)j * (ntile + 1) + tile], o1 = pbase[(int64_t)j * (ntile + 1) + tile + 1];
            const uint16_t *sj = srcp + (int64_t)j * rowlen;
            const uint32_t *dj = dst16 + (int64_t)j * (rowlen >> gl);
            float *oj = stg + stage_row(rg, n, rowlen, i, j - rg.j0);
            // four groups of 4 slots per thread and batch: their sources and positions are loaded unconditionally
            // (clamped addresses; o1 - o0 is a multiple of 4, at least 4) before the first is used
            for (uint32_t ob = o0 + threadIdx.x * 4; ob < o1; ob += blockDim.x * 4 * kScatterBatch) {
                uint2 packed4[kScatterBatch];
                int64_t at4[kScatterBatch];
#pragma unroll
                for (int uu = 0; uu < kScatterBatch; ++uu) {
                    const uint32_t o = ob + (uint32_t)uu * blockDim.x * 4, oc = o < o1 ? o : o1 - 4;
                    packed4[uu] = *reinterpret_cast<const uint2 *>(sj + oc);
                    at4[uu] = stage_pos(rg, n, dj[oc >> gl]) + (oc & ((1u << gl) - 1u));
                }
#pragma unroll
                for (int uu = 0; uu < kScatterBatch; ++uu) {
                    if (ob + (uint32_t)uu * blockDim.x * 4 < o1) {
                        const uint2 packed = packed4[uu];
                        const uint32_t s0 = packed.x & 0xffffu, s1 = packed.x >> 16, s2 = packed.y & 0xffffu,
                                       s3 = packed.y >> 16;
                        float4 v;
                        v.x = (s0 == kSrcPad) ? 0.f : tilebuf[s0 & 0x7fffu]; v.x = (s0 & 0x8000u) ? -v.x : v.x;
                        v.y = (s1 == kSrcPad) ? 0.f : tilebuf[s1 & 0x7fffu]; v.y = (s1 & 0x8000u) ? -v.y : v.y;
                        v.z = (s2 == kSrcPad) ? 0.f : tilebuf[s2 & 0x7fffu]; v.z = (s2 & 0x8000u) ? -v.z : v.z;
                        v.w = (s3 == kSrcPad) ? 0.f : tilebuf[s3 & 0x7fffu]; v.w = (s3 & 0x8000u) ? -v.w : v.w;
                        store_stream(reinterpret_cast<float4 *>(oj + at4[uu]), v);
                    }
                }
            }
        }
    }
}

// Pass 1 fused with the head of Alg. 2 (the m, u, h, v, vhat lines; see k_head): the tile of u that pass 1
// needs in LDS is produced on the spot from g, m and e, so u is never read back from memory.  The
// arithmetic is the same, operation for operation, as in the separate head kernel.  1024 threads, each
// owning the same 4-coordinate groups for every worker so that the worker sum of g stays in registers.

struct HeadArgs {
    const float *g;
    float *m, *e, *v, *vhat;
    const uint32_t *bitmap;
    float beta1, omb1, beta2, omb2, rho;
    const uint32_t *wordrank;   // with gsel: where the per-worker head leaves g on I_{t-1} (null: it does not)
    float *gsel;
    int64_t k_prev;
};

// PA: the head of Alg. 1 instead (every worker keeps its own v, vhat [n][d]; u = m / sqrt(vhat) + rho e).
template <bool PA>
__global__ void __launch_bounds__(kFusedThreads)
k_head_scatter(HeadArgs ha, const uint16_t *__restrict__ srcp, const uint32_t *__restrict__ dst16,
               const uint32_t *__restrict__ pbase, float *__restrict__ stg, int32_t n, RowGroup rg, int64_t d,
               int tile_log2, int64_t ntile, int64_t rowlen, int gl)
{
    extern __shared__ float tilebuf[];
    const int L = 1 << tile_log2;
    const int64_t per = (ntile + kNumXcd - 1) / kNumXcd;
    const int64_t tile = (int64_t)(blockIdx.x % kNumXcd) * per + blockIdx.x / kNumXcd;
    if (tile >= ntile) return;
    const int64_t l0 = tile << tile_log2;
    float gs[kFusedIters][4];
    uint32_t selbits[kFusedIters];
#pragma unroll
    for (int it = 0; it < kFusedIters; ++it) {
        const int p = (it * kFusedThreads + (int)threadIdx.x) * 4;
        selbits[it] = 0;
        if (p < L && l0 + p < d) selbits[it] = (ha.bitmap[(l0 + p) >> 5] >> ((l0 + p) & 31)) & 0xFu;
    }
    for (int32_t i = 0; i < n; ++i) {
        const int64_t wbase = (int64_t)i * d + l0;
#pragma unroll
        for (int it = 0; it < kFusedIters; ++it) {
            const int p = (it * kFusedThreads + (int)threadIdx.x) * 4;
            if (p < L) {
                float uv[4] = {0.f, 0.f, 0.f, 0.f};
                if (l0 + p < d) {
                    const float4 a = load_stream(reinterpret_cast<const float4 *>(ha.g + wbase + p));
                    const float4 b = load_stream(reinterpret_cast<const float4 *>(ha.m + wbase + p));
                    const float4 cc = load_stream(reinterpret_cast<const float4 *>(ha.e + wbase + p));
                    const float gv[4] = {a.x, a.y, a.z, a.w}, mv[4] = {b.x, b.y, b.z, b.w},
                                ev[4] = {cc.x, cc.y, cc.z, cc.w};
                    float mo[4];
                    if constexpr (PA) {
                        const float4 pv = load_stream(reinterpret_cast<const float4 *>(ha.v + wbase + p));
                        const float4 ph = load_stream(reinterpret_cast<const float4 *>(ha.vhat + wbase + p));
                        float vv[4] = {pv.x, pv.y, pv.z, pv.w}, vh[4] = {ph.x, ph.y, ph.z, ph.w};
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const float mm = (ha.beta1 * mv[t]) + (ha.omb1 * gv[t]);
                            const float v2 = (ha.beta2 * vv[t]) + (ha.omb2 * (gv[t] * gv[t]));
                            const float ein = ((selbits[it] >> t) & 1u) ? 0.0f : ev[t];   // e_t is zero on I_t
                            mo[t] = mm;
                            vv[t] = v2;
                            if (v2 > vh[t]) vh[t] = v2;
                            uv[t] = (mm / sqrtf(vh[t])) + (ha.rho * ein);
                        }
                        store_stream(reinterpret_cast<float4 *>(ha.v + wbase + p), make_float4(vv[0], vv[1], vv[2], vv[3]));
                        store_stream(reinterpret_cast<float4 *>(ha.vhat + wbase + p), make_float4(vh[0], vh[1], vh[2], vh[3]));
                    } else {
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const float mm = (ha.beta1 * mv[t]) + (ha.omb1 * gv[t]);
                            const float ein = ((selbits[it] >> t) & 1u) ? 0.0f : ev[t];   // e_t is zero on I_t
                            mo[t] = mm;
                            uv[t] = mm + (ha.rho * ein);
                            gs[it][t] = (i == 0) ? gv[t] : (gs[it][t] + gv[t]);
                        }
                    }
                    store_stream(reinterpret_cast<float4 *>(ha.m + wbase + p), make_float4(mo[0], mo[1], mo[2], mo[3]));
                    store_stream(reinterpret_cast<float4 *>(ha.e + wbase + p), make_float4(uv[0], uv[1], uv[2], uv[3]));
                }
                *reinterpret_cast<float4 *>(tilebuf + p) = make_float4(uv[0], uv[1], uv[2], uv[3]);
            }
        }
        __syncthreads();
        for (int32_t j = rg.j0; j < rg.j0 + rg.rj; ++j) {
            const uint32_t o0 = pbase[(int64_t)j * (ntile + 1) + tile], o1 = pbase[(int64_t)j * (ntile + 1) + tile + 1];
            const uint16_t *sj = srcp + (int64_t)j * rowlen;
            const uint32_t *dj = dst16 + (int64_t)j * (rowlen >> gl);
            float *oj = stg + stage_row(rg, n, rowlen, i, j - rg.j0);
            for (uint32_t o = o0 + threadIdx.x * 4; o < o1; o += blockDim.x * 4) {
                const uint2 packed = *reinterpret_cast<const uint2 *>(sj + o);
                const int64_t at = stage_pos(rg, n, dj[o >> gl]) + (o & ((1u << gl) - 1u));
                const uint32_t s0 = packed.x & 0xffffu, s1 = packed.x >> 16, s2 = packed.y & 0xffffu,
                               s3 = packed.y >> 16;
                float4 v;
                v.x = (s0 == kSrcPad) ? 0.f : tilebuf[s0 & 0x7fffu]; v.x = (s0 & 0x8000u) ? -v.x : v.x;
                v.y = (s1 == kSrcPad) ? 0.f : tilebuf[s1 & 0x7fffu]; v.y = (s1 & 0x8000u) ? -v.y : v.y;
                v.z = (s2 == kSrcPad) ? 0.f : tilebuf[s2 & 0x7fffu]; v.z = (s2 & 0x8000u) ? -v.z : v.z;
                v.w = (s3 == kSrcPad) ? 0.f : tilebuf[s3 & 0x7fffu]; v.w = (s3 & 0x8000u) ? -v.w : v.w;
                store_stream(reinterpret_cast<float4 *>(oj + at), v);
            }
        }
        __syncthreads();
    }
    if constexpr (PA) return;                                        // the second moments were per worker, above
    const float fn = (float)n;
#pragma unroll
    for (int it = 0; it < kFusedIters; ++it) {
        const int p = (it * kFusedThreads + (int)threadIdx.x) * 4;
        if (p < L && l0 + p < d) {
            const float4 vin = *reinterpret_cast<const float4 *>(ha.v + l0 + p);
            const float4 hin = *reinterpret_cast<const float4 *>(ha.vhat + l0 + p);
            float vv[4] = {vin.x, vin.y, vin.z, vin.w}, vh[4] = {hin.x, hin.y, hin.z, hin.w};
            bool moved = false;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float h = ((selbits[it] >> t) & 1u) ? (gs[it][t] / fn) : 0.0f;
                vv[t] = (ha.beta2 * vv[t]) + (ha.omb2 * (h * h));
                if (vv[t] > vh[t]) { vh[t] = vv[t]; moved = true; }
            }
            *reinterpret_cast<float4 *>(ha.v + l0 + p) = make_float4(vv[0], vv[1], vv[2], vv[3]);
            if (moved) *reinterpret_cast<float4 *>(ha.vhat + l0 + p) = make_float4(vh[0], vh[1], vh[2], vh[3]);
        }
    }
}

// The same work with one workgroup per (tile, worker): the n workgroups of a tile sit on the same XCD in
// consecutive slots and walk the tile's plan metadata at about the same time, so that it comes from HBM once
// and from that XCD's L2 for the others, instead of being re-read through the fabric once per worker.
// The second moments of Alg. 2 need the mean gradient over the workers, but only on I_{t-1}: worker 0's
// workgroup decays v everywhere (the update with h = 0, which is what every other coordinate gets) and
// k_head_sparse_v then adds the (1 - beta2) h^2 term on I_{t-1}.  Rounding is that of the one-step formula:
// v' = beta2 v (+ 0), then v = v' + (1 - beta2) h^2; vhat = max(max(vhat, v'), v) = max(vhat, v) since v >= v'.
// (Fetching the other workers' g for those coordinates inside worker 0's workgroup instead was tried: its
// divergent, dependent gathers made the kernel 1.5x slower.)
template <bool PA>
__global__ void __launch_bounds__(kFusedThreads)
k_head_scatter_w(HeadArgs ha, const uint16_t *__restrict__ srcp, const uint32_t *__restrict__ dst16,
                 const uint32_t *__restrict__ pbase, float *__restrict__ stg, int32_t n, RowGroup rg, int64_t d,
                 int tile_log2, int64_t ntile, int64_t rowlen, int gl)
{
    extern __shared__ float tilebuf[];
    const int L = 1 << tile_log2;
    const int64_t per = (ntile + kNumXcd - 1) / kNumXcd;
    const int64_t slot = blockIdx.x / kNumXcd;
    const int32_t i = (int32_t)(slot % n);
    const int64_t tile = (int64_t)(blockIdx.x % kNumXcd) * per + slot / n;
    if (slot / n >= per || tile >= ntile) return;
    const int64_t l0 = tile << tile_log2;
    const int64_t wbase = (int64_t)i * d + l0;
    float4 gkeep[kFusedIters];                                       // g and the bitmap word of the positions with a
    uint32_t wkeep[kFusedIters];                                     // member of I_{t-1}, for the compaction below
#pragma unroll
    for (int it = 0; it < kFusedIters; ++it) { gkeep[it] = make_float4(0.f, 0.f, 0.f, 0.f); wkeep[it] = 0u; }
#pragma unroll
    for (int it = 0; it < kFusedIters; ++it) {
        const int p = (it * kFusedThreads + (int)threadIdx.x) * 4;
        if (p < L) {
            float uv[4] = {0.f, 0.f, 0.f, 0.f};
            if (l0 + p < d) {
                const uint32_t bword = ha.bitmap[(l0 + p) >> 5];
                const uint32_t selbits = (bword >> ((l0 + p) & 31)) & 0xFu;
                const float4 a = load_stream(reinterpret_cast<const float4 *>(ha.g + wbase + p));
                const float4 b = load_stream(reinterpret_cast<const float4 *>(ha.m + wbase + p));
                const float4 cc = load_stream(reinterpret_cast<const float4 *>(ha.e + wbase + p));
                const float gv[4] = {a.x, a.y, a.z, a.w}, mv[4] = {b.x, b.y, b.z, b.w}, ev[4] = {cc.x, cc.y, cc.z, cc.w};
                float mo[4];
                if constexpr (PA) {
                    const float4 pv = load_stream(reinterpret_cast<const float4 *>(ha.v + wbase + p));
                    const float4 ph = load_stream(reinterpret_cast<const float4 *>(ha.vhat + wbase + p));
                    float vv[4] = {pv.x, pv.y, pv.z, pv.w}, vh[4] = {ph.x, ph.y, ph.z, ph.w};
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const float mm = (ha.beta1 * mv[t]) + (ha.omb1 * gv[t]);
                        const float v2 = (ha.beta2 * vv[t]) + (ha.omb2 * (gv[t] * gv[t]));
                        const float ein = ((selbits >> t) & 1u) ? 0.0f : ev[t];          // e_t is zero on I_t
                        mo[t] = mm;
                        vv[t] = v2;
                        if (v2 > vh[t]) vh[t] = v2;
                        uv[t] = (mm / sqrtf(vh[t])) + (ha.rho * ein);
                    }
                    store_stream(reinterpret_cast<float4 *>(ha.v + wbase + p), make_float4(vv[0], vv[1], vv[2], vv[3]));
                    store_stream(reinterpret_cast<float4 *>(ha.vhat + wbase + p), make_float4(vh[0], vh[1], vh[2], vh[3]));
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const float mm = (ha.beta1 * mv[t]) + (ha.omb1 * gv[t]);
                        const float ein = ((selbits >> t) & 1u) ? 0.0f : ev[t];          // e_t is zero on I_t
                        mo[t] = mm;
                        uv[t] = mm + (ha.rho * ein);
                    }
                    gkeep[it] = a;
                    wkeep[it] = selbits ? bword : 0u;
                    if (i == 0) {                                    // the decay of v, once per coordinate
                        const float4 vin = *reinterpret_cast<const float4 *>(ha.v + l0 + p);
                        const float4 hin = *reinterpret_cast<const float4 *>(ha.vhat + l0 + p);
                        float vv[4] = {vin.x, vin.y, vin.z, vin.w}, vh[4] = {hin.x, hin.y, hin.z, hin.w};
                        bool moved = false;
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            vv[t] = (ha.beta2 * vv[t]);              // + (1 - beta2) * 0^2, exactly
                            if (vv[t] > vh[t]) { vh[t] = vv[t]; moved = true; }
                        }
                        *reinterpret_cast<float4 *>(ha.v + l0 + p) = make_float4(vv[0], vv[1], vv[2], vv[3]);
                        if (moved) *reinterpret_cast<float4 *>(ha.vhat + l0 + p) = make_float4(vh[0], vh[1], vh[2], vh[3]);
                    }
                }
                store_stream(reinterpret_cast<float4 *>(ha.m + wbase + p), make_float4(mo[0], mo[1], mo[2], mo[3]));
                store_stream(reinterpret_cast<float4 *>(ha.e + wbase + p), make_float4(uv[0], uv[1], uv[2], uv[3]));
            }
            *reinterpret_cast<float4 *>(tilebuf + p) = make_float4(uv[0], uv[1], uv[2], uv[3]);
        }
    }
    if constexpr (!PA) {
        // g of this worker at the coordinates of I_{t-1}, at their rank in the index set: the rank of the word's
        // first member plus the members of the word below the coordinate.  Kept out of the streaming loop above,
        // whose loads a wait for the rank would hold up.
        if (ha.gsel) {
#pragma unroll
            for (int it = 0; it < kFusedIters; ++it) {
                const uint32_t selbits4 = (wkeep[it] >> ((uint32_t)((it * kFusedThreads + (int)threadIdx.x) * 4) & 31u)) & 0xFu;
                if (selbits4) {
                    const int p = (it * kFusedThreads + (int)threadIdx.x) * 4;
                    const uint32_t r0 = ha.wordrank[(l0 + p) >> 5];
                    const float gv[4] = {gkeep[it].x, gkeep[it].y, gkeep[it].z, gkeep[it].w};
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        if ((selbits4 >> t) & 1u) {
                            const uint32_t below = wkeep[it] & ((1u << (((uint32_t)p & 31u) + t)) - 1u);
                            ha.gsel[(int64_t)i * ha.k_prev + r0 + __popc(below)] = gv[t];
                        }
                }
            }
        }
    }
    __syncthreads();
    for (int32_t j = rg.j0; j < rg.j0 + rg.rj; ++j) {
        const uint32_t o0 = pbase[(int64_t)j * (ntile + 1) + tile], o1 = pbase[(int64_t)j * (ntile + 1) + tile + 1];
        const uint16_t *sj = srcp + (int64_t)j * rowlen;
        const uint32_t *dj = dst16 + (int64_t)j * (rowlen >> gl);
        float *oj = stg + stage_row(rg, n, rowlen, i, j - rg.j0);
        for (uint32_t o = o0 + threadIdx.x * 4; o < o1; o += blockDim.x * 4) {
            const uint2 packed = *reinterpret_cast<const uint2 *>(sj + o);
            const int64_t at = stage_pos(rg, n, dj[o >> gl]) + (o & ((1u << gl) - 1u));
            const uint32_t s0 = packed.x & 0xffffu, s1 = packed.x >> 16, s2 = packed.y & 0xffffu, s3 = packed.y >> 16;
            float4 v;
            v.x = (s0 == kSrcPad) ? 0.f : tilebuf[s0 & 0x7fffu]; v.x = (s0 & 0x8000u) ? -v.x : v.x;
            v.y = (s1 == kSrcPad) ? 0.f : tilebuf[s1 & 0x7fffu]; v.y = (s1 & 0x8000u) ? -v.y : v.y;
            v.z = (s2 == kSrcPad) ? 0.f : tilebuf[s2 & 0x7fffu]; v.z = (s2 & 0x8000u) ? -v.z : v.z;
            v.w = (s3 == kSrcPad) ? 0.f : tilebuf[s3 & 0x7fffu]; v.w = (s3 & 0x8000u) ? -v.w : v.w;
            store_stream(reinterpret_cast<float4 *>(oj + at), v);
        }
    }
}

// v and vhat on I_{t-1} after k_head_scatter_w has decayed them: h = mean over the workers of g (summed in
// worker order, as everywhere), v += (1 - beta2) h^2, vhat = max(vhat, v)   (Alg. 2, master lines)
__global__ void __launch_bounds__(256)
k_head_sparse_v(const float *__restrict__ g, const int32_t *__restrict__ idx, int64_t k_sel, int32_t n, int64_t d,
                float omb2, float *__restrict__ v, float *__restrict__ vhat)
{
    const int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q >= k_sel) return;
    const int64_t l = idx[q];
    float gs = 0.0f;
    for (int32_t i0 = 0; i0 < n; i0 += 8) {                          // eight loads in flight, added in worker order
        float val[8];
#pragma unroll
        for (int z = 0; z < 8; ++z) {
            const int32_t i = (i0 + z < n) ? (i0 + z) : (n - 1);
            val[z] = g[(int64_t)i * d + l];
        }
#pragma unroll
        for (int z = 0; z < 8; ++z)
            if (i0 + z < n) gs = (i0 + z == 0) ? val[z] : (gs + val[z]);
    }
    const float h = (gs / (float)n);
    const float vv = (v[l] + (omb2 * (h * h)));
    v[l] = vv;
    if (vv > vhat[l]) vhat[l] = vv;
}

// the same with 32 lanes per coordinate for many workers (see k_gather_wide)
__global__ void __launch_bounds__(256)
k_head_sparse_v_wide(const float *__restrict__ g, const int32_t *__restrict__ idx, int64_t k_sel, int32_t n,
                     int64_t d, float omb2, float *__restrict__ v, float *__restrict__ vhat)
{
    __shared__ float vals[kWideCoords * kMaxWorkers];
    const int ql = threadIdx.x >> 5, wl = threadIdx.x & 31;
    const int64_t q = blockIdx.x * (int64_t)kWideCoords + ql;
    const int64_t l = q < k_sel ? idx[q] : 0;
    if (q < k_sel)
        for (int32_t i = wl; i < n; i += 32) vals[ql * n + i] = g[(int64_t)i * d + l];
    __syncthreads();
    if (q < k_sel && wl == 0) {
        float gs = vals[ql * n];
        for (int32_t i = 1; i < n; ++i) gs = (gs + vals[ql * n + i]);
        const float h = (gs / (float)n);
        const float vv = (v[l] + (omb2 * (h * h)));
        v[l] = vv;
        if (vv > vhat[l]) vhat[l] = vv;
    }
}

// the same from the gradients the per-worker head has left in gsel[n][k_sel] (by rank in the index set): no gathers
__global__ void __launch_bounds__(256)
k_head_sparse_v_sel(const float *__restrict__ gsel, const int32_t *__restrict__ idx, int64_t k_sel, int32_t n, float omb2,
                    float *__restrict__ v, float *__restrict__ vhat)
{
    const int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q >= k_sel) return;
    const int64_t l = idx[q];
    float gs = gsel[q];
    for (int32_t i = 1; i < n; ++i) gs = (gs + gsel[(int64_t)i * k_sel + q]);
    const float h = (gs / (float)n);
    const float vv = (v[l] + (omb2 * (h * h)));
    v[l] = vv;
    if (vv > vhat[l]) vhat[l] = vv;
}

// ... with 32 lanes per coordinate for many workers
__global__ void __launch_bounds__(256)
k_head_sparse_v_sel_wide(const float *__restrict__ gsel, const int32_t *__restrict__ idx, int64_t k_sel, int32_t n,
                         float omb2, float *__restrict__ v, float *__restrict__ vhat)
{
    __shared__ float vals[kWideCoords * kMaxWorkers];
    const int ql = threadIdx.x >> 5, wl = threadIdx.x & 31;
    const int64_t q = blockIdx.x * (int64_t)kWideCoords + ql;
    if (q < k_sel)
        for (int32_t i = wl; i < n; i += 32) vals[ql * n + i] = gsel[(int64_t)i * k_sel + q];
    __syncthreads();
    if (q < k_sel && wl == 0) {
        const int64_t l = idx[q];
        float gs = vals[ql * n];
        for (int32_t i = 1; i < n; ++i) gs = (gs + vals[ql * n + i]);
        const float h = (gs / (float)n);
        const float vv = (v[l] + (omb2 * (h * h)));
        v[l] = vv;
        if (vv > vhat[l]) vhat[l] = vv;
    }
}

// ------------------------------------------------------------------------------------------
// pass 2: per (worker, row, bin), add the bin's stream into an LDS window, chunk by chunk
// ------------------------------------------------------------------------------------------
// The n workers of one (row, bin) are placed on the same XCD in consecutive slots, so that the meta
// words they share are read from HBM once and then served by that XCD's L2.
template <int THREADS, int UNROLL>
__global__ void __launch_bounds__(THREADS)
k_bin_accumulate(const float *__restrict__ stg, const uint32_t *__restrict__ meta,
                 const uint32_t *__restrict__ binbase, float *__restrict__ S, int32_t n, RowGroup rg, RowSel sel,
                 int64_t c, int win_log2, int64_t nbins, int64_t rowlen)
{
    constexpr int CH = THREADS * UNROLL;
    extern __shared__ float lds[];
    const int W = 1 << win_log2;
    float *win = lds;
    uint2 *xbuf = reinterpret_cast<uint2 *>(lds + W);               // [2][CH]: (value bits, meta word)
    const int64_t id = blockIdx.x;
    const int64_t slot = id / kNumXcd;
    const int64_t group = (id % kNumXcd) + kNumXcd * (slot / n);     // (row, bin) index
    const int32_t i = (int32_t)(slot % n);
    if (group >= (int64_t)sel.cnt * nbins) return;
    const int32_t j = sel.row[group / nbins], jj = j - rg.j0;
    const int64_t bin = group % nbins;
    for (int t = threadIdx.x; t < W; t += THREADS) win[t] = 0.f;
    const int64_t b0 = binbase[(int64_t)j * (nbins + 1) + bin], b1 = binbase[(int64_t)j * (nbins + 1) + bin + 1];
    // position b0 + x of the bin (x = chunk start + z * THREADS, a multiple of 32, plus the thread's index) is at
    // v[x * vmul + voff]
    const float *v = stg + stage_row(rg, n, rowlen, i, jj) + stage_pos(rg, n, (uint32_t)b0);
    const int64_t vmul = rg.ilv ? n : 1;
    const int64_t voff = stage_pos(rg, n, threadIdx.x);
    const uint32_t *m = meta + (int64_t)j * rowlen + b0;
    const int64_t nchunk = (b1 - b0) / CH;
    const uint32_t wmask = (uint32_t)W - 1u;
    // Register ring of kAccDepth chunks: once chunk q has been processed its registers receive chunk
    // q + kAccDepth.  Every load of the ring is issued unconditionally and in a fixed order (past the end of the
    // bin the last chunk is read again, which costs no HBM traffic; the scheduling barriers keep the groups in
    // program order), and straight into the registers the loop carries: the compiler can then wait for exactly
    // the oldest group, with kAccDepth - 1 younger groups still in flight.  With loads under a condition, or
    // into temporaries copied at the loop end, it waits for all of them.
    float rv[kAccDepth][UNROLL];
    uint32_t rm[kAccDepth][UNROLL];
    if (nchunk > 0) {                                                // uniform over the workgroup
        const int64_t last = nchunk - 1;
#pragma unroll
        for (int s = 0; s < kAccDepth; ++s) {
            const int64_t qs = s < last ? s : last;
#pragma unroll
            for (int z = 0; z < UNROLL; ++z) {
                rv[s][z] = __builtin_nontemporal_load(v + (qs * CH + z * THREADS) * vmul + voff);
                rm[s][z] = m[qs * CH + z * THREADS + threadIdx.x];
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        for (int64_t q0 = 0; q0 < nchunk; q0 += kAccDepth) {
#pragma unroll
            for (int s = 0; s < kAccDepth; ++s) {
                const int64_t q = q0 + s;
                if (q < nchunk) {                                    // uniform over the workgroup
                    uint2 *xb = xbuf + (q & 1) * CH;
#pragma unroll
                    for (int z = 0; z < UNROLL; ++z)
                        xb[z * THREADS + threadIdx.x] = make_uint2(__float_as_uint(rv[s][z]), rm[s][z]);
                    __syncthreads();   // also orders the previous chunk's window updates before this chunk's
#pragma unroll
                    for (int z = 0; z < UNROLL; ++z) {
                        uint32_t word = rm[s][z];
                        if (!(word & kMetaNotFirst)) {
                            const uint32_t w = word & wmask;
                            float x = win[w] + rv[s][z];
                            while (word & kMetaHasNext) {
                                uint2 e = xb[(word >> kMetaNextShift) & (CH - 1)];
                                x = x + __uint_as_float(e.x);
                                word = e.y;
                            }
                            win[w] = x;
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                const int64_t qn = (q + kAccDepth) < last ? (q + kAccDepth) : last;
#pragma unroll
                for (int z = 0; z < UNROLL; ++z) {
                    rv[s][z] = __builtin_nontemporal_load(v + (qn * CH + z * THREADS) * vmul + voff);
                    rm[s][z] = m[qn * CH + z * THREADS + threadIdx.x];
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    __syncthreads();
    const int64_t base = bin << win_log2;
    float *out = S + ((int64_t)i * rg.r + j) * c + base;
    const int64_t lim = (c - base) < W ? (c - base) : W;
    for (int t = threadIdx.x; t < lim; t += THREADS) out[t] = win[t];
}

// Variant with 16-byte loads (1024 threads, chunks of 2048 positions): the lower half of the workgroup streams
// the values, the upper half the meta words, four consecutive positions per thread and load; they meet in the
// LDS exchange buffers (values and meta words in arrays of their own), from which every thread then takes two
// consecutive positions and works as in k_bin_accumulate.  Same order of additions, same results.
__global__ void __launch_bounds__(1024)
k_bin_accumulate_q(const float *__restrict__ stg, const uint32_t *__restrict__ meta,
                   const uint32_t *__restrict__ binbase, float *__restrict__ S, int32_t n, RowGroup rg, RowSel sel,
                   int64_t c, int win_log2, int64_t nbins, int64_t rowlen)
{
    constexpr int CH = 2048;
    extern __shared__ float lds[];
    const int W = 1 << win_log2;
    float *win = lds;
    uint32_t *xv = reinterpret_cast<uint32_t *>(lds + W);            // [2][CH] value bits
    uint32_t *xm = xv + 2 * CH;                                      // [2][CH] meta words
    const int64_t id = blockIdx.x;
    const int64_t slot = id / kNumXcd;
    const int64_t group = (id % kNumXcd) + kNumXcd * (slot / n);     // (row, bin) index
    const int32_t i = (int32_t)(slot % n);
    if (group >= (int64_t)sel.cnt * nbins) return;
    const int32_t j = sel.row[group / nbins], jj = j - rg.j0;
    const int64_t bin = group % nbins;
    for (int t = threadIdx.x; t < W; t += 1024) win[t] = 0.f;
    const int64_t b0 = binbase[(int64_t)j * (nbins + 1) + bin], b1 = binbase[(int64_t)j * (nbins + 1) + bin + 1];
    const bool is_meta = threadIdx.x >= 512;                         // uniform over a wavefront
    const uint32_t tt = threadIdx.x & 511u;
    // this thread's stream: position b0 + x + 4 tt of the bin is at src[x * mul + off]
    const uint32_t *src;
    int64_t mul;
    if (is_meta) {
        src = meta + (int64_t)j * rowlen + b0 + 4 * tt;
        mul = 1;
    } else {
        src = reinterpret_cast<const uint32_t *>(stg) + stage_row(rg, n, rowlen, i, jj) + stage_pos(rg, n, (uint32_t)b0) +
              stage_pos(rg, n, 4 * tt);
        mul = rg.ilv ? n : 1;
    }
    uint32_t *xmine = (is_meta ? xm : xv) + 4 * tt;
    const int64_t nchunk = (b1 - b0) / CH;
    const uint32_t wmask = (uint32_t)W - 1u;
    typedef uint32_t vec4u __attribute__((ext_vector_type(4)));
    vec4u ring[kAccDepth];
    auto fetch = [&](int64_t q) -> vec4u {
        const vec4u *p = reinterpret_cast<const vec4u *>(src + q * CH * mul);
        // plain loads for both halves: a streaming hint on the meta words would keep the n workers from sharing
        // them through the L2 (measured: 5.3 instead of 4.6 ms), and the compiler folds the two halves' loads
        // into one instruction, so the values cannot carry a hint of their own
        return *p;
    };
    if (nchunk > 0) {                                                // uniform over the workgroup
        const int64_t last = nchunk - 1;
#pragma unroll
        for (int s = 0; s < kAccDepth; ++s) {
            ring[s] = fetch(s < last ? s : last);
            __builtin_amdgcn_sched_barrier(0);
        }
        for (int64_t q0 = 0; q0 < nchunk; q0 += kAccDepth) {
#pragma unroll
            for (int s = 0; s < kAccDepth; ++s) {
                const int64_t q = q0 + s;
                if (q < nchunk) {                                    // uniform over the workgroup
                    const int half = (int)(q & 1) * CH;
                    *reinterpret_cast<vec4u *>(xmine + half) = ring[s];
                    __syncthreads();   // also orders the previous chunk's window updates before this chunk's
                    const uint2 pv = *reinterpret_cast<const uint2 *>(xv + half + 2 * threadIdx.x);
                    const uint2 pm = *reinterpret_cast<const uint2 *>(xm + half + 2 * threadIdx.x);
                    const uint32_t vals[2] = {pv.x, pv.y}, words[2] = {pm.x, pm.y};
#pragma unroll
                    for (int z = 0; z < 2; ++z) {
                        uint32_t word = words[z];
                        if (!(word & kMetaNotFirst)) {
                            const uint32_t w = word & wmask;
                            float x = win[w] + __uint_as_float(vals[z]);
                            while (word & kMetaHasNext) {
                                const uint32_t at = (word >> kMetaNextShift) & (CH - 1);
                                x = x + __uint_as_float(xv[half + at]);
                                word = xm[half + at];
                            }
                            win[w] = x;
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                ring[s] = fetch((q + kAccDepth) < last ? (q + kAccDepth) : last);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    __syncthreads();
    const int64_t base = bin << win_log2;
    float *out = S + ((int64_t)i * rg.r + j) * c + base;
    const int64_t lim = (c - base) < W ? (c - base) : W;
    for (int t = threadIdx.x; t < lim; t += 1024) out[t] = win[t];
}

// Variant reading chunk records instead of meta words (1024 threads, chunks of 4096 positions, windows of up to 2^15
// buckets).  A thread owns four consecutive positions per chunk and keeps their values and codes in registers: one
// 16-byte streaming load of the values, one 8-byte load of the codes, and -- every thread pair (2e, 2e + 1) -- the
// 4-byte entry of chain e (the records are shared by the n workers of a (row, bin) through the L2).  Per chunk: the
// positions that share their bucket with another position of the chunk (about an eighth with 2^15 windows) put their
// values into a small LDS array at their rank; after the one barrier every other position adds its value to its
// bucket, a plain read-modify-write since nothing else touches that bucket before the next barrier, and thread 2e adds
// the values of chain e to the chain's bucket in rank order, which is stream order.  The buckets of the chains and of
// the single positions are disjoint, so the two need no barrier between them.  Every wave does the same work (a
// version in which the first two waves fetched the entries into LDS and the first eight processed the chains ran
// at the same speed with three copies of the loop).  Same order of additions per bucket, hence the same results,
// as k_bin_accumulate.
// Every load of the ring is issued unconditionally and in a fixed order, straight into the registers the loop
// carries, so that the compiler waits for exactly the oldest chunk.
__global__ void __launch_bounds__(1024)
k_bin_accumulate_r(const float *__restrict__ stg, const uint32_t *__restrict__ rec,
                   const uint32_t *__restrict__ binbase, float *__restrict__ S, int32_t n, RowGroup rg, RowSel sel,
                   int64_t c, int win_log2, int64_t nbins, int64_t rowlen)
{
    constexpr int CH = kRecChunk;
    constexpr int kMv = kRecRanks + kRecPadRanks;
    extern __shared__ float lds[];
    const int W = 1 << win_log2;
    float *win = lds;
    float *mv = lds + W;                                             // [2][kMv] values of chain positions, by chunk parity
    const int64_t id = blockIdx.x;
    const int64_t slot = id / kNumXcd;
    const int64_t group = (id % kNumXcd) + kNumXcd * (slot / n);     // (row, bin) index
    const int32_t i = (int32_t)(slot % n);
    if (group >= (int64_t)sel.cnt * nbins) return;
    const int32_t j = sel.row[group / nbins], jj = j - rg.j0;
    const int64_t bin = group % nbins;
    const int64_t b0 = binbase[(int64_t)j * (nbins + 1) + bin], b1 = binbase[(int64_t)j * (nbins + 1) + bin + 1];
    const int64_t nchunk = (b1 - b0) / CH;                           // bins are whole chunks (see plan_create)
    for (int t = threadIdx.x; t < W; t += 1024) win[t] = 0.f;
    if (nchunk > 0) {                                                // uniform over the workgroup
        const uint32_t t = threadIdx.x;
        // this thread's four positions of chunk q: values at vsrc[q * vstride], codes at csrc[q * (kRecWords / 2)],
        // the entry of chain t / 2 at esrc[q * kRecWords]
        const vec4f *vsrc = reinterpret_cast<const vec4f *>(stg + stage_row(rg, n, rowlen, i, jj) +
                                                            stage_pos(rg, n, (uint32_t)b0) + stage_pos(rg, n, 4 * t));
        const int64_t vstride = (int64_t)(CH / 4) * (rg.ilv ? n : 1);
        const uint32_t *r0 = rec + ((int64_t)j * (rowlen / CH) + b0 / CH) * kRecWords;
        const uint2 *csrc = reinterpret_cast<const uint2 *>(r0) + t;
        const uint32_t *esrc = r0 + kRecCodeWords + (t >> 1);
        const bool chain_thread = (t & 1u) == 0;
        vec4f rv[kRecDepth];
        uint2 rc[kRecDepth];
        uint32_t re[kRecDepth];
        const int64_t last = nchunk - 1;
#pragma unroll
        for (int s = 0; s < kRecDepth; ++s) {
            const int64_t qs = s < last ? s : last;
            rv[s] = __builtin_nontemporal_load(vsrc + qs * vstride);
            rc[s] = csrc[qs * (kRecWords / 2)];
            re[s] = esrc[qs * kRecWords];
            __builtin_amdgcn_sched_barrier(0);
        }
        for (int64_t q0 = 0; q0 < nchunk; q0 += kRecDepth) {
#pragma unroll
            for (int s = 0; s < kRecDepth; ++s) {
                const int64_t q = q0 + s;
                if (q < nchunk) {                                    // uniform over the workgroup
                    float *mvp = mv + (s & 1) * kMv;                  // q0 is even: the chunk's parity is that of s
                    const float vals[4] = {rv[s].x, rv[s].y, rv[s].z, rv[s].w};
                    const uint32_t codes[4] = {rc[s].x & 0xffffu, rc[s].x >> 16, rc[s].y & 0xffffu, rc[s].y >> 16};
#pragma unroll
                    for (int z = 0; z < 4; ++z)
                        if (codes[z] >= kCodeChain) mvp[codes[z] & kCodeRankMask] = vals[z];
                    __syncthreads();   // also orders the previous chunk's window updates before this chunk's
#pragma unroll
                    for (int z = 0; z < 4; ++z)
                        if (codes[z] < kCodeChain) win[codes[z]] = win[codes[z]] + vals[z];
                    const uint32_t word = re[s];
                    const uint32_t cnt = chain_thread ? word >> 25 : 0u;
                    if (cnt) {
                        const uint32_t w = word & 0x7fffu;
                        const float *mc = mvp + ((word >> 15) & (uint32_t)(kRecRanks - 1));
                        float x = win[w];
                        for (uint32_t o = 0; o < cnt; ++o) x = x + mc[o];
                        win[w] = x;
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                // (refilling the registers before the chunk is processed instead of after it changes nothing)
                const int64_t qn = (q + kRecDepth) < last ? (q + kRecDepth) : last;
                rv[s] = __builtin_nontemporal_load(vsrc + qn * vstride);
                rc[s] = csrc[qn * (kRecWords / 2)];
                re[s] = esrc[qn * kRecWords];
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    __syncthreads();
    const int64_t base = bin << win_log2;
    float *out = S + ((int64_t)i * rg.r + j) * c + base;
    const int64_t lim = (c - base) < W ? (c - base) : W;
    for (int t = threadIdx.x; t < lim; t += 1024) out[t] = win[t];
}

// ------------------------------------------------------------------------------------------
// the plan run backwards, for the recovery of stage 3 (Sec. II-C: the row estimates s_j(l) S[j,h_j(l)])
// ------------------------------------------------------------------------------------------
// Reading S[j][h_j(l)] for every coordinate is the same permutation as the sketch, in the other
// direction: k_bin_lookup gives one workgroup per (row, bin), which holds the bin's window of the mean
// table in LDS and writes the looked-up value of every stream position (contiguous); k_bin_collect
// gives one workgroup per tile, which brings the values of its slots back into coordinate order through
// LDS, applies the signs, and writes rowest[row][l] = s_row(l) * S[row][h_row(l)] (contiguous).
__global__ void __launch_bounds__(1024)
k_bin_lookup(const float *__restrict__ S_mean, const uint16_t *__restrict__ wlow,
             const uint32_t *__restrict__ binbase, float *__restrict__ lk, int64_t c, int win_log2,
             int64_t nbins, int64_t rowlen, int32_t j0, int32_t nsplit)
{
    extern __shared__ float win[];
    const int W = 1 << win_log2;
    const int64_t bin = blockIdx.x / nsplit;                         // nsplit workgroups share a bin's stream
    const int64_t part = blockIdx.x % nsplit;
    const int j = j0 + (int)blockIdx.y;
    const int64_t base = bin << win_log2;
    const float *Sj = S_mean + (int64_t)j * c + base;
    const int64_t lim = (c - base) < W ? (c - base) : W;
    for (int t = threadIdx.x; t < W; t += blockDim.x) win[t] = t < lim ? Sj[t] : 0.f;
    __syncthreads();
    const int64_t b0 = binbase[(int64_t)j * (nbins + 1) + bin], b1 = binbase[(int64_t)j * (nbins + 1) + bin + 1];
    // 4 positions per thread and step: their 2-byte buckets in one 8-byte load, one 16-byte store; a wavefront
    // reads and writes whole lines (bins start and end on multiples of the chunk, at least 64 positions)
    const uint2 *m4 = reinterpret_cast<const uint2 *>(wlow + (int64_t)j * rowlen + b0);
    float4 *o4 = reinterpret_cast<float4 *>(lk + (int64_t)blockIdx.y * rowlen + b0);
    const int64_t n4 = (b1 - b0) >> 2;
    const int64_t piece = (n4 + nsplit - 1) / nsplit;
    const int64_t q1 = (part + 1) * piece < n4 ? (part + 1) * piece : n4;
    // four steps' buckets are fetched before the first is used (clamped addresses past the piece's end: read, not
    // used), so that a thread has 32 bytes in flight instead of 8
    constexpr int kAhead = 4;
    for (int64_t q = part * piece + threadIdx.x; q < q1; q += (int64_t)blockDim.x * kAhead) {
        uint2 w[kAhead];
#pragma unroll
        for (int z = 0; z < kAhead; ++z) {
            const int64_t qz = q + (int64_t)z * blockDim.x;
            w[z] = load_stream2(m4 + (qz < q1 ? qz : q1 - 1));
        }
#pragma unroll
        for (int z = 0; z < kAhead; ++z) {
            const int64_t qz = q + (int64_t)z * blockDim.x;
            if (qz < q1)
                store_stream(o4 + qz, make_float4(win[w[z].x & 0xffffu], win[w[z].x >> 16], win[w[z].y & 0xffffu],
                                                  win[w[z].y >> 16]));
        }
    }
}

__global__ void __launch_bounds__(1024)
k_bin_collect(const float *__restrict__ lk, const uint16_t *__restrict__ srcp, const uint32_t *__restrict__ dst16,
              const uint32_t *__restrict__ pbase, float *__restrict__ rowest, int32_t j0, int32_t rj, int64_t d,
              int tile_log2, int64_t ntile, int64_t rowlen, int gl)
{
    extern __shared__ float rowbuf[];                                // [2][L]
    const int L = 1 << tile_log2;
    const int64_t tile = blockIdx.x;
    const int64_t l0 = tile << tile_log2;
    const bool vec = (d & 3) == 0;
    for (int32_t j = j0; j < j0 + rj; ++j) {
        float *buf = rowbuf + (j & 1) * L;
        const uint32_t o0 = pbase[(int64_t)j * (ntile + 1) + tile], o1 = pbase[(int64_t)j * (ntile + 1) + tile + 1];
        const uint16_t *sj = srcp + (int64_t)j * rowlen;
        const uint32_t *dj = dst16 + (int64_t)j * (rowlen >> gl);
        const float *lj = lk + (int64_t)(j - j0) * rowlen;
        for (uint32_t o = o0 + threadIdx.x * 4; o < o1; o += blockDim.x * 4) {
            const uint2 packed = *reinterpret_cast<const uint2 *>(sj + o);
            const uint32_t at = dj[o >> gl] + (o & ((1u << gl) - 1u));
            const float4 v = load_stream(reinterpret_cast<const float4 *>(lj + at));
            const uint32_t s0 = packed.x & 0xffffu, s1 = packed.x >> 16, s2 = packed.y & 0xffffu,
                           s3 = packed.y >> 16;
            if (s0 != kSrcPad) buf[s0 & 0x7fffu] = (s0 & 0x8000u) ? -v.x : v.x;
            if (s1 != kSrcPad) buf[s1 & 0x7fffu] = (s1 & 0x8000u) ? -v.y : v.y;
            if (s2 != kSrcPad) buf[s2 & 0x7fffu] = (s2 & 0x8000u) ? -v.z : v.z;
            if (s3 != kSrcPad) buf[s3 & 0x7fffu] = (s3 & 0x8000u) ? -v.w : v.w;
        }
        __syncthreads();   // the other buffer is free again once every thread has passed this barrier
        float *out = rowest + (int64_t)j * d + l0;
        if (vec) {
            for (int p = threadIdx.x * 4; p < L && l0 + p < d; p += blockDim.x * 4)
                store_stream(reinterpret_cast<float4 *>(out + p), *reinterpret_cast<const float4 *>(buf + p));
        } else {
            for (int p = threadIdx.x; p < L && l0 + p < d; p += blockDim.x) out[p] = buf[p];
        }
    }
}

// k_bin_collect with the median of Sec. II-C and the 1/sqrt(vhat) scaling of Alg. 3 fused in: each thread
// keeps the R row estimates of its 4 * ITERS coordinates in registers (tiles of at most 4096 * ITERS
// coordinates), so the per-row estimates never go to memory.
constexpr int kCollectAhead = 4;

template <int R, int ITERS>
__global__ void __launch_bounds__(kFusedThreads)
k_bin_collect_median(const float *__restrict__ lk, const uint16_t *__restrict__ srcp,
                     const uint32_t *__restrict__ dst16, const uint32_t *__restrict__ pbase,
                     const float *__restrict__ vhat, float *__restrict__ est, int64_t d, int tile_log2,
                     int64_t ntile, int64_t rowlen, int gl, uint32_t *__restrict__ hist)
{
    extern __shared__ float rowbuf[];                                // [2][L], at least kHistBins words in all
    const int L = 1 << tile_log2;
    const int64_t tile = blockIdx.x;
    const int64_t l0 = tile << tile_log2;
    float a[R][ITERS][4];
    // The loads of a row's first kCollectAhead sweeps are issued before the barrier of the row before it, so that
    // they are in flight while the workgroup (the only one on its compute unit) waits and empties the LDS buffer.
    // Past the tile's last slot group they read that group again (in bounds; not used).
    uint2 pk[kCollectAhead];
    float4 pv[kCollectAhead];
    uint32_t o0 = 0, o1 = 0;
    auto issue = [&](int j) {
        o0 = pbase[(int64_t)j * (ntile + 1) + tile];
        o1 = pbase[(int64_t)j * (ntile + 1) + tile + 1];
        const uint16_t *sj = srcp + (int64_t)j * rowlen;
        const uint32_t *dj = dst16 + (int64_t)j * (rowlen >> gl);
        const float *lj = lk + (int64_t)j * rowlen;
#pragma unroll
        for (int s = 0; s < kCollectAhead; ++s) {
            const uint32_t o = o0 + (uint32_t)(s * kFusedThreads + (int)threadIdx.x) * 4u;
            const uint32_t oc = o < o1 ? o : o1 - 4u;                // a tile has at least one group of 4 slots
            pk[s] = load_stream2(reinterpret_cast<const uint2 *>(sj + oc));
            pv[s] = load_stream(reinterpret_cast<const float4 *>(lj + dj[oc >> gl] + (oc & ((1u << gl) - 1u))));
        }
    };
    auto place = [&](float *buf, const uint2 packed, const float4 v) {
        const uint32_t s0 = packed.x & 0xffffu, s1 = packed.x >> 16, s2 = packed.y & 0xffffu, s3 = packed.y >> 16;
        if (s0 != kSrcPad) buf[s0 & 0x7fffu] = (s0 & 0x8000u) ? -v.x : v.x;
        if (s1 != kSrcPad) buf[s1 & 0x7fffu] = (s1 & 0x8000u) ? -v.y : v.y;
        if (s2 != kSrcPad) buf[s2 & 0x7fffu] = (s2 & 0x8000u) ? -v.z : v.z;
        if (s3 != kSrcPad) buf[s3 & 0x7fffu] = (s3 & 0x8000u) ? -v.w : v.w;
    };
    issue(0);
#pragma unroll
    for (int j = 0; j < R; ++j) {
        float *buf = rowbuf + (j & 1) * L;
        const uint32_t b0 = o0, b1 = o1;
#pragma unroll
        for (int s = 0; s < kCollectAhead; ++s)
            if (b0 + (uint32_t)(s * kFusedThreads + (int)threadIdx.x) * 4u < b1) place(buf, pk[s], pv[s]);
        {
            const uint16_t *sj = srcp + (int64_t)j * rowlen;
            const uint32_t *dj = dst16 + (int64_t)j * (rowlen >> gl);
            const float *lj = lk + (int64_t)j * rowlen;
            for (uint32_t o = b0 + (uint32_t)(kCollectAhead * kFusedThreads + (int)threadIdx.x) * 4u; o < b1;
                 o += kFusedThreads * 4) {
                const uint2 packed = load_stream2(reinterpret_cast<const uint2 *>(sj + o));
                const uint32_t at = dj[o >> gl] + (o & ((1u << gl) - 1u));
                place(buf, packed, load_stream(reinterpret_cast<const float4 *>(lj + at)));
            }
        }
        if (j + 1 < R) issue(j + 1);
        __syncthreads();   // the other buffer is free again once every thread has passed this barrier
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int p = (it * kFusedThreads + (int)threadIdx.x) * 4;
            float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
            if (p < L) q = *reinterpret_cast<const float4 *>(buf + p);
            a[j][it][0] = q.x; a[j][it][1] = q.y; a[j][it][2] = q.z; a[j][it][3] = q.w;
        }
    }
    // hist != null: the selection follows, and the histogram of the first radix digit of |est| (its top 11 bits)
    // is taken here, from the registers, instead of by a pass over the estimates of its own.  The row buffers are
    // free by now (every thread has copied its part of the last row) and hold the workgroup's histogram.
    uint32_t *lh = reinterpret_cast<uint32_t *>(rowbuf);
    if (hist) {
        __syncthreads();
        for (int b = threadIdx.x; b < kHistBins; b += kFusedThreads) lh[b] = 0;
        __syncthreads();
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int p = (it * kFusedThreads + (int)threadIdx.x) * 4;
        if (p < L && l0 + p < d) {
            float vh[4] = {1.f, 1.f, 1.f, 1.f};
            if (vhat) {
                const float4 q = *reinterpret_cast<const float4 *>(vhat + l0 + p);
                vh[0] = q.x; vh[1] = q.y; vh[2] = q.z; vh[3] = q.w;
            }
            float o[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                float col[R];
#pragma unroll
                for (int j = 0; j < R; ++j) col[j] = a[j][it][t];
                const float med = median_of<R>(col);
                o[t] = vhat ? (med / sqrtf(vh[t])) : med;
                if (hist) atomicAdd(&lh[(__float_as_uint(o[t]) & 0x7fffffffu) >> 20], 1u);
            }
            *reinterpret_cast<float4 *>(est + l0 + p) = make_float4(o[0], o[1], o[2], o[3]);
        }
    }
    if (hist) {
        __syncthreads();
        for (int b = threadIdx.x; b < kHistBins; b += kFusedThreads)
            if (lh[b]) atomicAdd(&hist[b], lh[b]);
    }
}

// R * ITERS * 4 row estimates per thread must stay in registers: up to 6 rows with tiles of 2^14 coordinates,
// 12 rows with 2^13, 16 rows with 2^12
static int fused_median_iters(int32_t r, int tile_log2)
{
    if (r <= 6 && tile_log2 <= 14) return 4;
    if (r <= 12 && tile_log2 <= 13) return 2;
    if (r <= SAMS_MAX_ROWS && tile_log2 <= 12) return 1;
    return 0;
}
// (rows, ITERS) pairs that are instantiated: the ITERS fused_median_iters gives for that many rows
#define SAMS_FUSED_MEDIAN_VARIANTS(X)                                                              \
    X(1, 4) X(2, 4) X(3, 4) X(4, 4) X(5, 4) X(6, 4) X(7, 2) X(8, 2) X(9, 2) X(10, 2) X(11, 2) X(12, 2) \
    X(13, 1) X(14, 1) X(15, 1) X(16, 1)

// Workgroups per (row, bin) of the lookup: enough of them to give every compute unit a few, while a
// workgroup still has a good many positions per window it loads.
static int32_t lookup_split(const Plan &pl, int32_t rows)
{
    const int64_t groups = pl.nbins * rows;
    int64_t nsplit = (1024 + groups - 1) / groups;
    const int64_t per_bin = pl.rowlen / pl.nbins;                   // about the positions of one bin
    while (nsplit > 1 && per_bin / nsplit < (int64_t)8 << pl.win_log2) --nsplit;
    return (int32_t)(nsplit < 1 ? 1 : (nsplit > 64 ? 64 : nsplit));
}

int enqueue_estimates_planned_fused(sams_ctx *ctx, const float *S_mean, const float *vhat, float *est, bool *done,
                                    uint32_t *hist)
{
    Plan &pl = ctx->plan;
    *done = false;
    if (!pl.fused_median) return SAMS_OK;
    const int64_t L = (int64_t)1 << pl.tile_log2, W = (int64_t)1 << pl.win_log2;
    float *lk = pl.stg;
    pl.staged_u = nullptr;                                           // the looked-up values overwrite any staged vector
    {
        ProfScope ps(ctx, KID_BIN_LOOKUP);
        const int32_t nsplit = lookup_split(pl, ctx->r);
        hipLaunchKernelGGL(k_bin_lookup, dim3((unsigned)(pl.nbins * nsplit), (unsigned)ctx->r), dim3(1024),
                           (size_t)(W * 4), ctx->stream, S_mean, pl.wlow, pl.binbase, lk, ctx->c, pl.win_log2,
                           pl.nbins, pl.rowlen, 0, nsplit);
    }
    {
        ProfScope ps(ctx, KID_BIN_COLLECT);
        const size_t lds = (size_t)(2 * L * 4) > (size_t)kHistBins * 4 ? (size_t)(2 * L * 4) : (size_t)kHistBins * 4;
#define SAMS_CM(RR, IT)                                                                                   \
    case RR:                                                                                              \
        hipLaunchKernelGGL((k_bin_collect_median<RR, IT>), dim3((unsigned)pl.ntile), dim3(kFusedThreads), \
                           lds, ctx->stream, lk, pl.srcp, pl.dst16, pl.pbase, vhat, est,                   \
                           ctx->d, pl.tile_log2, pl.ntile, pl.rowlen, pl.grp_log2, hist);                 \
        break;
        switch (ctx->r) {
            SAMS_FUSED_MEDIAN_VARIANTS(SAMS_CM)
        }
#undef SAMS_CM
    }
    SAMS_HIP(hipGetLastError());
    *done = true;
    return SAMS_OK;
}

int enqueue_row_estimates_planned(sams_ctx *ctx, const float *S_mean, float *rowest)
{
    Plan &pl = ctx->plan;
    const int64_t L = (int64_t)1 << pl.tile_log2, W = (int64_t)1 << pl.win_log2;
    float *lk = pl.stg;                                              // the staging buffer is idle between two sketches
    pl.staged_u = nullptr;                                           // ... and whatever vector it held is overwritten
    const int64_t cap = (int64_t)ctx->n * pl.stage_rows;             // rows of looked-up values it can hold
    for (int32_t j0 = 0; j0 < ctx->r; j0 += (int32_t)cap) {
        const int32_t rj = (ctx->r - j0) < cap ? (ctx->r - j0) : (int32_t)cap;
        {
            ProfScope ps(ctx, KID_BIN_LOOKUP);
            const int32_t nsplit = lookup_split(pl, rj);
            hipLaunchKernelGGL(k_bin_lookup, dim3((unsigned)(pl.nbins * nsplit), (unsigned)rj), dim3(1024),
                               (size_t)(W * 4), ctx->stream, S_mean, pl.wlow, pl.binbase, lk, ctx->c, pl.win_log2,
                               pl.nbins, pl.rowlen, j0, nsplit);
        }
        {
            ProfScope ps(ctx, KID_BIN_COLLECT);
            hipLaunchKernelGGL(k_bin_collect, dim3((unsigned)pl.ntile), dim3(1024), (size_t)(2 * L * 4),
                               ctx->stream, lk, pl.srcp, pl.dst16, pl.pbase, rowest, j0, rj, ctx->d, pl.tile_log2,
                               pl.ntile, pl.rowlen, pl.grp_log2);
        }
    }
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
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
// The staging buffer as one range of virtual addresses backed by 1 GiB physical chunks picked at even distances over
// all free device memory.  Device memory is striped over the HBM stacks in coarse pieces: a buffer that is contiguous in
// physical memory reaches only part of the stacks (scattered 512-byte writes into it run at 5.4 TB/s), one scattered
// over all of physical memory reaches all (7.2 TB/s).  To pick the chunks the call holds nearly all free memory for a
// moment: every chunk the device can give is created, the wanted ones are mapped, the others released.
static void spread_free(Plan &pl)
{
    if (!pl.stg_chunks) return;
    hipMemGenericAllocationHandle_t *h = static_cast<hipMemGenericAllocationHandle_t *>(pl.stg_chunks);
    if (pl.stg) {
        (void)hipMemUnmap(pl.stg, (size_t)pl.stg_va_bytes);
        (void)hipMemAddressFree(pl.stg, (size_t)pl.stg_va_bytes);
    }
    for (int64_t q = 0; q < pl.stg_nchunks; ++q) (void)hipMemRelease(h[q]);
    delete[] h;
    pl.stg_chunks = nullptr;
    pl.stg = nullptr;
    pl.stg_nchunks = pl.stg_va_bytes = 0;
}

// SAMS_OK with pl.stg set, or SAMS_ENOMEM with nothing held (the caller then takes an ordinary allocation)
static int spread_alloc(sams_ctx *ctx, int64_t bytes)
{
    Plan &pl = ctx->plan;
    const size_t chunk = (size_t)1 << 30;
    const int64_t need = (int64_t)(((size_t)bytes + chunk - 1) / chunk);
    int dev = 0;
    size_t free_b = 0, total_b = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipMemGetInfo(&free_b, &total_b) != hipSuccess) {
        (void)hipGetLastError();
        return SAMS_ENOMEM;
    }
    hipMemAllocationProp prop = {};
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = dev;
    size_t gran = 0;
    if (hipMemGetAllocationGranularity(&gran, &prop, hipMemAllocationGranularityRecommended) != hipSuccess || gran == 0 ||
        chunk % gran != 0) {
        (void)hipGetLastError();
        return SAMS_ENOMEM;
    }
    const int64_t most = (int64_t)((double)free_b * 0.97 / (double)chunk);
    if (most < need) return SAMS_ENOMEM;
    hipMemGenericAllocationHandle_t *all = new (std::nothrow) hipMemGenericAllocationHandle_t[most];
    hipMemGenericAllocationHandle_t *kept = new (std::nothrow) hipMemGenericAllocationHandle_t[need];
    if (!all || !kept) {
        delete[] all;
        delete[] kept;
        return SAMS_ENOMEM;
    }
    int64_t made = 0;
    for (; made < most; ++made)
        if (hipMemCreate(&all[made], chunk, &prop, 0) != hipSuccess) {
            (void)hipGetLastError();
            break;
        }
    void *va = nullptr;
    bool ok = made >= need && hipMemAddressReserve(&va, (size_t)need * chunk, 0, nullptr, 0) == hipSuccess;
    int64_t mapped = 0;
    if (ok) {
        for (int64_t q = 0, next = 0; q < made; ++q) {
            const int64_t want = next < need ? (next * made + made / 2) / need : -1;   // evenly spaced, centred
            if (q == want) {
                kept[next] = all[q];
                if (ok && hipMemMap(static_cast<char *>(va) + (size_t)next * chunk, chunk, 0, all[q], 0) == hipSuccess)
                    ++mapped;
                else
                    ok = false;
                ++next;
            } else {
                (void)hipMemRelease(all[q]);
            }
        }
        if (ok) {
            hipMemAccessDesc ad = {};
            ad.location = prop.location;
            ad.flags = hipMemAccessFlagsProtReadWrite;
            ok = hipMemSetAccess(va, (size_t)need * chunk, &ad, 1) == hipSuccess;
        }
        if (!ok) {
            (void)hipGetLastError();
            if (mapped) (void)hipMemUnmap(va, (size_t)mapped * chunk);
            for (int64_t q = 0; q < need; ++q) (void)hipMemRelease(kept[q]);
            (void)hipMemAddressFree(va, (size_t)need * chunk);
        }
    } else {
        (void)hipGetLastError();
        for (int64_t q = 0; q < made; ++q) (void)hipMemRelease(all[q]);
        if (va) (void)hipMemAddressFree(va, (size_t)need * chunk);
    }
    delete[] all;
    if (!ok) {
        delete[] kept;
        return SAMS_ENOMEM;
    }
    pl.stg = static_cast<float *>(va);
    pl.stg_chunks = kept;
    pl.stg_nchunks = need;
    pl.stg_va_bytes = (int64_t)((size_t)need * chunk);
    ctx->scratch_bytes += pl.stg_va_bytes;
    return SAMS_OK;
}

static int dev_alloc(sams_ctx *ctx, void **p, int64_t bytes)
{
    hipError_t e = hipMalloc(p, (size_t)(bytes > 0 ? bytes : 4));
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        (void)hipGetLastError();
        return SAMS_ENOMEM;
    }
    ctx->scratch_bytes += bytes;
    return SAMS_OK;
}

// (threads, unroll) variants of the accumulate kernel, selected by acc_threads / chunk_log2
template <int TH, int UN>
static int launch_acc(sams_ctx *ctx, float *S_workers, RowGroup rg, RowSel sel, bool set_attr)
{
    Plan &pl = ctx->plan;
    const size_t lds = ((size_t)4 << pl.win_log2) + (size_t)2 * TH * UN * sizeof(uint2);
    if (set_attr) {
        SAMS_HIP(hipFuncSetAttribute((const void *)k_bin_accumulate<TH, UN>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes));
        return SAMS_OK;
    }
    const int64_t groups = (int64_t)sel.cnt * pl.nbins;
    const int64_t gpad = (groups + kNumXcd - 1) / kNumXcd * kNumXcd;
    ProfScope ps(ctx, KID_BIN_ACCUMULATE);
    hipLaunchKernelGGL((k_bin_accumulate<TH, UN>), dim3((unsigned)(gpad * ctx->n)), dim3(TH), lds, ctx->stream,
                       pl.stg, pl.meta, pl.binbase, S_workers, ctx->n, rg, sel, ctx->c, pl.win_log2, pl.nbins,
                       pl.rowlen);
    return SAMS_OK;
}

// Pass 2 for the rows of one row group: the rows whose chunks fit the record format (pl.rec_mask) go to the kernel
// that reads chunk records, the others to a kernel that reads meta words.
static int dispatch_acc(sams_ctx *ctx, float *S_workers, RowGroup rg, bool set_attr)
{
    const Plan &pl = ctx->plan;
    const int un = (1 << pl.chunk_log2) / pl.acc_threads;
    if (set_attr) {
        SAMS_HIP(hipFuncSetAttribute((const void *)k_bin_accumulate_q, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes));
        SAMS_HIP(hipFuncSetAttribute((const void *)k_bin_accumulate_r, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes));
    }
    RowSel with_rec = {0, {0}}, with_meta = {0, {0}};
    for (int32_t j = rg.j0; j < rg.j0 + rg.rj; ++j) {
        RowSel &dst = ((pl.rec_mask >> j) & 1u) ? with_rec : with_meta;
        dst.row[dst.cnt++] = (int8_t)j;
    }
    if (!set_attr && with_rec.cnt > 0) {
        const int64_t groups = (int64_t)with_rec.cnt * pl.nbins;
        const int64_t gpad = (groups + kNumXcd - 1) / kNumXcd * kNumXcd;
        const size_t lds = ((size_t)4 << pl.win_log2) + (size_t)2 * (kRecRanks + kRecPadRanks) * 4;
        ProfScope ps(ctx, KID_BIN_ACCUMULATE);
        hipLaunchKernelGGL(k_bin_accumulate_r, dim3((unsigned)(gpad * ctx->n)), dim3(1024), lds, ctx->stream, pl.stg,
                           pl.rec, pl.binbase, S_workers, ctx->n, rg, with_rec, ctx->c, pl.win_log2, pl.nbins, pl.rowlen);
    }
    if (!set_attr && with_meta.cnt == 0) return SAMS_OK;
    if (!set_attr && pl.acc_variant >= 1) {
        const int64_t groups = (int64_t)with_meta.cnt * pl.nbins;
        const int64_t gpad = (groups + kNumXcd - 1) / kNumXcd * kNumXcd;
        const size_t lds = ((size_t)4 << pl.win_log2) + (size_t)4 * 2048 * 4;
        ProfScope ps(ctx, KID_BIN_ACCUMULATE);
        hipLaunchKernelGGL(k_bin_accumulate_q, dim3((unsigned)(gpad * ctx->n)), dim3(1024), lds, ctx->stream, pl.stg,
                           pl.meta, pl.binbase, S_workers, ctx->n, rg, with_meta, ctx->c, pl.win_log2, pl.nbins, pl.rowlen);
        return SAMS_OK;
    }
#define SAMS_ACC(TH, UN) \
    if (pl.acc_threads == TH && un == UN) return launch_acc<TH, UN>(ctx, S_workers, rg, with_meta, set_attr);
    SAMS_ACC(1024, 1) SAMS_ACC(1024, 2) SAMS_ACC(512, 1) SAMS_ACC(512, 2) SAMS_ACC(512, 4)
    SAMS_ACC(256, 1) SAMS_ACC(256, 2) SAMS_ACC(256, 4) SAMS_ACC(256, 8)
#undef SAMS_ACC
    return SAMS_EINVAL;
}

int plan_create(sams_ctx *ctx, const Tunables &tun)
{
    Plan &pl = ctx->plan;
    pl.win_log2 = tun.win_log2;
    pl.tile_log2 = tun.tile_log2;
    if (pl.tile_log2 == 0) {
        // automatic tile: 2^14 coordinates (2^13 above 6 rows, 2^12 above 12, so that a thread can keep the row
        // estimates of its coordinates in registers for the median), halved (down to 2^8) while pass 1 and the
        // dense update would have too few workgroups for the chip's 256 compute units: one per tile with
        // fuse_head = 1 (at least 256 wanted), one per (tile, worker) otherwise (at least 1024 wanted, the
        // recovery still has one per tile)
        pl.tile_log2 = ctx->r <= 6 ? 14 : (ctx->r <= 12 ? 13 : 12);
        const int64_t per_tile = tun.fuse_head == 1 ? 1 : ctx->n, want = tun.fuse_head == 1 ? 256 : 1024;
        while (pl.tile_log2 > 8 && ((ctx->d + ((int64_t)1 << pl.tile_log2) - 1) >> pl.tile_log2) * per_tile < want)
            --pl.tile_log2;
    }
    if (pl.win_log2 == 0) {
        // automatic window: the largest one (longest runs, least padding) that still leaves about eight
        // accumulate workgroups per compute unit (256 units); never more than the table needs
        pl.win_log2 = 15;
        while (pl.win_log2 > 12 &&
               (int64_t)ctx->n * ctx->r * ((ctx->c + ((int64_t)1 << pl.win_log2) - 1) >> pl.win_log2) < 2048)
            --pl.win_log2;
        while (pl.win_log2 < 15 && ((int64_t)1 << pl.win_log2) < ctx->c &&
               (((int64_t)1 << pl.tile_log2) << pl.win_log2) / ctx->c < 64)
            ++pl.win_log2;                                           // but keep runs of at least 64 positions
        // a small table under a short vector: nothing there is bound by bandwidth, and one workgroup per (worker, row)
        // would walk the whole vector chunk after chunk; smaller windows (down to 2^7 buckets) share that walk out
        if (ctx->c <= ((int64_t)1 << pl.win_log2) && ctx->d <= kOrderedSingleBinMaxD)
            while (pl.win_log2 > 7 &&
                   (int64_t)ctx->n * ctx->r * ((ctx->c + ((int64_t)1 << pl.win_log2) - 1) >> pl.win_log2) < 1024)
                --pl.win_log2;
    }
    // a 32K window leaves room for one workgroup per unit: 1024 threads, 2048-position chunks; smaller
    // windows run two or more 512-thread workgroups per unit with 1024-position chunks
    pl.chunk_log2 = tun.chunk_log2 ? tun.chunk_log2 : (pl.win_log2 >= 15 ? 11 : 10);
    pl.acc_threads = tun.acc_threads ? tun.acc_threads : (pl.win_log2 >= 15 ? 1024 : 512);
    pl.run_pad = tun.run_pad;
    pl.grp_log2 = tun.run_pad >= 16 ? 4 : (tun.run_pad == 8 ? 3 : 2);   // slot groups: the run padding, at most 16 slots
    pl.stage_ilv = tun.stage_interleave ? 1 : 0;
    pl.acc_wide = tun.acc_wide;
    pl.stage_rows = (tun.stage_rows <= 0 || tun.stage_rows > ctx->r) ? ctx->r : tun.stage_rows;
    const int64_t W = (int64_t)1 << pl.win_log2, L = (int64_t)1 << pl.tile_log2, CH = (int64_t)1 << pl.chunk_log2;
    pl.nbins = (ctx->c + W - 1) / W;
    // a table that fits one window: the binned machinery with a single bin keeps the order of the adds (one
    // workgroup per (worker, row) walks all d coordinates, fine while d is small); LDS atomics over
    // many workgroups do not, but scale with d
    const bool ordered_single = tun.sketch_path == 2 || (tun.sketch_path == 0 && ctx->d <= kOrderedSingleBinMaxD);
    pl.mode = (pl.nbins > 1 || ordered_single) ? PLAN_BINNED : PLAN_LDS_ROW;
    if (pl.mode == PLAN_LDS_ROW) {
        SAMS_HIP(hipFuncSetAttribute((const void *)k_sketch_lds, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes));
        return SAMS_OK;
    }
    // sort keys must fit 32 bits; LDS must hold a window plus the chunk exchange buffers
    if ((pl.nbins << pl.tile_log2) >= ((int64_t)1 << 32) - 1) return SAMS_EINVAL;
    if (pl.win_log2 + pl.chunk_log2 > 31 || pl.chunk_log2 > 11 || CH < pl.acc_threads) return SAMS_EINVAL;
    if (W * 4 + 2 * CH * 8 > 160 * 1024) return SAMS_EINVAL;
    pl.ntile = (ctx->d + L - 1) / L;
    pl.dpad = pl.ntile * L;
    const int64_t r = ctx->r, n = ctx->n, NB = pl.nbins;
    if (pl.tile_log2 > 14 || NB > 8192) return SAMS_EINVAL;          // kSrcPad; LDS prefix in k_plan_place
    SAMS_TRY(dev_alloc(ctx, (void **)&pl.binbase, r * (NB + 1) * 4));
    SAMS_TRY(dev_alloc(ctx, (void **)&pl.pbase, r * (pl.ntile + 1) * 4));
    // build-time only: tile-sorted sources, run starts, per-(bin, tile) offsets, totals, tile lengths
    uint16_t *src = nullptr, *bst = nullptr;
    uint32_t *off = nullptr, *total = nullptr, *tilelen = nullptr;
    void **tmp[] = {(void **)&src, (void **)&bst, (void **)&off, (void **)&total, (void **)&tilelen};
    const int64_t tmpbytes[] = {r * pl.dpad * 2, r * pl.ntile * (NB + 1) * 2, r * NB * pl.ntile * 4, r * NB * 4,
                                r * pl.ntile * 4};
    int rc = SAMS_OK;
    for (int q = 0; q < 5 && rc == SAMS_OK; ++q)
        if (hipMalloc(tmp[q], (size_t)tmpbytes[q]) != hipSuccess) { (void)hipGetLastError(); rc = SAMS_ENOMEM; }
    uint32_t *h_total = (uint32_t *)malloc((size_t)(r * NB * 4));
    uint32_t *h_base = (uint32_t *)malloc((size_t)(r * (NB + 1) * 4));
    uint32_t *h_tile = (uint32_t *)malloc((size_t)(r * (pl.ntile + 1) * 4));
    do {
        if (rc != SAMS_OK) break;
        if (!h_total || !h_base || !h_tile) { rc = SAMS_ENOMEM; break; }
        hipError_t e = hipFuncSetAttribute((const void *)k_plan_sort, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_plan_chain, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_bin_scatter, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_head_scatter<false>, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_head_scatter<true>, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_head_scatter_w<false>, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_head_scatter_w<true>, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
#define SAMS_CM(RR, IT)                                                                            \
    if (e == hipSuccess)                                                                           \
        e = hipFuncSetAttribute((const void *)k_bin_collect_median<RR, IT>,                        \
                                hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
        SAMS_FUSED_MEDIAN_VARIANTS(SAMS_CM)
#undef SAMS_CM
        if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_bin_lookup, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_bin_collect, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_plan_place, hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);   // + 1 KiB static
        if (e != hipSuccess) { g_last_hip_error = (int)e; rc = SAMS_EHIP; break; }
        rc = dispatch_acc(ctx, nullptr, RowGroup{0, 0, 0, 0, 0}, true);
        if (rc != SAMS_OK) break;
        {
            ProfScope ps(ctx, KID_PLAN_BUILD);
            hipLaunchKernelGGL(k_plan_sort, dim3((unsigned)pl.ntile, (unsigned)r), dim3(kPlanThreads),
                               (size_t)(L * 4), ctx->stream, ctx->hp, ctx->d, pl.tile_log2, pl.win_log2, NB,
                               pl.ntile, pl.dpad, src, bst);
            hipLaunchKernelGGL(k_plan_runlen, dim3((unsigned)NB, (unsigned)r), dim3(256), 0, ctx->stream,
                               bst, pl.run_pad, NB, pl.ntile, off, total);
            hipLaunchKernelGGL(k_plan_tilelen, dim3((unsigned)pl.ntile, (unsigned)r), dim3(256), 0, ctx->stream,
                               bst, pl.run_pad, NB, pl.ntile, tilelen);
        }
        e = hipMemcpyAsync(h_total, total, (size_t)(r * NB * 4), hipMemcpyDeviceToHost, ctx->stream);
        if (e == hipSuccess)
            e = hipMemcpyAsync(h_tile, tilelen, (size_t)(r * pl.ntile * 4), hipMemcpyDeviceToHost, ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        if (e != hipSuccess) { g_last_hip_error = (int)e; rc = SAMS_EHIP; break; }
        // bins are padded to whole chunks of the accumulate kernel that will read them: 4096 positions where the
        // chunk-record kernel may run (its shape: 1024 threads, nominal chunks of 2048), else the chunk itself
        const bool wide_shape = pl.acc_threads == 1024 && CH == 2048;
        const int64_t BP = (wide_shape && pl.acc_wide >= 2) ? (int64_t)kRecChunk : CH;
        int64_t rowlen = 0;
        bool overflow = false;
        for (int64_t j = 0; j < r; ++j) {
            int64_t run = 0;
            for (int64_t b = 0; b < NB; ++b) {
                h_base[j * (NB + 1) + b] = (uint32_t)run;
                run += ((int64_t)h_total[j * NB + b] + BP - 1) / BP * BP;
            }
            h_base[j * (NB + 1) + NB] = (uint32_t)run;
            if (run >= ((int64_t)1 << 32)) overflow = true;
            if (run > rowlen) rowlen = run;
        }
        if (overflow) { rc = SAMS_EINVAL; break; }
        pl.rowlen = rowlen;
        // exclusive prefix of the tile lengths, in place, back to front so that nothing is overwritten early
        for (int64_t j = r - 1; j >= 0; --j) {
            uint32_t run = 0;
            uint32_t *row = (uint32_t *)malloc((size_t)((pl.ntile + 1) * 4));
            if (!row) { rc = SAMS_ENOMEM; break; }
            for (int64_t q = 0; q < pl.ntile; ++q) { row[q] = run; run += h_tile[j * pl.ntile + q]; }
            row[pl.ntile] = run;
            for (int64_t q = 0; q <= pl.ntile; ++q) h_tile[j * (pl.ntile + 1) + q] = row[q];
            free(row);
        }
        if (rc != SAMS_OK) break;
        rc = dev_alloc(ctx, (void **)&pl.srcp, r * rowlen * 2);
        if (rc == SAMS_OK) rc = dev_alloc(ctx, (void **)&pl.dst16, r * (rowlen >> pl.grp_log2) * 4);
        if (rc == SAMS_OK) rc = dev_alloc(ctx, (void **)&pl.meta, r * rowlen * 4);
        if (rc == SAMS_OK) rc = dev_alloc(ctx, (void **)&pl.wlow, r * rowlen * 2);
        if (rc != SAMS_OK) break;
        e = hipMemcpyAsync(pl.binbase, h_base, (size_t)(r * (NB + 1) * 4), hipMemcpyHostToDevice, ctx->stream);
        if (e == hipSuccess)
            e = hipMemcpyAsync(pl.pbase, h_tile, (size_t)(r * (pl.ntile + 1) * 4), hipMemcpyHostToDevice, ctx->stream);
        if (e != hipSuccess) { g_last_hip_error = (int)e; rc = SAMS_EHIP; break; }
        rc = enqueue_fill_u32(ctx, pl.meta, r * rowlen, kMetaNotFirst | kMetaPad);
        if (rc == SAMS_OK) rc = enqueue_fill_u32(ctx, reinterpret_cast<uint32_t *>(pl.wlow), r * rowlen / 2, 0u);   // padding: bucket 0
        if (rc != SAMS_OK) break;
        {
            ProfScope ps(ctx, KID_PLAN_BUILD);
            hipLaunchKernelGGL(k_plan_place, dim3((unsigned)pl.ntile, (unsigned)r), dim3(256),
                               (size_t)((NB + 1) * 4), ctx->stream, ctx->hp, pl.run_pad, pl.grp_log2, pl.tile_log2, pl.win_log2, NB,
                               pl.ntile, pl.dpad, rowlen, src, bst, off, pl.binbase, pl.pbase, pl.srcp, pl.dst16,
                               pl.meta, pl.wlow);
        }
        e = hipStreamSynchronize(ctx->stream);                       // h_base and off are released below
        if (e == hipSuccess) e = hipGetLastError();
        if (e != hipSuccess) { g_last_hip_error = (int)e; rc = SAMS_EHIP; break; }
        // the build-time arrays are no longer needed: release them before anything else is allocated
        for (int q = 0; q < 5; ++q)
            if (*tmp[q]) { (void)hipFree(*tmp[q]); *tmp[q] = nullptr; }
        // which accumulate kernel: the generic one, the one with 16-byte loads, or the one reading chunk records
        pl.acc_variant = (wide_shape && pl.acc_wide >= 1) ? 1 : 0;
        pl.rec_mask = 0;
        if (wide_shape && pl.acc_wide >= 2) {
            uint32_t *over = nullptr, h_over[SAMS_MAX_ROWS] = {0};
            if (hipMalloc((void **)&over, SAMS_MAX_ROWS * 4) != hipSuccess) { (void)hipGetLastError(); rc = SAMS_ENOMEM; break; }
            rc = dev_alloc(ctx, (void **)&pl.rec, r * (rowlen / kRecChunk) * kRecWords * 4);
            if (rc == SAMS_OK) rc = enqueue_fill_u32(ctx, over, SAMS_MAX_ROWS, 0u);
            if (rc == SAMS_OK) {
                ProfScope ps(ctx, KID_PLAN_BUILD);
                hipLaunchKernelGGL(k_plan_records, dim3((unsigned)(rowlen / kRecChunk), (unsigned)r), dim3(kPlanThreads), 0,
                                   ctx->stream, pl.meta, pl.rec, rowlen, over);
                e = hipMemcpyAsync(h_over, over, SAMS_MAX_ROWS * 4, hipMemcpyDeviceToHost, ctx->stream);
                if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
                if (e == hipSuccess) e = hipGetLastError();
                if (e != hipSuccess) { g_last_hip_error = (int)e; rc = SAMS_EHIP; }
            }
            (void)hipFree(over);
            if (rc != SAMS_OK) break;
            // rows every chunk of which fits the record format use the records; the others keep their meta words
            for (int64_t j = 0; j < r; ++j)
                if (!h_over[j]) pl.rec_mask |= 1u << j;
            if (pl.rec_mask == (r >= 32 ? 0xffffffffu : ((1u << r) - 1u))) {
                pl.acc_variant = 2;
                (void)hipFree(pl.meta);
                pl.meta = nullptr;
                ctx->scratch_bytes -= r * rowlen * 4;
            } else if (pl.rec_mask == 0) {
                (void)hipFree(pl.rec);
                pl.rec = nullptr;
                ctx->scratch_bytes -= r * (rowlen / kRecChunk) * kRecWords * 4;
            }
        }
        if (pl.acc_variant != 2) {                                   // the kernels that read meta words need the chains
            ProfScope ps(ctx, KID_PLAN_BUILD);
            hipLaunchKernelGGL(k_plan_chain, dim3((unsigned)(rowlen / CH), (unsigned)r),
                               dim3(CH < kPlanThreads ? (unsigned)CH : kPlanThreads), (size_t)(CH * 4), ctx->stream,
                               pl.chunk_log2, rowlen, pl.meta);
            e = hipStreamSynchronize(ctx->stream);
            if (e == hipSuccess) e = hipGetLastError();
            if (e != hipSuccess) { g_last_hip_error = (int)e; rc = SAMS_EHIP; break; }
        }
        const int64_t stg_bytes = n * pl.stage_rows * rowlen * 4;
        rc = (tun.stage_spread && stg_bytes >= ((int64_t)2 << 30)) ? spread_alloc(ctx, stg_bytes) : SAMS_ENOMEM;
        if (rc != SAMS_OK) rc = dev_alloc(ctx, (void **)&pl.stg, stg_bytes);
        // the median is fused when a thread can hold the row estimates of its coordinates and the staging
        // buffer can hold the looked-up values of all r rows; otherwise they go through rowest
        pl.fused_median = tun.fuse_median && fused_median_iters(ctx->r, pl.tile_log2) > 0 && (ctx->d & 3) == 0 &&
                          n * pl.stage_rows >= r;
        if (rc == SAMS_OK && !pl.fused_median) rc = dev_alloc(ctx, (void **)&pl.rowest, r * ctx->d * 4);
        if (rc != SAMS_OK) break;
    } while (0);
    free(h_total);
    free(h_base);
    free(h_tile);
    for (int q = 0; q < 5; ++q)
        if (*tmp[q]) (void)hipFree(*tmp[q]);
    return rc;
}

void plan_destroy(sams_ctx *ctx)
{
    Plan &pl = ctx->plan;
    spread_free(pl);                                                 // leaves pl.stg null when it was mapped from chunks
    void *ptrs[] = {pl.srcp, pl.dst16, pl.pbase, pl.binbase, pl.meta, pl.rec, pl.wlow, pl.stg, pl.rowest};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    pl.srcp = nullptr;
    pl.dst16 = pl.pbase = pl.binbase = pl.meta = pl.rec = nullptr;
    pl.wlow = nullptr;
    pl.stg = pl.rowest = nullptr;
}

bool head_compacts_g(const sams_ctx *ctx) { return ctx->wordrank != nullptr && ctx->gsel != nullptr; }

bool head_can_fuse(const sams_ctx *ctx)
{
    return ctx->tun.fuse_head && ctx->plan.mode == PLAN_BINNED && (ctx->d & 3) == 0 && ctx->plan.tile_log2 <= 14;
}

int enqueue_head_scatter(sams_ctx *ctx, const float *g, float *m, float *e_u, float *v, float *vhat,
                         float beta1, float beta2, float rho, bool pa, const int32_t *idx_prev, int64_t k_prev)
{
    Plan &pl = ctx->plan;
    const int64_t L = (int64_t)1 << pl.tile_log2;
    const int64_t per = (pl.ntile + kNumXcd - 1) / kNumXcd;
    const bool compact = head_compacts_g(ctx) && !pa && k_prev > 0;
    HeadArgs ha = {g, m, e_u, v, vhat, ctx->bitmap, beta1, 1.0f - beta1, beta2, 1.0f - beta2, rho,
                   compact ? ctx->wordrank : nullptr, compact ? ctx->gsel : nullptr, k_prev};
    {
        ProfScope ps(ctx, KID_HEAD_SCATTER);
        const dim3 grid((unsigned)(per * kNumXcd));
        const RowGroup rg = {0, pl.stage_rows, pl.stage_rows, ctx->r, pl.stage_ilv};
        if (ctx->tun.fuse_head == 2) {                                  // one workgroup per (tile, worker)
            const dim3 wgrid((unsigned)(per * kNumXcd * ctx->n));
            if (pa)
                hipLaunchKernelGGL(k_head_scatter_w<true>, wgrid, dim3(kFusedThreads), (size_t)(L * 4), ctx->stream,
                                   ha, pl.srcp, pl.dst16, pl.pbase, pl.stg, ctx->n, rg, ctx->d, pl.tile_log2,
                                   pl.ntile, pl.rowlen, pl.grp_log2);
            else
                hipLaunchKernelGGL(k_head_scatter_w<false>, wgrid, dim3(kFusedThreads), (size_t)(L * 4), ctx->stream,
                                   ha, pl.srcp, pl.dst16, pl.pbase, pl.stg, ctx->n, rg, ctx->d, pl.tile_log2,
                                   pl.ntile, pl.rowlen, pl.grp_log2);
        } else if (pa)
            hipLaunchKernelGGL(k_head_scatter<true>, grid, dim3(kFusedThreads), (size_t)(L * 4), ctx->stream, ha,
                               pl.srcp, pl.dst16, pl.pbase, pl.stg, ctx->n, rg, ctx->d, pl.tile_log2, pl.ntile,
                               pl.rowlen, pl.grp_log2);
        else
            hipLaunchKernelGGL(k_head_scatter<false>, grid, dim3(kFusedThreads), (size_t)(L * 4), ctx->stream, ha,
                               pl.srcp, pl.dst16, pl.pbase, pl.stg, ctx->n, rg, ctx->d, pl.tile_log2, pl.ntile,
                               pl.rowlen, pl.grp_log2);
    }
    if (compact) {
        if (ctx->n >= kWideMinWorkers)
            SAMS_LAUNCH(ctx, KID_HEAD_SPARSE_V, k_head_sparse_v_sel_wide, (unsigned)((k_prev + kWideCoords - 1) / kWideCoords),
                        256, ctx->gsel, idx_prev, k_prev, ctx->n, 1.0f - beta2, v, vhat);
        else
            SAMS_LAUNCH(ctx, KID_HEAD_SPARSE_V, k_head_sparse_v_sel, (unsigned)((k_prev + 255) / 256), 256, ctx->gsel, idx_prev,
                        k_prev, ctx->n, 1.0f - beta2, v, vhat);
    } else if (ctx->tun.fuse_head == 2 && !pa && k_prev > 0) {
        if (ctx->n >= kWideMinWorkers)
            SAMS_LAUNCH(ctx, KID_HEAD_SPARSE_V, k_head_sparse_v_wide, (unsigned)((k_prev + kWideCoords - 1) / kWideCoords),
                        256, g, idx_prev, k_prev, ctx->n, ctx->d, 1.0f - beta2, v, vhat);
        else
            SAMS_LAUNCH(ctx, KID_HEAD_SPARSE_V, k_head_sparse_v, (unsigned)((k_prev + 255) / 256), 256, g, idx_prev,
                        k_prev, ctx->n, ctx->d, 1.0f - beta2, v, vhat);
    }
    SAMS_HIP(hipGetLastError());
    pl.staged_u = e_u;          // the staging now holds the sorted copy of this vector
    return SAMS_OK;
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
    const int64_t L = (int64_t)1 << pl.tile_log2;
    const int64_t per = (pl.ntile + kNumXcd - 1) / kNumXcd;
    for (int32_t j0 = 0; j0 < ctx->r; j0 += pl.stage_rows) {
        const RowGroup rg = {j0, (ctx->r - j0) < pl.stage_rows ? (ctx->r - j0) : pl.stage_rows, pl.stage_rows, ctx->r, pl.stage_ilv};
        if (j0 > 0 || pl.staged_u != u) {                            // not staged by a fused head: pass 1 now
            ProfScope ps(ctx, KID_BIN_SCATTER);
            hipLaunchKernelGGL(k_bin_scatter, dim3((unsigned)(per * kNumXcd * ctx->n)), dim3((unsigned)ctx->tun.scatter_threads),
                               (size_t)(L * 4), ctx->stream, u, pl.srcp, pl.dst16, pl.pbase, pl.stg, ctx->n, rg,
                               ctx->d, pl.tile_log2, pl.ntile, pl.rowlen, pl.grp_log2);
        }
        SAMS_HIP(hipGetLastError());
        SAMS_TRY(dispatch_acc(ctx, S_workers, rg, false));
        SAMS_HIP(hipGetLastError());
    }
    if (pl.stage_rows < ctx->r) pl.staged_u = nullptr;               // the staging now holds the last row group
    return SAMS_OK;
}

}  // namespace sams
