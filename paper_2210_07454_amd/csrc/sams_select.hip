// Stage 3 of the pipeline declared in sams.h: per-coordinate estimates (median over rows, Sec. II-C,
// with the 1/sqrt(vhat) scaling of Alg. 3) and the exact top-k selection of Alg. 2.
#include "sams_ctx.h"

// Every formula below is evaluated as separate IEEE-754 binary32 operations, rounded to nearest:
// no fused multiply-add is formed (here and with -ffp-contract=off on the command line), and
// x / y and sqrtf(x) are the correctly rounded ones (hipcc's default; never build this file with
// -ffast-math or -fno-hip-fp32-correctly-rounded-divide-sqrt).
#pragma clang fp contract(off)

namespace sams {
// ------------------------------------------------------------------------------------------
// stage 3a: per-coordinate estimates (Sec. II-C median, Alg. 3 scaling)
// ------------------------------------------------------------------------------------------
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

// est[l] = median_j(rowest[j][l]) / sqrt(vhat[l]) from row estimates already in coordinate order
template <int R>
__global__ void __launch_bounds__(256)
k_est_median(const float *__restrict__ rowest, const float *__restrict__ vhat, float *__restrict__ est,
             int64_t d)
{
    int64_t l = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (l >= d) return;
    float a[R];
#pragma unroll
    for (int j = 0; j < R; ++j) a[j] = rowest[(int64_t)j * d + l];
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

// The streaming passes of the selection read four consecutive keys per lane with one 16-byte load
// (the entry points accept 16-byte aligned arrays only; the last, partial group of four is read key by key).  Absent keys
// (at or beyond len) are reported through the mask `have`.
struct Keys4 {
    float v[4];
    uint32_t have;   // bit z set: v[z] is a key
};
__device__ __forceinline__ Keys4 load_keys4(const float *__restrict__ keys, int64_t l, int64_t len)
{
    Keys4 q;
    if (l + 3 < len) {
        typedef float vec4f __attribute__((ext_vector_type(4)));
        const vec4f t = __builtin_nontemporal_load(reinterpret_cast<const vec4f *>(keys + l));   // streamed: read once per pass
        q.v[0] = t.x; q.v[1] = t.y; q.v[2] = t.z; q.v[3] = t.w;
        q.have = 0xfu;
    } else {
        q.have = 0u;
#pragma unroll
        for (int z = 0; z < 4; ++z) {
            q.v[z] = (l + z < len) ? keys[l + z] : 0.0f;
            q.have |= (l + z < len) ? (1u << z) : 0u;
        }
    }
    return q;
}

// sum over the lanes below this one, and over the whole wavefront, of a per-lane count in 0..7
__device__ __forceinline__ void wave_prefix3(uint32_t cnt, uint64_t below, uint32_t *excl, uint32_t *total)
{
    uint32_t e = 0, t = 0;
#pragma unroll
    for (int b = 0; b < 3; ++b) {
        const uint64_t m = __ballot((cnt >> b) & 1u);
        e += (uint32_t)__popcll(m & below) << b;
        t += (uint32_t)__popcll(m) << b;
    }
    *excl = e;
    *total = t;
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
    const int64_t stride = (int64_t)gridDim.x * blockDim.x * 4;
    for (int64_t l = (blockIdx.x * (int64_t)blockDim.x + threadIdx.x) * 4; l < d; l += stride) {
        const Keys4 q = load_keys4(est, l, d);
#pragma unroll
        for (int z = 0; z < 4; ++z) {
            const uint32_t key = mag_key(q.v[z]);
            if (((q.have >> z) & 1u) && (key >> (shift + width)) == prefix)
                atomicAdd(&lh[(key >> shift) & dmask], 1u);
        }
    }
    __syncthreads();
    for (int t = threadIdx.x; t < kHistBins; t += blockDim.x)
        if (lh[t]) atomicAdd(&hist[t], lh[t]);
}

// choose the digit in which the k_rem-th largest key lies; clear the histogram for the next pass.
// 1024 threads; thread t looks at the two bins 2t and 2t+1 counted from the top.
__global__ void __launch_bounds__(1024)
k_sel_pick(SelState *st, uint32_t *hist, int pass)
{
    __shared__ uint32_t part[16];
    const int nb = 1 << sel_width(pass);
    const int t = threadIdx.x;
    const int b0 = nb - 1 - 2 * t, b1 = nb - 2 - 2 * t;             // descending bins
    const uint32_t v0 = b0 >= 0 ? hist[b0] : 0u, v1 = b1 >= 0 ? hist[b1] : 0u;
    const uint32_t k_rem = st->k_rem, prefix_in = st->prefix;
    const uint32_t above0 = block_exclusive_scan_1024(v0 + v1, part), above1 = above0 + v0;
    hist[2 * t] = 0;
    hist[2 * t + 1] = 0;
    int b = -1;
    uint32_t above = 0;
    if (b0 >= 0 && above0 < k_rem && k_rem <= above0 + v0) { b = b0; above = above0; }
    if (b1 >= 0 && above1 < k_rem && k_rem <= above1 + v1) { b = b1; above = above1; }
    if (b >= 0) {                                                    // exactly one thread, since k_rem <= total
        const uint32_t prefix = (prefix_in << sel_width(pass)) | (uint32_t)b;
        st->prefix = prefix;
        st->k_rem = k_rem - above;
        if (pass == kSelPasses - 1) {
            st->tau = prefix;
            st->k_eq = k_rem - above;
        }
    }
}

// a lane's four keys against the threshold: adds to its counts of keys above tau and equal to it
__device__ __forceinline__ void count_keys4(const Keys4 &q, uint32_t tau, uint32_t &ngt, uint32_t &neq)
{
#pragma unroll
    for (int z = 0; z < 4; ++z) {
        const uint32_t key = mag_key(q.v[z]);
        const bool have = (q.have >> z) & 1u;
        ngt += (have && key > tau) ? 1u : 0u;
        neq += (have && key == tau) ? 1u : 0u;
    }
}

// sums of the lanes' counts over the wavefront (in every lane)
__device__ __forceinline__ void wave_sum2(uint32_t &a, uint32_t &b)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        a += __shfl_xor(a, off);
        b += __shfl_xor(b, off);
    }
}

// one wavefront over the keys [base, base + span): how many exceed tau, how many equal it (in every lane)
__device__ __forceinline__ void wave_count(const float *__restrict__ est, int64_t d, int64_t base, int span,
                                           uint32_t tau, int lane, uint32_t *gt_out, uint32_t *eq_out)
{
    uint32_t ngt = 0, neq = 0;                                       // this lane's counts
    for (int s = 0; s < span; s += kWave * 4) count_keys4(load_keys4(est, base + s + lane * 4, d), tau, ngt, neq);
    wave_sum2(ngt, neq);
    *gt_out = ngt;
    *eq_out = neq;
}

// per wavefront tile of kSelTile consecutive coordinates: how many keys exceed tau, how many equal it
__global__ void __launch_bounds__(256)
k_sel_count(const float *__restrict__ est, int64_t d, const SelState *__restrict__ st,
            uint32_t *__restrict__ cnt_gt, uint32_t *__restrict__ cnt_eq, int64_t ntile)
{
    const int lane = threadIdx.x & (kWave - 1);
    int64_t tile = blockIdx.x * (int64_t)(blockDim.x / kWave) + (threadIdx.x / kWave);
    if (tile >= ntile) return;
    uint32_t ngt, neq;
    wave_count(est, d, tile * kSelTile, kSelTile, st->tau, lane, &ngt, &neq);
    if (lane == 0) {
        cnt_gt[tile] = ngt;
        cnt_eq[tile] = neq;
    }
}

// single block: exclusive prefixes over the tiles.  eq_base = equal keys before the tile;
// sel_base = selected coordinates before the tile, where a tile contributes all its greater keys
// and as many of its equal keys as are still wanted (k_eq counted from the smallest index).
// Rounds of 1024 x kScanItems consecutive tiles; a thread owns kScanItems consecutive tiles of a round.
constexpr int kScanItems = 8;

__global__ void __launch_bounds__(1024)
k_sel_scan(const uint32_t *__restrict__ cnt_gt, const uint32_t *__restrict__ cnt_eq, int64_t ntile,
           const SelState *__restrict__ st, uint32_t *__restrict__ sel_base,
           uint32_t *__restrict__ eq_base)
{
    __shared__ uint32_t part[16];
    __shared__ uint32_t carry[2];
    const int t = threadIdx.x;
    const uint32_t k_eq = st->k_eq;
    uint32_t eq_run = 0, sel_run = 0;                                // totals of the rounds already done
    for (int64_t q0 = 0; q0 < ntile; q0 += 1024 * kScanItems) {
        const int64_t lo = q0 + (int64_t)t * kScanItems;
        uint32_t ce[kScanItems], cg[kScanItems];
        uint32_t eq_sum = 0;
#pragma unroll
        for (int z = 0; z < kScanItems; ++z) {
            ce[z] = lo + z < ntile ? cnt_eq[lo + z] : 0u;
            cg[z] = lo + z < ntile ? cnt_gt[lo + z] : 0u;
            eq_sum += ce[z];
        }
        const uint32_t eb0 = eq_run + block_exclusive_scan_1024(eq_sum, part);
        uint32_t eb = eb0, take_sum = 0;
#pragma unroll
        for (int z = 0; z < kScanItems; ++z) {
            const uint32_t want = eb < k_eq ? k_eq - eb : 0u;
            take_sum += cg[z] + (ce[z] < want ? ce[z] : want);
            eb += ce[z];
        }
        uint32_t sb = sel_run + block_exclusive_scan_1024(take_sum, part);
        if (t == 1023) {
            carry[0] = eb;
            carry[1] = sb + take_sum;
        }
        eb = eb0;
#pragma unroll
        for (int z = 0; z < kScanItems; ++z) {
            const uint32_t want = eb < k_eq ? k_eq - eb : 0u;
            if (lo + z < ntile) {
                eq_base[lo + z] = eb;
                sel_base[lo + z] = sb;
            }
            sb += cg[z] + (ce[z] < want ? ce[z] : want);
            eb += ce[z];
        }
        __syncthreads();
        eq_run = carry[0];
        sel_run = carry[1];
        __syncthreads();
    }
}

// One sweep of the ordered compaction: the wavefront's lanes hold four consecutive keys each, starting at coordinate
// l0 in this lane; the selected ones (key > tau, or key == tau and among the first k_eq such keys) are written at
// their rank.  out, eqr: selected and equal keys before this sweep, updated for the next one.
__device__ __forceinline__ void compact_keys4(const Keys4 &q, int64_t l0, uint32_t tau, uint32_t k_eq, uint64_t below,
                                              uint32_t &out, uint32_t &eqr, int64_t k, int32_t *__restrict__ idx,
                                              float *__restrict__ est_sel)
{
    uint32_t gt = 0, eq = 0;                                         // bit z: key z is above / at the threshold
#pragma unroll
    for (int z = 0; z < 4; ++z) {
        const uint32_t key = mag_key(q.v[z]);
        const bool have = (q.have >> z) & 1u;
        gt |= (have && key > tau) ? (1u << z) : 0u;
        eq |= (have && key == tau) ? (1u << z) : 0u;
    }
    // Most sweeps hold no key at the threshold and at most one selected key per lane: both prefixes then come from
    // one ballot instead of three (the branches are uniform over the wavefront).
    uint32_t take = gt;
    if (__ballot(eq != 0u) != 0) {
        uint32_t eq_before, eq_total;
        wave_prefix3((uint32_t)__popc(eq), below, &eq_before, &eq_total);
#pragma unroll
        for (int z = 0; z < 4; ++z) {
            const uint32_t rank = eqr + eq_before + (uint32_t)__popc(eq & ((1u << z) - 1u));
            if (((eq >> z) & 1u) && rank < k_eq) take |= 1u << z;
        }
        eqr += eq_total;
    }
    const uint64_t any = __ballot(take != 0u);
    if (any == 0) return;
    uint32_t take_before, take_total;
    if (__ballot((take & (take - 1u)) != 0u) == 0) {                 // no lane selects two of its keys
        take_before = (uint32_t)__popcll(any & below);
        take_total = (uint32_t)__popcll(any);
    } else {
        wave_prefix3((uint32_t)__popc(take), below, &take_before, &take_total);
    }
#pragma unroll
    for (int z = 0; z < 4; ++z) {
        if ((take >> z) & 1u) {
            const int64_t pos = (int64_t)out + take_before + __popc(take & ((1u << z) - 1u));
            if (pos < k) {
                idx[pos] = (int32_t)(l0 + z);
                if (est_sel) est_sel[pos] = q.v[z];
            }
        }
    }
    out += take_total;
}

// one wavefront walks the keys [base, base + span) in index order and writes the selected ones at their rank;
// out, eqr: selected and equal keys before base
__device__ __forceinline__ void wave_compact(const float *__restrict__ est, int64_t d, int64_t base, int span,
                                             uint32_t tau, uint32_t k_eq, int lane, uint32_t out, uint32_t eqr,
                                             int64_t k, int32_t *__restrict__ idx, float *__restrict__ est_sel)
{
    const uint64_t below = ((uint64_t)1 << lane) - 1;
    for (int s = 0; s < span; s += kWave * 4) {
        const int64_t l0 = base + s + lane * 4;                      // this lane's four consecutive keys
        compact_keys4(load_keys4(est, l0, d), l0, tau, k_eq, below, out, eqr, k, idx, est_sel);
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
    wave_compact(est, d, tile * kSelTile, kSelTile, st->tau, st->k_eq, lane, sel_base[tile], eq_base[tile], k, idx,
                 est_sel);
}

// The whole selection in one workgroup of 1024 threads for len <= kSelSmallMax keys: the histogram of the first
// digit with its pick, one sweep that lists the keys sharing that digit in LDS (the later digits, and the counts at
// the threshold per segment of kSelSmallSeg keys, then come from the list), prefixes, and the ordered compaction (one
// wavefront per segment).  Same arithmetic as the kernels above; replaces ten launches, which is most of the step's
// time when the vector has only tens of thousands of coordinates.  Its time is the instruction issue of one compute
// unit, about 5 us per sweep over 65,536 keys plus 10 us for the compaction: three sweeps instead of five brought it
// from 40 to 32 us; four counters per histogram bin, the keys kept in registers across the phases, or the loads of
// eight sweeps issued together each changed nothing.
constexpr int kSmallCand = 8192;             // keys sharing the threshold's first digit that the one-workgroup selection can list in LDS
__global__ void __launch_bounds__(1024)
k_sel_small(const float *__restrict__ keys, int64_t len, uint32_t k, int32_t *__restrict__ idx,
            float *__restrict__ val_sel)
{
    __shared__ uint32_t lh[kHistBins];
    __shared__ uint32_t cand[kSmallCand];                            // (segment << 20) | low 20 bits of a listed key
    __shared__ uint32_t ncand;
    __shared__ uint32_t part[16];
    __shared__ uint32_t sh[2];                                       // prefix, k_rem after a pick
    __shared__ uint32_t seg_gt[16], seg_eq[16], seg_sel_base[16], seg_eq_base[16];
    const int t = threadIdx.x;
    const int lane = t & (kWave - 1), seg = t / kWave;               // 16 wavefronts, one segment of the keys each
    const int64_t base = (int64_t)seg * kSelSmallSeg;
    uint32_t prefix = 0, k_rem = k;
    // lh holds the histogram of the next `width` bits over the keys whose higher bits equal prefix: find the bin of
    // the k_rem-th largest, extend the prefix by it
    auto pick = [&](int width) {
        const int nb = 1 << width;
        const int b0 = nb - 1 - 2 * t, b1 = nb - 2 - 2 * t;          // descending bins, two per thread
        const uint32_t v0 = b0 >= 0 ? lh[b0] : 0u, v1 = b1 >= 0 ? lh[b1] : 0u;
        const uint32_t above0 = block_exclusive_scan_1024(v0 + v1, part), above1 = above0 + v0;
        int b = -1;
        uint32_t above = 0;
        if (b0 >= 0 && above0 < k_rem && k_rem <= above0 + v0) { b = b0; above = above0; }
        if (b1 >= 0 && above1 < k_rem && k_rem <= above1 + v1) { b = b1; above = above1; }
        if (b >= 0) {                                                // exactly one thread, since k_rem <= total
            sh[0] = (prefix << width) | (uint32_t)b;
            sh[1] = k_rem - above;
        }
        __syncthreads();
        prefix = sh[0];
        k_rem = sh[1];
        __syncthreads();
    };
    auto clear_hist = [&]() {
        for (int b = t; b < kHistBins; b += 1024) lh[b] = 0;
        __syncthreads();
    };
    auto hist_over_keys = [&](int pass) {
        const int shift = sel_shift(pass), width = sel_width(pass);
        const uint32_t dmask = (1u << width) - 1u;
        clear_hist();
        for (int64_t l = (int64_t)t * 4; l < len; l += 4096) {
            const Keys4 q = load_keys4(keys, l, len);
#pragma unroll
            for (int z = 0; z < 4; ++z) {
                const uint32_t key = mag_key(q.v[z]);
                if (((q.have >> z) & 1u) && (key >> (shift + width)) == prefix)
                    atomicAdd(&lh[(key >> shift) & dmask], 1u);
            }
        }
        __syncthreads();
    };
    hist_over_keys(0);
    if (t == 0) ncand = 0;
    pick(sel_width(0));                                              // its barriers also publish ncand = 0
    // One sweep lists the keys that share the threshold's first digit (few, unless many keys are equal) and counts, per
    // segment, the keys above that digit; the last two digits and the counts at the threshold then come from the
    // list instead of from three more sweeps over all keys.
    {
        uint32_t ngt = 0;
        for (int s = 0; s < kSelSmallSeg; s += kWave * 4) {
            const Keys4 q = load_keys4(keys, base + s + lane * 4, len);
#pragma unroll
            for (int z = 0; z < 4; ++z) {
                const uint32_t key = mag_key(q.v[z]);
                if ((q.have >> z) & 1u) {
                    const uint32_t top = key >> sel_shift(0);
                    ngt += top > prefix ? 1u : 0u;
                    if (top == prefix) {
                        const uint32_t slot = atomicAdd(&ncand, 1u);
                        if (slot < (uint32_t)kSmallCand) cand[slot] = ((uint32_t)seg << 20) | (key & 0xFFFFFu);
                    }
                }
            }
        }
        uint32_t zero = 0;
        wave_sum2(ngt, zero);
        if (lane == 0) {
            seg_gt[seg] = ngt;
            seg_eq[seg] = 0;
        }
    }
    __syncthreads();
    const uint32_t listed = ncand;
    if (listed <= (uint32_t)kSmallCand) {
        clear_hist();
        for (uint32_t q = t; q < listed; q += 1024) atomicAdd(&lh[(cand[q] >> 10) & 1023u], 1u);
        __syncthreads();
        pick(sel_width(1));
        const uint32_t digit1 = prefix & 1023u;
        clear_hist();
        for (uint32_t q = t; q < listed; q += 1024) {
            const uint32_t e = cand[q];
            if (((e >> 10) & 1023u) == digit1) atomicAdd(&lh[e & 1023u], 1u);
        }
        __syncthreads();
        pick(sel_width(2));
        const uint32_t tau20 = prefix & 0xFFFFFu;
        for (uint32_t q = t; q < listed; q += 1024) {
            const uint32_t e = cand[q], low = e & 0xFFFFFu;
            if (low > tau20) atomicAdd(&seg_gt[e >> 20], 1u);
            if (low == tau20) atomicAdd(&seg_eq[e >> 20], 1u);
        }
    } else {                                                         // too many to list: sweeps over all keys
        hist_over_keys(1);
        pick(sel_width(1));
        hist_over_keys(2);
        pick(sel_width(2));
        uint32_t ngt = 0, neq = 0;
        if (base < len) wave_count(keys, len, base, kSelSmallSeg, prefix, lane, &ngt, &neq);
        if (lane == 0) {
            seg_gt[seg] = ngt;
            seg_eq[seg] = neq;
        }
    }
    const uint32_t tau = prefix, k_eq = k_rem;
    __syncthreads();
    if (t == 0) {
        uint32_t eb = 0, sb = 0;
        for (int q = 0; q < 16; ++q) {
            seg_eq_base[q] = eb;
            seg_sel_base[q] = sb;
            const uint32_t want = eb < k_eq ? k_eq - eb : 0u;
            sb += seg_gt[q] + (seg_eq[q] < want ? seg_eq[q] : want);
            eb += seg_eq[q];
        }
    }
    __syncthreads();
    if (base < len)
        wave_compact(keys, len, base, kSelSmallSeg, tau, k_eq, lane, seg_sel_base[seg], seg_eq_base[seg], (int64_t)k, idx,
                     val_sel);
}

// hist != null: the caller is about to select over est and has reset the selection state (enqueue_select_begin);
// *hist_done tells whether the estimate kernel also took the histogram of the first radix digit
constexpr int64_t kGatherEstimateMaxTableBytes = 1 << 20, kGatherEstimateMaxD = (int64_t)1 << 22;
int enqueue_estimate(sams_ctx *ctx, const float *S_mean, const float *vhat, float *est, uint32_t *hist, bool *hist_done)
{
    if (hist_done) *hist_done = false;
    const int block = 256;
    const int grid = grid_for(ctx->d, block);
    // A small table under a short vector stays in every L2: r gathers per coordinate in one launch then beat the two
    // launches of the plan-driven recovery (C1: 6 us against 23), which is made for tables far larger than any cache.
    const bool small = (int64_t)ctx->r * ctx->c * 4 <= kGatherEstimateMaxTableBytes && ctx->d <= kGatherEstimateMaxD;
    if (ctx->plan.mode == PLAN_BINNED && (ctx->tun.estimate_path == 2 || (ctx->tun.estimate_path == 0 && !small))) {
        bool done = false;
        SAMS_TRY(enqueue_estimates_planned_fused(ctx, S_mean, vhat, est, &done, hist));
        if (done) {
            if (hist_done) *hist_done = hist != nullptr;
            return SAMS_OK;
        }
        SAMS_TRY(enqueue_row_estimates_planned(ctx, S_mean, ctx->plan.rowest));
        switch (ctx->r) {
#define SAMS_CASE(R)                                                                                  \
    case R:                                                                                           \
        SAMS_LAUNCH(ctx, KID_EST_MEDIAN, (k_est_median<R>), grid, block, ctx->plan.rowest, vhat, est, \
                    ctx->d);                                                                          \
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
    switch (ctx->r) {
#define SAMS_CASE(R)                                                                             \
    case R:                                                                                      \
        SAMS_LAUNCH(ctx, KID_ESTIMATE, (k_estimate<R>), grid, block, S_mean, vhat, est, ctx->hp, \
                    ctx->d, ctx->c);                                                             \
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

// idx_out[q] = idx_in[pos[q]]: positions among the candidates back to coordinates
__global__ void __launch_bounds__(256)
k_refine_map(const int32_t *__restrict__ idx_in, const int32_t *__restrict__ pos, int64_t k_out,
             int32_t *__restrict__ idx_out)
{
    int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (q < k_out) idx_out[q] = idx_in[pos[q]];
}

SelScratch ctx_sel_scratch(const sams_ctx *ctx)
{
    return SelScratch{ctx->hist, ctx->sel, ctx->cnt, ctx->base, ctx->ntile};
}

// resets the selection state and the histogram for a selection of k out of len keys; nothing to do for the
// one-workgroup selection of short vectors (returns false)
bool select_uses_passes(int64_t len) { return len > kSelSmallMax; }

int enqueue_select_begin(sams_ctx *ctx, hipStream_t stream, const SelScratch &sc, int64_t k)
{
    SAMS_LAUNCH_ON(ctx, stream, KID_SEL_INIT, k_sel_init, 1, 256, sc.sel, (uint32_t)k, sc.hist);
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

// the k entries of keys[0..len) with the largest magnitude, ties to the smaller position; positions ascending.
// begun: enqueue_select_begin has been called for this selection (otherwise it is called here);
// hist0_done: the histogram of the first digit has been accumulated into sc.hist since then
int enqueue_select(sams_ctx *ctx, hipStream_t stream, const SelScratch &sc, const float *keys, int64_t len, int64_t k,
                   int32_t *idx, float *val_sel, bool begun, bool hist0_done)
{
    if (len <= kSelSmallMax) {
        SAMS_LAUNCH_ON(ctx, stream, KID_SEL_SMALL, k_sel_small, 1, 1024, keys, len, (uint32_t)k, idx, val_sel);
        SAMS_HIP(hipGetLastError());
        return SAMS_OK;
    }
    const int64_t nt = (len + kSelTile - 1) / kSelTile;
    if (nt > sc.ntile_cap) return SAMS_EINVAL;
    uint32_t *cnt_gt = sc.cnt, *cnt_eq = sc.cnt + sc.ntile_cap;
    uint32_t *sel_base = sc.base, *eq_base = sc.base + sc.ntile_cap;
    if (!begun) SAMS_TRY(enqueue_select_begin(ctx, stream, sc, k));
    for (int pass = 0; pass < kSelPasses; ++pass) {
        if (pass > 0 || !(begun && hist0_done))
            SAMS_LAUNCH_ON(ctx, stream, KID_SEL_HIST, k_sel_hist, grid_for(len, 256 * 16, 4096), 256, keys, len, pass,
                           sc.sel, sc.hist);
        SAMS_LAUNCH_ON(ctx, stream, KID_SEL_PICK, k_sel_pick, 1, 1024, sc.sel, sc.hist, pass);
    }
    const int waves_per_block = 256 / kWave;
    const int tgrid = (int)((nt + waves_per_block - 1) / waves_per_block);
    SAMS_LAUNCH_ON(ctx, stream, KID_SEL_COUNT, k_sel_count, tgrid, 256, keys, len, sc.sel, cnt_gt, cnt_eq, nt);
    SAMS_LAUNCH_ON(ctx, stream, KID_SEL_SCAN, k_sel_scan, 1, 1024, cnt_gt, cnt_eq, nt, sc.sel, sel_base, eq_base);
    SAMS_LAUNCH_ON(ctx, stream, KID_SEL_WRITE, k_sel_write, tgrid, 256, keys, len, sc.sel, sel_base, eq_base, nt, k,
                   idx, val_sel);
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

// Second round with over-selection (Sec. III-A): the k_out candidates with the largest |delta_in|.  pos: k_out
// int32 of scratch (positions among the candidates).
int enqueue_refine(sams_ctx *ctx, hipStream_t stream, const SelScratch &sc, int32_t *pos, const int32_t *idx_in,
                   const float *delta_in, int64_t k_in, int64_t k_out, int32_t *idx_out, float *delta_out)
{
    SAMS_TRY(enqueue_select(ctx, stream, sc, delta_in, k_in, k_out, pos, delta_out, false, false));
    SAMS_LAUNCH_ON(ctx, stream, KID_REFINE_MAP, k_refine_map, grid_for(k_out, 256), 256, idx_in, pos, k_out, idx_out);
    SAMS_HIP(hipGetLastError());
    return SAMS_OK;
}

}  // namespace sams
