/*
 * sams.h -- C ABI of the MI355X (gfx950) hot path of SketchedAMSGrad with gradient
 * averaging (Algorithm 2 of arXiv 2210.07454): per optimisation step, the n workers'
 * error-compensated momentum vectors are Count-Sketched, the sketches averaged, every
 * coordinate recovered (median over rows, scaled by 1/sqrt(vhat)), the k largest
 * selected, their exact values gathered, and the AMSGrad state updated.  The n workers
 * are batched buffers on one GPU.
 *
 * Conventions for every entry point
 *   - All tensor arguments are DEVICE pointers into caller-owned memory (fp32 unless said
 *     otherwise), 16-byte aligned, row-major with the shapes given, non-overlapping unless
 *     "in place" is stated.  Only `hash_host` of sams_create is a HOST pointer.
 *   - Work is enqueued on the hipStream_t given to sams_create and is asynchronous with
 *     respect to the host; no entry point synchronises the host with the device.  Calls on one
 *     context must be issued from one host thread at a time; a context's scratch is shared
 *     by its calls, which the stream orders.
 *   - The library never frees or retains caller memory beyond the call, except that
 *     amsgrad_ef_update records the selected index set in the context (a bitmap) for
 *     the next call's second-moment update.
 *   - Return value: SAMS_OK, or a negative code.  SAMS_EINVAL: a null or misaligned pointer,
 *     or a size outside the documented range -- nothing was enqueued.  SAMS_ENOMEM: the
 *     context's scratch could not be allocated.  SAMS_EHIP: the HIP runtime reported an error
 *     (sams_last_hip_error() returns its hipError_t value).
 *   - Non-finite inputs are not detected; NaNs make the ordering of the selection undefined.
 *   - Coordinates are 0-based; d < 2^31 - 1 (the hash modulus).
 */
#ifndef SAMS_H
#define SAMS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SAMS_OK 0
#define SAMS_EINVAL (-1)
#define SAMS_ENOMEM (-2)
#define SAMS_EHIP (-3)

#define SAMS_MAX_ROWS 16
#define SAMS_STATIC_MAX_CANDIDATES 8388608   /* largest k_in topk_refine_static accepts (2^23) */

typedef struct sams_ctx sams_ctx;

/*
 * Create a context for d coordinates, n workers, an r x c Count Sketch and k selected
 * coordinates per step.
 *   hash_host  HOST pointer to r*4 uint32: per row (a_h, b_h, a_s, b_s).  The bucket hash of row j is
 *              h_j(l) = ((a_h*l + b_h) mod (2^31-1)) mod c and the sign hash is s_j(l) = +1 if
 *              ((a_s*l + b_s) mod (2^31-1)) is even, -1 if odd (the paper, Sec. II-C, only asks for
 *              bucket and sign hashes without fixing a family; this 2-universal one is this library's choice).
 *              Requires 1 <= a < 2^31-1, 0 <= b < 2^31-1.  The values are copied.
 *   hip_stream the hipStream_t (as void*) every later call on this context is enqueued on; NULL =
 *              the default stream.
 * Ranges: 1 <= d < 2^31-1, 1 <= n <= 1024, 1 <= r <= SAMS_MAX_ROWS, 1 <= c < 2^31-1, 1 <= k <= d.
 * Allocates the context's device scratch: about 4d bytes for the estimates, d/8 for the index bitmap,
 * small selection state and, when c exceeds one LDS window, the sketch plan and its staging buffer
 * (4*r*d bytes of plan + 4*n*r*d bytes of staging); sams_scratch_bytes reports the total.  The plan is
 * built on the stream by this call.
 * For an even r the median of Sec. II-C is the lower middle element.
 */
int sams_create(sams_ctx **out, int64_t d, int32_t n, int32_t r, int64_t c, int64_t k,
                const uint32_t *hash_host, void *hip_stream);

/*
 * Process-wide tuning knobs (never change results beyond the order of fp32 additions inside a bucket).
 * sams_create copies the current set into the new context, and every later call on that context reads only that
 * copy: changing a knob never affects a context that already exists.  sams_configure and the copy are serialised
 * against each other, so they may be called from different threads.  Keys:
 *   "tile_log2"   0 or 6..14 (default 0): log2 of the coordinates per tile of the binned sketch path.  0 = chosen
 *                 from r, d, n: 2^14 (2^13 for r > 6, 2^12 for r > 12), or less (down to 2^8) while the first pass
 *                 would have too few workgroups to fill the chip (it has one per tile with "fuse_head" 1, one per
 *                 (tile, worker) otherwise)
 *   "win_log2"    0 or 4..15 (default 0): log2 of the buckets per LDS window (the bins of the binned path; a
 *                 table with c <= 2^win_log2 is a single bin, see "sketch_path").  0 = chosen from n, r, c:
 *                 2^15, or less (down to 2^12) when that is needed to give the chip enough windows to work on
 *   "chunk_log2"  0 or 6..11 (default 0 = 11 for 2^15 windows, else 10): log2 of the stream positions the binned accumulation handles
 *                 between two barriers
 *   "acc_threads" 0, 256, 512 or 1024 (default 0 = 1024 for 2^15 windows, else 512): workgroup size of the binned accumulation; must not
 *                 exceed 2^chunk_log2, and a window plus two chunks of 8 bytes must fit in 160 KiB of LDS
 *                 (otherwise sams_create returns SAMS_EINVAL)
 *   "run_pad"     4, 8, 16 (default) or 32: stream positions a (tile, window) run is padded to, so that a run
 *                 is written to the staging buffer as whole 16-, 32-, 64- or 128-byte pieces (less padding means
 *                 fewer staged bytes, but runs that share a memory line with their neighbours)
 *   "scatter_threads" 256, 512 or 1024 (default 1024): workgroup size of the binned scatter pass
 *   "fuse_head"   0 (default), 1 or 2: with 1 or 2, amsgrad_ef_update or amsgrad_ef_update_pa (when it runs the head and the context uses
 *                 the binned path) also writes the sorted copy of e_u that sketch_accumulate needs, and a
 *                 following sketch_accumulate called with that same e_u pointer skips its first pass.
 *                 The caller must then not write to e_u between the two calls (the algorithm never does).
 *                 The sorted copy lives in the context's staging buffer and is forgotten as soon as anything else
 *                 uses that buffer (unsketch_topk, unsketch_estimates, a sketch_accumulate that stages row groups)
 *                 or e_u changes through this library (any amsgrad_ef_update*): a later sketch_accumulate of the
 *                 same pointer then runs both passes again.
 *                 1: one workgroup per tile loops over the workers; 2: one workgroup per (tile, worker), the
 *                 workers of a tile sharing the plan's metadata through one L2, and the (1 - beta2) h^2 term of
 *                 v on I_{t-1} added by a small kernel of its own (same results bit for bit).
 *   "stage_rows"  0..16 (default 0 = all r rows): rows of the sketch staged at once on the binned path; the
 *                 staging buffer holds 4*n*stage_rows*(1.1 to 1.5)*d bytes and stage 1 runs row group after
 *                 row group (each group after the first re-reads u)
 *   "stage_interleave" 0 (default) or 1: layout of the staging buffer.  0: one contiguous copy per (worker, row), so that
 *                 a workgroup of the second pass streams one contiguous region; 1: the n workers' copies of the same
 *                 32 stream positions lie next to each other (one 128-byte line each), so that the workgroups of the
 *                 workers, which run side by side, write and read one region per (row, window) instead of n distant
 *                 ones.  Same results either way (at d = 124M the contiguous layout is 2 % faster as a whole step).
 *   "stage_spread" 0 (default) or 1: with 1, sams_create maps a staging buffer of 2 GiB or more from 1 GiB physical chunks
 *                 picked at even distances over all free device memory, instead of taking one allocation.  Device
 *                 memory is striped over the HBM stacks in coarse pieces, so a buffer that is contiguous in physical
 *                 memory reaches only part of them; scattered over all of it, it reaches all (the first sketch pass is
 *                 20 % faster than with the contiguous buffer a fresh process gets, and no slower than after
 *                 sams_precondition_device_memory).  To pick the chunks sams_create holds nearly all free device
 *                 memory for a moment -- other allocations made on the device meanwhile can fail -- and falls back to
 *                 the ordinary allocation when it cannot.  Same results.
 *   "acc_wide"    2 (default), 1 or 0: with 1024 threads and 2048-position chunks the binned accumulation reads its
 *                 streams with 16-byte loads instead of 4-byte loads (1, 2), and with 2 the per-position metadata
 *                 (4 bytes) is replaced by per-chunk records (2-byte codes plus a list of the groups of positions
 *                 that share a bucket inside a chunk of 4096: 2.5 bytes per position) and a thread keeps the values
 *                 of its four positions in registers.  Decided per row: a row whose hash gives some chunk more than
 *                 512 such groups, 1024 such positions or a group of more than 127 keeps the meta words.  Same results.
 *   "fuse_median" 1 (default) or 0: with 1 the plan-driven recovery keeps the row estimates in registers
 *                 (needs r <= 6 with tiles of 2^14, r <= 12 with 2^13, any r with 2^12 or less); with 0
 *                 they go through a [r][d] scratch array
 *   "estimate_path" 0 (default): stage 3 reads the mean table through the same plan, run backwards, unless the
 *                 table is at most 1 MiB and d <= 2^22 (then as with 1: such a table stays in cache);
 *                 1: one gather per (row, coordinate) straight from the table; 2: through the plan whenever there is one
 *   "sketch_path" 0 (default): the binned, order-preserving path whenever c exceeds one LDS window, and
 *                 also for smaller tables while d <= 2^22 (one bin; one workgroup per (worker, row) walks the
 *                 vector); LDS atomics for small tables with larger d; 1: one global atomic add per term
 *                 (no plan memory); 2: the order-preserving path always; 3: LDS atomics whenever c fits one
 *                 window
 * Returns SAMS_EINVAL for an unknown key or a value out of range.
 */
int sams_configure(const char *key, int value);

/* Waits for the context's stream, frees its scratch and the context.  NULL is a no-op. */
int sams_destroy(sams_ctx *ctx);

/* How this context carries out sketch_accumulate: 0 = one global atomic add per term, 1 = row by row in LDS
 * (c fits one window), 2 = the binned, order-preserving path.  -1 for a NULL context. */
int sams_sketch_mode(const sams_ctx *ctx);

/* How the second pass of the binned path reads its metadata in this context (see "acc_wide"): 2 = every row through
 * compact chunk records; 1 or 0 = some or all rows through per-position meta words, with 16-byte (1) or 4-byte (0)
 * loads.  -1 when the context does not use the binned path (or is NULL).
 * sams_record_rows: bit j set = row j goes through chunk records (decided per row when the plan is built: a row whose
 * hash puts too many positions of one 4096-position chunk into shared buckets keeps its meta words); -1 as above. */
int sams_accumulate_variant(const sams_ctx *ctx);
int64_t sams_record_rows(const sams_ctx *ctx);

/* Device bytes the context allocated. */
int64_t sams_scratch_bytes(const sams_ctx *ctx);

/*
 * Optional, once per process before sams_create and before the caller allocates its buffers: allocates the
 * free memory of the current device in 1 GiB blocks (up to `fraction` of it, 0 < fraction <= 1; stops early
 * when an allocation fails) and frees every block again.  Computes nothing and keeps nothing.  On MI355X
 * the memory manager places later allocations -- of this and of later processes -- differently afterwards, and
 * with that placement the kernels of a step run 3 to 14 % faster (measured: memory that is contiguous in physical
 * address reaches only part of the HBM stacks, memory scattered over all of it reaches all of them).  It
 * has to come first: a process that makes the pass after it has allocated its own buffers, or after sams_create,
 * stays as slow as one that never makes it.  ("stage_spread" gives the context's staging buffer, the one buffer the
 * effect hinges on, the scattered placement whatever came before.)  Synchronises the device.  Returns the number of GiB it held at the peak, or
 * a negative code (SAMS_EINVAL for a fraction out of range, SAMS_EHIP).
 */
int64_t sams_precondition_device_memory(double fraction);

/* hipError_t of the most recent failure reported as SAMS_EHIP by this process (0 if none). */
int sams_last_hip_error(void);

/*
 * Optional per-kernel timing, for benchmarks.  While enabled, every kernel the context launches is
 * bracketed by a HIP event pair recorded on the context's stream (at most 8192 launches per window;
 * later ones are not timed).  This measures the kernels named by sams_profile_name on the device
 * time line; it is not part of the method and changes no result.
 *   sams_profile_kernels   number of distinct kernels the library can launch
 *   sams_profile_name      name of kernel `kernel` (0 <= kernel < sams_profile_kernels()), static string
 *   sams_profile_enable    on != 0: clear the totals and start a window; on == 0: stop recording
 *   sams_profile_only      restricts the timing to one kernel (kernel = its index; -1 = every kernel, the default),
 *                          so that a timed region carries two event records per step instead of two per launch;
 *                          takes effect from the next launch
 *   sams_profile_read      waits for the stream, then writes, per kernel, the summed duration in
 *                          milliseconds and the number of timed launches since the window started
 *                          (total_ms, launches: HOST arrays of sams_profile_kernels() elements)
 */
int sams_profile_kernels(void);
const char *sams_profile_name(int kernel);
int sams_profile_enable(sams_ctx *ctx, int on);
int sams_profile_only(sams_ctx *ctx, int kernel);
int sams_profile_read(sams_ctx *ctx, double *total_ms, int64_t *launches);

/*
 * Writes h_j(l) and s_j(l) for every row and coordinate (the hash functions of Sec. II-C as defined
 * under sams_create), so that they can be compared one by one with another implementation.
 *   bucket  [r][d] int32, device, out     sign  [r][d] int8 (+1 / -1), device, out
 */
int sams_hash_dump(sams_ctx *ctx, int32_t *bucket, int8_t *sign);

/*
 * Stage 1 -- Count Sketch of every worker's vector (Sec. II-C update rule; the worker line of Alg. 2 that
 * sketches the momentum plus the step-size-weighted residual):
 *     S_workers[i][j][h_j(l)] += s_j(l) * u[i][l]      for all workers i, rows j, coordinates l.
 *   u          [n][d] in    the vectors to sketch (what amsgrad_ef_update leaves in e_u)
 *   S_workers  [n][r][c] out, overwritten (zeroed by the call, then accumulated)
 * On the binned path (sams_sketch_mode() == 2: the default unless c fits one LDS window and d > 2^22)
 * the terms of a bucket are added in ascending coordinate order, i.e. the result equals a sequential
 * loop over l bit for bit and is reproducible.
 * On the other paths (LDS atomics, or "sketch_path" = 1) the order is
 * not specified and fp32 rounding may differ from the sequential sum in the last bits; on inputs whose
 * partial sums are exact the result is exact on every path.
 */
int sketch_accumulate(sams_ctx *ctx, const float *u, float *S_workers);

/*
 * Stage 2 -- aggregation on the master (the aggregation line of Alg. 2: the mean of the workers' sketches; linearity, Eq. 3):
 *     S_mean[j][b] = (S_workers[0][j][b] + S_workers[1][j][b] + ... ) / n, workers added in ascending i.
 *   S_workers [n][r][c] in     S_mean [r][c] out
 */
int sketch_reduce(sams_ctx *ctx, const float *S_workers, float *S_mean);

/*
 * Stage 3 -- heavy-coordinate recovery and selection (Sec. II-C unsketch; Alg. 3; Alg. 2 master line
 * that unsketches with vhat_t and keeps the top k):
 *     est[l] = median_j( s_j(l) * S_mean[j][h_j(l)] ) / sqrt(vhat[l])        for every l < d
 *     idx    = the k coordinates with the largest |est|, ties going to the smaller coordinate,
 *              written in ascending order.
 * Alg. 3 is read as this per-coordinate scaling (its result must equal sketching vhat^{-1/2}(m + e) and
 * unsketching normally, as the text under Alg. 2 says).
 *   S_mean  [r][c] in        vhat  [d] in, strictly positive; NULL = plain operator U_0 (no scaling, Alg. 1)
 *   idx     [k] int32 out    est_sel [k] out or NULL: est at the selected coordinates
 */
int unsketch_topk(sams_ctx *ctx, const float *S_mean, const float *vhat, int32_t *idx, float *est_sel);

/* The recovery half of stage 3 alone: est [d] out (all coordinates).  For inspection and tests. */
int unsketch_estimates(sams_ctx *ctx, const float *S_mean, const float *vhat, float *est);

/*
 * Stage 4 -- second round (Sec. III-A; definition of Delta_t^(i) and Delta_t under Alg. 2): exact values of
 * the selected coordinates from every worker, averaged and scaled,
 *     U_workers[i][q] = u[i][idx[q]] ;   delta[q] = ((sum_i U_workers[i][q]) / n) / sqrt(vhat[idx[q]])
 * (workers added in ascending i; vhat == NULL skips the scaling).
 *   u [n][d] in   vhat [d] in or NULL   idx [k] int32 in (each < d)   U_workers [n][k] out   delta [k] out
 */
int gather_topk(sams_ctx *ctx, const float *u, const float *vhat, const int32_t *idx, float *U_workers,
                float *delta);

/*
 * Second round with over-selection (Sec. III-A): P*k candidates are taken by their estimates, their exact values
 * are fetched, and the k largest of those are kept.  For a context created with k = P*k_out:
 * after unsketch_topk (P*k_out candidates) and gather_topk (their exact averaged values), keep the k_out
 * candidates with the largest |delta_in|, ties going to the smaller coordinate, in ascending coordinate order.
 *   idx_in   [k] int32 in, ascending (unsketch_topk's output)     delta_in  [k] in (gather_topk's output)
 *   k_out    1 <= k_out <= k
 *   idx_out  [k_out] int32 out      delta_out [k_out] out
 * The results feed amsgrad_ef_update with k_sel = k_out.  Uses the context's estimate scratch.
 */
int topk_refine(sams_ctx *ctx, const int32_t *idx_in, const float *delta_in, int64_t k_out, int32_t *idx_out,
                float *delta_out);

/*
 * topk_refine for callers that cannot allocate device memory or create a context: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same selection, same kernels, same results as
 * topk_refine(ctx, ...) with ctx->k = k_in, but context-free: the scratch of the selection (k_out positions, a radix
 * histogram, per-tile counts and prefixes; about 4*SAMS_STATIC_MAX_CANDIDATES + 64 KiB bytes) is a static device
 * array inside the library, which every GPU the library runs on holds until the process ends.  The call allocates
 * and frees nothing and records no memset (every clear is a kernel).
 *   idx_in   [k_in] int32 in, ascending     delta_in [k_in] in      1 <= k_out <= k_in <= SAMS_STATIC_MAX_CANDIDATES
 *   idx_out  [k_out] int32 out              delta_out [k_out] out   (all device pointers of the current device, 16-byte aligned)
 *   hip_stream  the hipStream_t (as void*) of the current device to enqueue on; NULL = the default stream
 * Returns SAMS_EINVAL for a null or misaligned pointer or a size outside the range above (nothing enqueued),
 * SAMS_EHIP for a runtime error.  The first call on a device looks up the array's address (hipGetSymbolAddress;
 * sams_create does the same look-up, so a process that has created a context on the device has it already) and
 * should be made outside stream capture.  All calls on one GPU share the one array, which keeps the previous call's
 * contents: calls that overlap in time on the same GPU (different streams, or graphs replayed concurrently) race; calls
 * ordered by a stream or by events do not.
 * topk_refine_static_max_candidates() returns SAMS_STATIC_MAX_CANDIDATES as the library was built.
 */
int topk_refine_static(const int32_t *idx_in, const float *delta_in, int64_t k_in, int64_t k_out, int32_t *idx_out,
                       float *delta_out, void *hip_stream);
int64_t topk_refine_static_max_candidates(void);

/*
 * Stage 5 -- AMSGrad update with error feedback (Alg. 2).  One call finishes iteration t and starts
 * iteration t+1:
 *   finish t ("tail"; lines for e_t and x_{t+1}; e_t is zero on I_t as the proof of Lemma 3 states),
 *   if k_sel > 0:
 *       e_u[i][idx[q]] = 0 for all i ;   x[idx[q]] -= lr * delta[q] ;   I_t = {idx[q]} is recorded.
 *   start t+1 ("head"; lines for m, h, v, vhat and the vector to sketch), if g_next != NULL:
 *       m[i][l]   = beta1 * m[i][l] + (1-beta1) * g_next[i][l]
 *       e_u[i][l] = m[i][l] + ef_ratio * e_u[i][l]                       (now holds u_{t+1}^(i))
 *       h[l]      = (sum_i g_next[i][l]) / n  if l in I_t, else 0
 *       v[l]      = beta2 * v[l] + (1-beta2) * h[l]^2 ;   vhat[l] = max(vhat[l], v[l])
 *   (v decays on every coordinate, as the algorithm box writes it.)
 * The first call of a run passes k_sel = 0 (I_0 is empty: head only); the last may pass g_next = NULL.
 *   g_next [n][d] in or NULL     m, e_u [n][d] in place     v, vhat, x [d] in place
 *   idx [k_sel] int32 in, strictly ascending, each < d;  delta [k_sel] in;  0 <= k_sel <= k
 *   ef_ratio = alpha_{t}/alpha_{t+1} (1 for a constant step size)
 * Initial state per Alg. 2: m = e_u = 0, v = vhat = eps (a positive constant), x = x_1.
 */
int amsgrad_ef_update(sams_ctx *ctx, const float *g_next, float *m, float *e_u, float *v, float *vhat,
                      float *x, const int32_t *idx, const float *delta, int64_t k_sel, float beta1,
                      float beta2, float lr, float ef_ratio);

/*
 * Stage 5 of the parameter-averaging variant (Alg. 1): same tail as amsgrad_ef_update, and the head
 *       m[i][l]    = beta1 * m[i][l] + (1-beta1) * g_next[i][l]
 *       v_workers[i][l]    = beta2 * v_workers[i][l] + (1-beta2) * g_next[i][l]^2
 *       vhat_workers[i][l] = max(vhat_workers[i][l], v_workers[i][l])
 *       e_u[i][l]  = m[i][l] / sqrt(vhat_workers[i][l]) + ef_ratio * e_u[i][l]
 * with every worker keeping its own second moments.  The other stages are called with vhat = NULL (Alg. 1 uses
 * the plain unsketch operator and the values it averages are already scaled).
 *   v_workers, vhat_workers [n][d] in place (initially eps);  everything else as in amsgrad_ef_update.
 */
int amsgrad_ef_update_pa(sams_ctx *ctx, const float *g_next, float *m, float *e_u, float *v_workers,
                         float *vhat_workers, float *x, const int32_t *idx, const float *delta, int64_t k_sel,
                         float beta1, float beta2, float lr, float ef_ratio);

#ifdef __cplusplus
}
#endif
#endif /* SAMS_H */
