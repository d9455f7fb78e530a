/*
 * CPU oracle for the SketchedAMSGrad (gradient averaging) step -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the body of the oracle, written once for a floating type REAL and
 * included twice by sams_oracle.c (REAL = float, suffix _f32; REAL = double,
 * suffix _f64).  It is deliberately slow and plain: one loop per line of the
 * algorithm, ascending index order, no blocking, no fusion, no threads.  It shares
 * no code, header, table or constant with the HIP library and must never be
 * called from the product path; only tests, the smoke check and the benchmark's
 * cpu_baseline leg may use it.
 *
 * What each function follows (paper = arXiv 2210.07454):
 *   hash family .............. not fixed by the paper (Sec. II-C only names "bucket
 *                              hashes" h_j and "sign hashes" s_j); the reading used is
 *                              y = (a*l + b) mod (2^31-1), bucket = y mod c,
 *                              sign = +1 if the sign-hash y is even, else -1.
 *   sketch ................... Sec. II-C update rule S[j,h_j(l)] += s_j(l) f_l.
 *   sketch_mean .............. Alg. 2, the master's aggregation line: mean of the workers' sketches.
 *   unsketch ................. Sec. II-C (median over rows of s_j(l) S[j,h_j(l)]) and
 *                              Alg. 3 read as a per-coordinate scaling by 1/sqrt(v_l)
 *                              (the text below Alg. 2 says the operator must equal
 *                              sketching v^{-1/2}(m + rho e) and unsketching normally).
 *   topk ..................... Alg. 2, the Top-k of the unsketched vector: k largest magnitudes,
 *                              ties to the smaller index, result ascending by index.
 *   gather ................... Sec. III-A second round + definition of Delta_t^(i)
 *                              (coordinates of vhat^{-1/2}(m + rho e) on I_t), mean over workers.
 *   head ..................... Alg. 2 worker lines for m_t, h_t, the sketched vector
 *                              u = m_t + rho e_{t-1}, and master lines for v_t, vhat_t.
 *   tail ..................... Alg. 2 e_t and x_{t+1} lines, with e_t = 0 on I_t as the
 *                              proof of Lemma 3 states.
 *
 * Readings that nothing in the paper decides ("parity unpinned"):
 *   - v decays by beta2 on every coordinate, also off I_{t-1} (the algorithm box),
 *     whereas the proof of Lemma 3 speaks of such coordinates keeping their value;
 *   - for an even number of rows the median is the lower middle element.
 */

#define ORC_CAT_(a, b) a##b
#define ORC_CAT(a, b) ORC_CAT_(a, b)
#define FN(name) ORC_CAT(name, SUFFIX)

/* Sec. II-C: zero the r x c table, then for every row j and coordinate l (ascending)
 * add s_j(l) * u_l into bucket h_j(l). */
void FN(orc_sketch)(const REAL *u, int64_t d, int32_t r, int64_t c,
                    const uint32_t *hash /* [r][4] = a_h, b_h, a_s, b_s */,
                    REAL *S /* [r][c] */)
{
    for (int64_t t = 0; t < (int64_t)r * c; ++t) S[t] = (REAL)0;
    for (int32_t j = 0; j < r; ++j) {
        const uint32_t *hp = hash + 4 * j;
        for (int64_t l = 0; l < d; ++l) {
            int64_t b = orc_bucket(hp[0], hp[1], (uint32_t)l, c);
            int sg = orc_sign(hp[2], hp[3], (uint32_t)l);
            REAL term = (sg > 0) ? u[l] : -u[l];
            S[(int64_t)j * c + b] = S[(int64_t)j * c + b] + term;
        }
    }
}

/* Alg. 2, master: S_t = (1/n) sum_i S_t^(i); workers added in ascending i, one divide. */
void FN(orc_sketch_mean)(const REAL *S_w /* [n][r][c] */, int32_t n, int32_t r, int64_t c,
                         REAL *S_mean /* [r][c] */)
{
    int64_t rc = (int64_t)r * c;
    for (int64_t t = 0; t < rc; ++t) {
        REAL acc = S_w[t];
        for (int32_t i = 1; i < n; ++i) acc = acc + S_w[(int64_t)i * rc + t];
        S_mean[t] = acc / (REAL)n;
    }
}

/* Sec. II-C + Alg. 3: est_l = median_j( s_j(l) S[j,h_j(l)] ) / sqrt(vhat_l);
 * vhat == NULL gives the plain operator U_0.  Median = element floor((r-1)/2) of the
 * ascending sort of the r row estimates.  The d coordinates l0 .. l0+d-1 are recovered;
 * vhat and est are indexed from l0 (l0 = 0 for the whole vector). */
void FN(orc_unsketch)(const REAL *S /* [r][c] */, const REAL *vhat /* [d] or NULL */,
                      int64_t d, int32_t r, int64_t c, const uint32_t *hash, REAL *est /* [d] */,
                      int64_t l0)
{
    REAL vals[64];
    for (int64_t t = 0; t < d; ++t) {
        const int64_t l = l0 + t;
        for (int32_t j = 0; j < r; ++j) {
            const uint32_t *hp = hash + 4 * j;
            int64_t b = orc_bucket(hp[0], hp[1], (uint32_t)l, c);
            int sg = orc_sign(hp[2], hp[3], (uint32_t)l);
            REAL q = S[(int64_t)j * c + b];
            vals[j] = (sg > 0) ? q : -q;
        }
        for (int32_t a = 1; a < r; ++a) { /* insertion sort, ascending */
            REAL key = vals[a];
            int32_t p = a - 1;
            while (p >= 0 && vals[p] > key) { vals[p + 1] = vals[p]; --p; }
            vals[p + 1] = key;
        }
        REAL med = vals[(r - 1) / 2];
        est[t] = vhat ? med / FN(orc_sqrt)(vhat[t]) : med;
    }
}

typedef struct { REAL mag; int32_t idx; } FN(orc_pair);

static int FN(orc_cmp_mag_desc)(const void *pa, const void *pb)
{
    const FN(orc_pair) *a = (const FN(orc_pair) *)pa, *b = (const FN(orc_pair) *)pb;
    if (a->mag > b->mag) return -1;
    if (a->mag < b->mag) return 1;
    return (a->idx > b->idx) - (a->idx < b->idx);
}

/* Top-k of |est|: full sort by (magnitude descending, index ascending), keep the first k,
 * return their indices in ascending order.  Returns 0, or -1 if memory runs out. */
int FN(orc_topk)(const REAL *est, int64_t d, int64_t k, int32_t *idx /* [k] */)
{
    FN(orc_pair) *p = (FN(orc_pair) *)malloc((size_t)d * sizeof(*p));
    if (!p) return -1;
    for (int64_t l = 0; l < d; ++l) {
        p[l].mag = est[l] < (REAL)0 ? -est[l] : est[l];
        if (p[l].mag == (REAL)0) p[l].mag = (REAL)0; /* -0 and +0 are the same magnitude */
        p[l].idx = (int32_t)l;
    }
    qsort(p, (size_t)d, sizeof(*p), FN(orc_cmp_mag_desc));
    for (int64_t q = 0; q < k; ++q) idx[q] = p[q].idx;
    free(p);
    qsort(idx, (size_t)k, sizeof(int32_t), orc_cmp_i32);
    return 0;
}

/* Sec. III-A, over-selection: among k_in candidates (ascending coordinates idx_in with their exact averaged
 * values delta_in) keep the k_out with the largest magnitude, ties to the smaller coordinate, ascending. */
int FN(orc_refine)(const int32_t *idx_in, const REAL *delta_in, int64_t k_in, int64_t k_out, int32_t *idx_out,
                   REAL *delta_out)
{
    int32_t *pos = (int32_t *)malloc((size_t)k_out * sizeof(int32_t));
    if (!pos) return -1;
    if (FN(orc_topk)(delta_in, k_in, k_out, pos) != 0) { free(pos); return -1; }
    for (int64_t q = 0; q < k_out; ++q) {
        idx_out[q] = idx_in[pos[q]];
        delta_out[q] = delta_in[pos[q]];
    }
    free(pos);
    return 0;
}

/* Second round (Sec. III-A) and the definition of Delta_t^(i) under Alg. 2:
 * U^(i)[q] = u^(i)[idx[q]];  Delta[q] = ((sum_i U^(i)[q]) / n) / sqrt(vhat[idx[q]]). */
void FN(orc_gather)(const REAL *u /* [n][d] */, const REAL *vhat /* [d] or NULL */,
                    const int32_t *idx, int64_t k, int32_t n, int64_t d,
                    REAL *U_w /* [n][k] */, REAL *delta /* [k] */)
{
    for (int64_t q = 0; q < k; ++q) {
        int64_t l = idx[q];
        REAL acc = (REAL)0;
        for (int32_t i = 0; i < n; ++i) {
            REAL val = u[(int64_t)i * d + l];
            U_w[(int64_t)i * k + q] = val;
            acc = (i == 0) ? val : acc + val;
        }
        REAL mean = acc / (REAL)n;
        delta[q] = vhat ? mean / FN(orc_sqrt)(vhat[l]) : mean;
    }
}

/* Alg. 2, first half of iteration t.
 *   worker i:  m_t = beta1 m_{t-1} + (1-beta1) g_t ;  u = m_t + rho e_{t-1}   (u is written over e)
 *   master:    h_t = mean_i g_t^(i) on I_{t-1}, 0 elsewhere
 *              v_t = beta2 v_{t-1} + (1-beta2) h_t^2 ;  vhat_t = max(vhat_{t-1}, v_t)
 * in_prev[l] != 0 marks l in I_{t-1} (NULL = empty set, the first iteration).
 * omb1 = 1-beta1 and omb2 = 1-beta2 are passed in, already rounded to REAL. */
void FN(orc_head)(const REAL *g /* [n][d] */, REAL *m /* [n][d] */, REAL *e_u /* [n][d] */,
                  REAL *v, REAL *vhat /* [d] */, const uint8_t *in_prev /* [d] or NULL */,
                  int32_t n, int64_t d, REAL beta1, REAL omb1, REAL beta2, REAL omb2, REAL rho)
{
    for (int32_t i = 0; i < n; ++i) {
        for (int64_t l = 0; l < d; ++l) {
            int64_t t = (int64_t)i * d + l;
            REAL mm = beta1 * m[t] + omb1 * g[t];
            m[t] = mm;
            e_u[t] = mm + rho * e_u[t];
        }
    }
    for (int64_t l = 0; l < d; ++l) {
        REAL h = (REAL)0;
        if (in_prev && in_prev[l]) {
            REAL acc = g[l];
            for (int32_t i = 1; i < n; ++i) acc = acc + g[(int64_t)i * d + l];
            h = acc / (REAL)n;
        }
        REAL vv = beta2 * v[l] + omb2 * (h * h);
        v[l] = vv;
        if (vv > vhat[l]) vhat[l] = vv;
    }
}

/* Alg. 1 (parameter averaging), worker lines of iteration t; every worker keeps its own second moments:
 *   m_t = beta1 m_{t-1} + (1-beta1) g_t ;  v_t = beta2 v_{t-1} + (1-beta2) g_t^2 ;  vhat_t = max(vhat_{t-1}, v_t)
 *   u = m_t / sqrt(vhat_t) + rho e_{t-1}        (the vector that is sketched; written over e)
 * The rest of the iteration is Alg. 1's master lines: plain unsketch U_0 (no second input), Top-k, and the
 * same e_t / x_{t+1} lines as in Alg. 2 (orc_tail). */
void FN(orc_head_pa)(const REAL *g /* [n][d] */, REAL *m, REAL *e_u, REAL *v_w, REAL *vhat_w /* [n][d] each */,
                     int32_t n, int64_t d, REAL beta1, REAL omb1, REAL beta2, REAL omb2, REAL rho)
{
    for (int64_t t = 0; t < (int64_t)n * d; ++t) {
        REAL mm = beta1 * m[t] + omb1 * g[t];
        REAL vv = beta2 * v_w[t] + omb2 * (g[t] * g[t]);
        m[t] = mm;
        v_w[t] = vv;
        if (vv > vhat_w[t]) vhat_w[t] = vv;
        e_u[t] = mm / FN(orc_sqrt)(vhat_w[t]) + rho * e_u[t];
    }
}

/* Alg. 2, second half of iteration t.
 *   e_t^(i) = u^(i) off I_t, 0 on I_t (proof of Lemma 3);  x_{t+1} = x_t - alpha_t Delta_t,
 *   Delta_t being non-zero only on I_t. */
void FN(orc_tail)(REAL *e_u /* [n][d]: u in, e out */, REAL *x /* [d] */, const int32_t *idx,
                  const REAL *delta, int64_t k, int32_t n, int64_t d, REAL lr)
{
    for (int64_t q = 0; q < k; ++q) {
        int64_t l = idx[q];
        for (int32_t i = 0; i < n; ++i) e_u[(int64_t)i * d + l] = (REAL)0;
        x[l] = x[l] - lr * delta[q];
    }
}

/* One full iteration of Alg. 2 in the paper's order.  State (m, e, v, vhat, x, in_prev) is
 * updated in place; idx/delta receive I_t and Delta_t; S_w, S_mean, est, U_w are scratch the
 * caller provides so that every intermediate can be inspected.  Returns 0 or -1 (no memory). */
int FN(orc_step)(const REAL *g, REAL *m, REAL *e_u, REAL *v, REAL *vhat, REAL *x,
                 uint8_t *in_prev /* [d], updated to I_t */, int32_t n, int64_t d, int32_t r,
                 int64_t c, int64_t k, const uint32_t *hash, REAL beta1, REAL omb1, REAL beta2,
                 REAL omb2, REAL rho, REAL lr, int use_vhat, REAL *S_w /* [n][r][c] */,
                 REAL *S_mean /* [r][c] */, REAL *est /* [d] */, int32_t *idx /* [k] */,
                 REAL *U_w /* [n][k] */, REAL *delta /* [k] */)
{
    FN(orc_head)(g, m, e_u, v, vhat, in_prev, n, d, beta1, omb1, beta2, omb2, rho);
    for (int32_t i = 0; i < n; ++i)
        FN(orc_sketch)(e_u + (int64_t)i * d, d, r, c, hash, S_w + (int64_t)i * r * c);
    FN(orc_sketch_mean)(S_w, n, r, c, S_mean);
    FN(orc_unsketch)(S_mean, use_vhat ? vhat : NULL, d, r, c, hash, est, 0);
    if (FN(orc_topk)(est, d, k, idx) != 0) return -1;
    FN(orc_gather)(e_u, use_vhat ? vhat : NULL, idx, k, n, d, U_w, delta);
    FN(orc_tail)(e_u, x, idx, delta, k, n, d, lr);
    for (int64_t l = 0; l < d; ++l) in_prev[l] = 0;
    for (int64_t q = 0; q < k; ++q) in_prev[idx[q]] = 1;
    return 0;
}

#undef FN
#undef ORC_CAT
#undef ORC_CAT_
