/*
 * CPU oracle for the CSAttention offline table build and online decode step.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, written from the paper's definitions; it shares no
 * code with the HIP library and the library never calls it.  Only the test-suite, the smoke
 * check and the benchmark's "cpu_baseline" leg may load it.
 *
 * Every function cites the passage of the paper (arXiv 2604.08584) it follows.  Where the
 * paper leaves a choice open the reading taken is stated at the function.
 *
 * Geometry implemented: the head dimension is cut uniformly into S subspaces of d/S dimensions
 * (Sec. 3.1 (i)); each subspace has its own C centroids and its own C table rows; a query
 * probes the tau best centroids of every subspace (Sec. 3.3 (1) for tau = 1, the centroid
 * back-off of Sec. 4.4 for tau > 1), M = S * tau rows in all.  S = 1 is the single-subspace
 * geometry of the benchmark configurations; S = 8, tau = 1 is the paper's default.  Row r of a
 * KV head's table belongs to subspace r / C and centroid r % C.  Everything after centroid
 * choice (Sec. 3.3 steps 2-4) is independent of how the probed rows were chosen.
 *
 * Precision: the three places where floating point decides an integer are taken in fp32 with
 * a fixed operation order, so that any implementation can reproduce them bit for bit:
 *   - centroid-query scores and centroid-key scores: one fused-multiply-add chain over
 *     ascending dimension, starting from +0, inputs widened from bf16;
 *   - table scores are rounded to the grid 2^-F (round half to even) when the table is
 *     built; with m * max|score| * 2^F < 2^24 every partial sum of at most m scores is exact
 *     in fp32, so the per-key accumulation does not depend on the order of the additions.
 * Attention itself (logits, softmax, weighted sum) is done in fp64.
 *
 * Compile with -ffp-contract=off: the only fused operations are the explicit fmaf calls.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- bf16 helpers */

static float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round-to-nearest-even fp32 -> bf16 (finite inputs) */
static uint16_t f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* ---------------------------------------------------------------- ordering helpers */

typedef struct {
    float score;
    int32_t idx;
} pair_t;

/* larger score first; equal scores: smaller index first (compared as real numbers, so
 * -0 and +0 tie) */
static int cmp_score_desc_idx_asc(const void *a, const void *b)
{
    const pair_t *x = (const pair_t *)a, *y = (const pair_t *)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    if (x->idx < y->idx) return -1;
    if (x->idx > y->idx) return 1;
    return 0;
}

static int cmp_i32_asc(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* fp32 inner product as one fma chain over ascending dimension, from +0 */
static float dot_chain_bf16(const uint16_t *a, const uint16_t *b, int d)
{
    float acc = 0.0f;
    for (int t = 0; t < d; ++t)
        acc = fmaf(bf16_to_f32(a[t]), bf16_to_f32(b[t]), acc);
    return acc;
}

/* ---------------------------------------------------------------- dense attention */

/*
 * Sec. 2.1: a = softmax(q K^T / sqrt(d)), o = a V, over rows [0, n) of K and V.
 * Also the plain definition that the sparse path must reduce to when nothing is pruned.
 */
void oracle_dense_attention(const uint16_t *q, const uint16_t *K, const uint16_t *V,
                            int64_t n, int d, float *out)
{
    double *logit = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    double mx = -INFINITY;
    for (int64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int t = 0; t < d; ++t)
            s += (double)bf16_to_f32(q[t]) * (double)bf16_to_f32(K[i * d + t]);
        logit[i] = s / sqrt((double)d);
        if (logit[i] > mx) mx = logit[i];
    }
    double *o = (double *)calloc((size_t)d, sizeof(double));
    double den = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double p = exp(logit[i] - mx);
        den += p;
        for (int t = 0; t < d; ++t) o[t] += p * (double)bf16_to_f32(V[i * d + t]);
    }
    for (int t = 0; t < d; ++t) out[t] = n > 0 ? (float)(o[t] / den) : 0.0f;
    free(o);
    free(logit);
}

/*
 * Sec. 3.3 step 4 ("only these K keys are used in attention") with Sec. 2.1's formula: the
 * same softmax attention, restricted to the listed rows.  An empty list gives a zero output.
 */
static void attention_over(const uint16_t *q, const uint16_t *K, const uint16_t *V,
                           const int32_t *ids, int64_t n_ids, int d, float *out)
{
    double *logit = (double *)malloc(sizeof(double) * (size_t)(n_ids > 0 ? n_ids : 1));
    double mx = -INFINITY;
    for (int64_t a = 0; a < n_ids; ++a) {
        const uint16_t *kr = K + (int64_t)ids[a] * d;
        double s = 0.0;
        for (int t = 0; t < d; ++t)
            s += (double)bf16_to_f32(q[t]) * (double)bf16_to_f32(kr[t]);
        logit[a] = s / sqrt((double)d);
        if (logit[a] > mx) mx = logit[a];
    }
    double *o = (double *)calloc((size_t)d, sizeof(double));
    double den = 0.0;
    for (int64_t a = 0; a < n_ids; ++a) {
        const uint16_t *vr = V + (int64_t)ids[a] * d;
        double p = exp(logit[a] - mx);
        den += p;
        for (int t = 0; t < d; ++t) o[t] += p * (double)bf16_to_f32(vr[t]);
    }
    for (int t = 0; t < d; ++t) out[t] = n_ids > 0 ? (float)(o[t] / den) : 0.0f;
    free(o);
    free(logit);
}

/* ---------------------------------------------------------------- offline: clustering */

/*
 * Sec. 3.2 (1): cosine k-means on the l2-normalised prefill queries, unit-norm centroids,
 * k-means++ seeding, `iters` Lloyd iterations (full batch: the mini-batch size is not given).
 *   x      [n][d] fp32 prefill queries (any scale)
 *   u_seed [C]    uniforms in [0,1) that drive the seeding (passed in, never drawn here)
 *   cent   [C][d] fp32 out, unit norm
 *   objective [iters+1] out: sum_q min_j ||q~ - c_j||^2 before each iteration and after
 *             the last one (non-increasing for Lloyd iterations).
 * An empty cluster keeps its centroid.  Assignment ties go to the lowest centroid.
 */
void oracle_kmeans(const float *x, int64_t n, int d, int C, int iters, const double *u_seed,
                   float *cent, double *objective)
{
    double *xn = (double *)malloc(sizeof(double) * (size_t)n * d);
    double *c = (double *)malloc(sizeof(double) * (size_t)C * d);
    double *dist = (double *)malloc(sizeof(double) * (size_t)n);
    int32_t *asg = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    for (int64_t i = 0; i < n; ++i) {
        double nn = 0.0;
        for (int t = 0; t < d; ++t) nn += (double)x[i * d + t] * x[i * d + t];
        nn = sqrt(nn);
        for (int t = 0; t < d; ++t) xn[i * d + t] = nn > 0 ? x[i * d + t] / nn : 0.0;
    }
    /* k-means++: first centre uniform, then proportional to squared distance to the
     * nearest chosen centre */
    int64_t first = (int64_t)(u_seed[0] * (double)n);
    if (first >= n) first = n - 1;
    memcpy(c, xn + first * d, sizeof(double) * d);
    for (int64_t i = 0; i < n; ++i) dist[i] = INFINITY;
    for (int j = 1; j <= C; ++j) {
        /* fold centre j-1 into the nearest-centre distances */
        double tot = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            double s = 0.0;
            for (int t = 0; t < d; ++t) {
                double df = xn[i * d + t] - c[(j - 1) * d + t];
                s += df * df;
            }
            if (s < dist[i]) dist[i] = s;
            tot += dist[i];
        }
        if (j == C) break;
        double target = u_seed[j] * tot, run = 0.0;
        int64_t pick = n - 1;
        for (int64_t i = 0; i < n; ++i) {
            run += dist[i];
            if (run > target) { pick = i; break; }
        }
        memcpy(c + (size_t)j * d, xn + pick * d, sizeof(double) * d);
    }
    double *sum = (double *)malloc(sizeof(double) * (size_t)C * d);
    int64_t *cnt = (int64_t *)malloc(sizeof(int64_t) * (size_t)C);
    for (int it = 0; it <= iters; ++it) {
        double obj = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            int best = 0;
            double bc = -INFINITY;
            for (int j = 0; j < C; ++j) {
                double s = 0.0;
                for (int t = 0; t < d; ++t) s += xn[i * d + t] * c[(size_t)j * d + t];
                if (s > bc) { bc = s; best = j; }
            }
            asg[i] = best;
            double dd = 0.0;
            for (int t = 0; t < d; ++t) {
                double df = xn[i * d + t] - c[(size_t)best * d + t];
                dd += df * df;
            }
            obj += dd;
        }
        objective[it] = obj;
        if (it == iters) break;
        memset(sum, 0, sizeof(double) * (size_t)C * d);
        memset(cnt, 0, sizeof(int64_t) * (size_t)C);
        for (int64_t i = 0; i < n; ++i) {
            cnt[asg[i]]++;
            for (int t = 0; t < d; ++t) sum[(size_t)asg[i] * d + t] += xn[i * d + t];
        }
        for (int j = 0; j < C; ++j) {
            double nn = 0.0;
            for (int t = 0; t < d; ++t) nn += sum[(size_t)j * d + t] * sum[(size_t)j * d + t];
            nn = sqrt(nn);
            if (cnt[j] == 0 || nn == 0.0) continue;
            for (int t = 0; t < d; ++t) c[(size_t)j * d + t] = sum[(size_t)j * d + t] / nn;
        }
    }
    for (size_t e = 0; e < (size_t)C * d; ++e) cent[e] = (float)c[e];
    free(sum); free(cnt); free(xn); free(c); free(dist); free(asg);
}

/*
 * The same clustering with the centroids held in bf16 between the steps - the form in which
 * the tables' build consumes them - split into its two parts so that each can be checked on its
 * own: k-means++ seeding (every seed is a normalised data point, rounded to bf16; the next one is
 * drawn with probability proportional to the squared distance to the nearest seed so far, from the
 * uniform u_seed[j]) and one Lloyd step (cosine assignment against the bf16 centroids, ties to
 * the lowest centroid; centroid <- mean of its normalised members, re-normalised, rounded to
 * bf16; an empty cluster keeps its centroid).
 *   x [n][d] fp32 (any scale), cent bf16 [C][d].
 *   oracle_kmeans_step also returns, per point, its assignment and the gap between its best and
 *   second-best cosine (how close the decision was), and the mean best cosine.
 */
void oracle_kmeans_seed(const float *x, int64_t n, int d, int C, const double *u_seed, uint16_t *cent,
                        int64_t *picks, double *margin)
{
    /* picks[j] (optional): the point taken as seed j.  margin[j] (optional, j >= 1): how far the
     * draw's target u_j * total was from the nearer end of the picked point's stretch of the running
     * sum, as a fraction of the total - a draw with a tiny margin is one that rounding may move to a
     * neighbouring point.  margin[0] = 0. */
    double *xn = (double *)malloc(sizeof(double) * (size_t)d);
    double *dist = (double *)malloc(sizeof(double) * (size_t)n);
    for (int64_t i = 0; i < n; ++i) dist[i] = INFINITY;
    int64_t pick = (int64_t)(u_seed[0] * (double)n);
    if (pick >= n) pick = n - 1;
    if (margin) margin[0] = 0.0;
    for (int j = 0; j < C; ++j) {
        if (picks) picks[j] = pick;
        /* seed j = the normalised point `pick`, rounded to bf16 */
        double nn = 0.0;
        for (int t = 0; t < d; ++t) nn += (double)x[pick * d + t] * x[pick * d + t];
        nn = sqrt(nn);
        for (int t = 0; t < d; ++t) cent[(int64_t)j * d + t] = f32_to_bf16(nn > 0 ? (float)(x[pick * d + t] / nn) : 0.0f);
        if (j + 1 == C) break;
        /* fold it into the nearest-seed distances, draw the next one */
        double tot = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            double ni = 0.0, s = 0.0;
            for (int t = 0; t < d; ++t) ni += (double)x[i * d + t] * x[i * d + t];
            ni = sqrt(ni);
            for (int t = 0; t < d; ++t) {
                double df = (ni > 0 ? x[i * d + t] / ni : 0.0) - (double)bf16_to_f32(cent[(int64_t)j * d + t]);
                s += df * df;
            }
            if (s < dist[i]) dist[i] = s;
            tot += dist[i];
        }
        double target = u_seed[j + 1] * tot, run = 0.0, before = 0.0;
        pick = n - 1;
        for (int64_t i = 0; i < n; ++i) {
            before = run;
            run += dist[i];
            if (run > target) { pick = i; break; }
        }
        if (margin) {
            const double lo = target - before, hi = run - target;
            margin[j + 1] = tot > 0.0 ? fmin(fabs(lo), fabs(hi)) / tot : 0.0;
        }
    }
    free(xn); free(dist);
}

/*
 * One step of the mini-batch form of the same clustering (Sec. 3.2 (1) names mini-batch k-means;
 * the update is the per-centre running mean of the mini-batch k-means algorithm, Sculley 2010: a
 * centre is the mean of every point ever assigned to it, the starting centre carrying no weight -
 * here the mean direction, re-normalised and rounded to bf16).  The points of this batch are
 * assigned to the bf16 centroids as in oracle_kmeans_step, then added to the running sums and
 * counts, which the caller keeps between the steps (all zero before the first); a centre whose
 * running count is still zero keeps its centroid.  With one batch holding every point and zeroed
 * sums this is oracle_kmeans_step.
 *   run_sum [C][d] fp64, run_cnt [C] int64: in/out.
 */
double oracle_kmeans_minibatch_step(const float *x, int64_t n, int d, int C, const uint16_t *cent_in,
                                    uint16_t *cent_out, int32_t *assign, double *gap, double *run_sum,
                                    int64_t *run_cnt)
{
    double *xn = (double *)malloc(sizeof(double) * (size_t)d);
    double cos_sum = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double nn = 0.0;
        for (int t = 0; t < d; ++t) nn += (double)x[i * d + t] * x[i * d + t];
        nn = sqrt(nn);
        for (int t = 0; t < d; ++t) xn[t] = nn > 0 ? x[i * d + t] / nn : 0.0;
        int best = 0;
        double b1 = -INFINITY, b2 = -INFINITY;
        for (int j = 0; j < C; ++j) {
            double s = 0.0;
            for (int t = 0; t < d; ++t) s += xn[t] * (double)bf16_to_f32(cent_in[(int64_t)j * d + t]);
            if (s > b1) { b2 = b1; b1 = s; best = j; }
            else if (s > b2) b2 = s;
        }
        assign[i] = best;
        if (gap) gap[i] = b1 - b2;
        cos_sum += b1;
        run_cnt[best]++;
        for (int t = 0; t < d; ++t) run_sum[(int64_t)best * d + t] += xn[t];
    }
    for (int j = 0; j < C; ++j) {
        double nn = 0.0;
        for (int t = 0; t < d; ++t) nn += run_sum[(int64_t)j * d + t] * run_sum[(int64_t)j * d + t];
        nn = sqrt(nn);
        for (int t = 0; t < d; ++t)
            cent_out[(int64_t)j * d + t] = (run_cnt[j] == 0 || nn == 0.0)
                                               ? cent_in[(int64_t)j * d + t]
                                               : f32_to_bf16((float)(run_sum[(int64_t)j * d + t] / nn));
    }
    free(xn);
    return n > 0 ? cos_sum / (double)n : 0.0;
}

double oracle_kmeans_step(const float *x, int64_t n, int d, int C, const uint16_t *cent_in,
                          uint16_t *cent_out, int32_t *assign, double *gap)
{
    double *sum = (double *)calloc((size_t)C * d, sizeof(double));
    int64_t *cnt = (int64_t *)calloc((size_t)C, sizeof(int64_t));
    double *xn = (double *)malloc(sizeof(double) * (size_t)d);
    double cos_sum = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double nn = 0.0;
        for (int t = 0; t < d; ++t) nn += (double)x[i * d + t] * x[i * d + t];
        nn = sqrt(nn);
        for (int t = 0; t < d; ++t) xn[t] = nn > 0 ? x[i * d + t] / nn : 0.0;
        int best = 0;
        double b1 = -INFINITY, b2 = -INFINITY;
        for (int j = 0; j < C; ++j) {
            double s = 0.0;
            for (int t = 0; t < d; ++t) s += xn[t] * (double)bf16_to_f32(cent_in[(int64_t)j * d + t]);
            if (s > b1) { b2 = b1; b1 = s; best = j; }
            else if (s > b2) b2 = s;
        }
        assign[i] = best;
        if (gap) gap[i] = b1 - b2;
        cos_sum += b1;
        cnt[best]++;
        for (int t = 0; t < d; ++t) sum[(int64_t)best * d + t] += xn[t];
    }
    for (int j = 0; j < C; ++j) {
        double nn = 0.0;
        for (int t = 0; t < d; ++t) nn += sum[(int64_t)j * d + t] * sum[(int64_t)j * d + t];
        nn = sqrt(nn);
        for (int t = 0; t < d; ++t)
            cent_out[(int64_t)j * d + t] = (cnt[j] == 0 || nn == 0.0)
                                               ? cent_in[(int64_t)j * d + t]
                                               : f32_to_bf16((float)(sum[(int64_t)j * d + t] / nn));
    }
    free(sum); free(cnt); free(xn);
    return n > 0 ? cos_sum / (double)n : 0.0;
}

/* fp32 -> bf16 rounding of a centroid matrix, done once after clustering */
void oracle_round_bf16(const float *x, int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = f32_to_bf16(x[i]);
}

/* ---------------------------------------------------------------- offline: table rows */

/*
 * Sec. 3.2 (2): s_j^(b)(i) = c_j^(b) . k_i^(b) for every prefill key i (raw key sub-vectors, unit
 * centroids, as the equation is written), keep the Top-L pairs, stored sorted by score
 * (Sec. 3.1 (iii)).  Ties go to the lower key index.  Scores are rounded to the grid 2^-F before
 * the ranking.  Rows shorter than L (n_pre < L) are padded with idx = -1, score = 0.
 *   K        [n_pre][d] bf16
 *   cent     [S][C][d/S] bf16 (S = n_sub subspaces, dimensions [b*d/S, (b+1)*d/S) of the head)
 *   row_ids  [n_rows]  which rows to build (row = b*C + j; any subset, any order)
 *   idx_out / score_out [n_rows][L]
 * Returns the largest |q| = |round(s * 2^F)| seen, as a double (for the exactness check
 * M * max|q| < 2^24).
 */
double oracle_build_rows(const uint16_t *K, int64_t n_pre, int d, int n_sub, int C,
                         const uint16_t *cent, const int32_t *row_ids, int n_rows, int L, int F,
                         int32_t *idx_out, float *score_out)
{
    double max_abs_q = 0.0;
    const float up = ldexpf(1.0f, F), down = ldexpf(1.0f, -F);
    const int db = d / n_sub;
#pragma omp parallel for schedule(dynamic) reduction(max : max_abs_q)
    for (int r = 0; r < n_rows; ++r) {
        pair_t *all = (pair_t *)malloc(sizeof(pair_t) * (size_t)(n_pre > 0 ? n_pre : 1));
        const int b = row_ids[r] / C;
        const uint16_t *c = cent + (int64_t)row_ids[r] * db;
        for (int64_t i = 0; i < n_pre; ++i) {
            float s = dot_chain_bf16(c, K + i * d + (int64_t)b * db, db);
            float qf = rintf(s * up); /* default rounding mode: half to even */
            if (fabs((double)qf) > max_abs_q) max_abs_q = fabs((double)qf);
            all[i].score = qf * down;
            all[i].idx = (int32_t)i;
        }
        qsort(all, (size_t)n_pre, sizeof(pair_t), cmp_score_desc_idx_asc);
        for (int p = 0; p < L; ++p) {
            if (p < n_pre) {
                idx_out[(int64_t)r * L + p] = all[p].idx;
                score_out[(int64_t)r * L + p] = all[p].score;
            } else {
                idx_out[(int64_t)r * L + p] = -1;
                score_out[(int64_t)r * L + p] = 0.0f;
            }
        }
        free(all);
    }
    return max_abs_q;
}

/* ---------------------------------------------------------------- online: streaming updates */

/*
 * Sec. 3.3 (5): after a new key k_S (index idx_new, larger than every index in the tables) has
 * been appended, score it against every centroid of every subspace, score = c_j^(b) . k_S^(b)
 * (same fma chain and grid as the table build), and try-insert it into that centroid's
 * fixed-capacity Top-L list: a list with a free slot takes it; a full list takes it only if it
 * beats the list's minimum, which is evicted (an equal score does not beat it: the older key has
 * the lower index).  Lists stay sorted by (score desc, idx asc); capacity L never changes.
 *   tbl_idx / tbl_score [S*C][L] in place.  Returns the largest |q| of the new key's scores.
 */
double oracle_try_insert(int32_t *tbl_idx, float *tbl_score, int L, const uint16_t *cent,
                         int n_sub, int C, int d, const uint16_t *k_new, int32_t idx_new, int F)
{
    const float up = ldexpf(1.0f, F), down = ldexpf(1.0f, -F);
    const int db = d / n_sub;
    double max_abs_q = 0.0;
    for (int r = 0; r < n_sub * C; ++r) {
        int32_t *I = tbl_idx + (int64_t)r * L;
        float *S = tbl_score + (int64_t)r * L;
        const int b = r / C;
        float qf = rintf(dot_chain_bf16(cent + (int64_t)r * db, k_new + b * db, db) * up);
        if (fabs((double)qf) > max_abs_q) max_abs_q = fabs((double)qf);
        float sc = qf * down;
        int cnt = 0;
        while (cnt < L && I[cnt] >= 0) ++cnt;
        if (cnt == L) {
            if (!(sc > S[L - 1])) continue; /* does not beat the minimum */
            cnt = L - 1;                    /* evict it */
        }
        int p = cnt; /* slide larger-index-or-smaller-score entries one slot down */
        while (p > 0 && S[p - 1] < sc) {
            I[p] = I[p - 1];
            S[p] = S[p - 1];
            --p;
        }
        I[p] = idx_new;
        S[p] = sc;
    }
    return max_abs_q;
}

/* ---------------------------------------------------------------- online: decode */

/*
 * Sec. 3.3 step 1 with the back-off of Sec. 4.4: in every subspace b, z_j = q^(b) . c_j^(b), the
 * tau largest, ties to the lower j.  q is not normalised: a positive factor per subspace cannot
 * change that subspace's ranking.
 *   cent [S][C][d/S]; rows_out [S*tau]: subspace-major, best first, as table rows b*C + j;
 *   z_out [S][C] or NULL.
 */
void oracle_top_centroids(const uint16_t *q, const uint16_t *cent, int n_sub, int C, int d, int tau,
                          int32_t *rows_out, float *z_out)
{
    const int db = d / n_sub;
    pair_t *z = (pair_t *)malloc(sizeof(pair_t) * (size_t)C);
    for (int b = 0; b < n_sub; ++b) {
        for (int j = 0; j < C; ++j) {
            z[j].score = dot_chain_bf16(q + b * db, cent + ((int64_t)b * C + j) * db, db);
            z[j].idx = j;
            if (z_out) z_out[(int64_t)b * C + j] = z[j].score;
        }
        qsort(z, (size_t)C, sizeof(pair_t), cmp_score_desc_idx_asc);
        for (int r = 0; r < tau; ++r) rows_out[b * tau + r] = r < C ? b * C + z[r].idx : -1;
    }
    free(z);
}

/*
 * Sec. 3.3 steps 2-4 for one query head, given the probed rows.
 *   step 2: read the m rows (I_j, V_j) -> up to m*L (idx, score) pairs;
 *   step 3: score(i) = sum over the probed rows that contain i of that row's score for i
 *           (w_b = 1); U = the keys that occur in at least one probed row; a key that is
 *           absent from a row gets nothing from it;
 *   step 4: keep the min(k, |U|) members of U with the largest score, ties to the lower
 *           index; reported in ascending index order, padded with -1.
 * Only key indices below n_pre are candidates: entries at or above it (keys of the always-attended
 * recent window, which streaming updates may have put into the tables) are skipped.
 * acc_out (optional, [n_pre]) receives score(i), NaN for keys outside U.
 * Returns |U|.
 */
int64_t oracle_select_keys(const int32_t *tbl_idx, const float *tbl_score, int L,
                           const int32_t *rows, int m, int64_t n_pre, int k,
                           int32_t *sel_out, int32_t *sel_count, float *acc_out)
{
    float *acc = (float *)calloc((size_t)(n_pre > 0 ? n_pre : 1), sizeof(float));
    uint8_t *seen = (uint8_t *)calloc((size_t)(n_pre > 0 ? n_pre : 1), 1);
    for (int r = 0; r < m; ++r) {
        if (rows[r] < 0) continue;
        const int32_t *I = tbl_idx + (int64_t)rows[r] * L;
        const float *S = tbl_score + (int64_t)rows[r] * L;
        for (int p = 0; p < L; ++p) {
            int32_t i = I[p];
            if (i < 0 || i >= n_pre) continue;
            acc[i] += S[p];
            seen[i] = 1;
        }
    }
    int64_t nU = 0;
    for (int64_t i = 0; i < n_pre; ++i) nU += seen[i];
    pair_t *u = (pair_t *)malloc(sizeof(pair_t) * (size_t)(nU > 0 ? nU : 1));
    int64_t w = 0;
    for (int64_t i = 0; i < n_pre; ++i)
        if (seen[i]) {
            u[w].score = acc[i];
            u[w].idx = (int32_t)i;
            ++w;
        }
    qsort(u, (size_t)nU, sizeof(pair_t), cmp_score_desc_idx_asc);
    int keff = (int64_t)k < nU ? k : (int)nU;
    for (int a = 0; a < keff; ++a) sel_out[a] = u[a].idx;
    qsort(sel_out, (size_t)keff, sizeof(int32_t), cmp_i32_asc);
    for (int a = keff; a < k; ++a) sel_out[a] = -1;
    *sel_count = keff;
    if (acc_out)
        for (int64_t i = 0; i < n_pre; ++i) acc_out[i] = seen[i] ? acc[i] : NAN;
    free(u); free(acc); free(seen);
    return nU;
}

/*
 * One decode step for one query head: Sec. 3.3 steps 1-4 followed by exact attention over
 * the selected keys plus the recent window, rows [n_pre, n): always attended, never competing
 * for the k slots.  Without streaming updates the window is every key appended after prefill and
 * n_pre is the prefill length; with them (Sec. 3.3 (5)) older appended keys compete through the
 * tables and the caller passes n_pre = max(0, n - R), the start of the last R positions.
 *   q [d], cent [S][C][d/S], K / V [>= n][d] bf16; tables [S*C][L]; tau probes per subspace.
 *   rows_out [S*tau], sel_out [k] (ascending, -1 padded), sel_count [1], out [d] fp32.
 */
void oracle_decode_head(const uint16_t *q, const uint16_t *cent, int n_sub, int C, int d,
                        const int32_t *tbl_idx, const float *tbl_score, int L, int tau, int k,
                        const uint16_t *K, const uint16_t *V, int64_t n_pre, int64_t n,
                        int32_t *rows_out, int32_t *sel_out, int32_t *sel_count, float *out)
{
    const int m = n_sub * tau;
    oracle_top_centroids(q, cent, n_sub, C, d, tau, rows_out, NULL);
    oracle_select_keys(tbl_idx, tbl_score, L, rows_out, m, n_pre, k, sel_out, sel_count, NULL);
    int64_t n_att = *sel_count + (n - n_pre);
    int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_att > 0 ? n_att : 1));
    for (int a = 0; a < *sel_count; ++a) ids[a] = sel_out[a];
    for (int64_t i = n_pre; i < n; ++i) ids[*sel_count + (i - n_pre)] = (int32_t)i;
    attention_over(q, K, V, ids, n_att, d, out);
    free(ids);
}

/*
 * A decode step inside a search period (App. "Schedules" / complexity appendix: with search
 * period P the index set found by the last searching step is reused for the next P-1 steps):
 * no centroid scoring, no table access - exact attention over the given index set plus every
 * key appended after prefill, rows [n_pre, n), with the current query.
 *   sel [count]: prefill key indices (any order, distinct), each < n_pre.
 */
void oracle_attend_selected(const uint16_t *q, const uint16_t *K, const uint16_t *V,
                            const int32_t *sel, int count, int64_t n_pre, int64_t n, int d,
                            float *out)
{
    int64_t n_att = count + (n - n_pre);
    int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_att > 0 ? n_att : 1));
    for (int a = 0; a < count; ++a) ids[a] = sel[a];
    for (int64_t i = n_pre; i < n; ++i) ids[count + (i - n_pre)] = (int32_t)i;
    attention_over(q, K, V, ids, n_att, d, out);
    free(ids);
}

/*
 * The same step for a list of independent (sequence, query head) items, spread over
 * `n_threads` OpenMP threads (0 = the runtime's default).  Item t uses q[t], cent[t] (its KV
 * head's centroids), tbl_idx[t] / tbl_score[t] (its KV head's tables) and K[t] / V[t] (its KV
 * head's cache); outputs are packed [n_items][S*tau], [n_items][k], [n_items], [n_items][d].
 * Returns the number of threads used.
 */
int oracle_decode_items(int n_items, const uint16_t *const *q, const uint16_t *const *cent,
                        const int32_t *const *tbl_idx, const float *const *tbl_score,
                        const uint16_t *const *K, const uint16_t *const *V, int n_sub, int C, int d,
                        int L, int tau, int k, int64_t n_pre, int64_t n, int32_t *rows_out,
                        int32_t *sel_out, int32_t *sel_count, float *out, int n_threads)
{
    int used = 1;
    const int m = n_sub * tau;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#endif
#pragma omp parallel for schedule(dynamic)
    for (int t = 0; t < n_items; ++t)
        oracle_decode_head(q[t], cent[t], n_sub, C, d, tbl_idx[t], tbl_score[t], L, tau, k, K[t],
                           V[t], n_pre, n, rows_out + (int64_t)t * m, sel_out + (int64_t)t * k,
                           sel_count + t, out + (int64_t)t * d);
    return used;
}
