/*
 * CHAI (Clustered Head Attention) -- plain CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct
 * statement of what the clustered-head decode path computes.  It shares no
 * code, header, table or helper with the HIP library; only the tests, the
 * smoke check and the benchmark's cpu_baseline leg may call it.  The product
 * path never routes through it.
 *
 * Every floating-point quantity is accumulated in fp64, in the index order
 * the definitions state, with no blocking, fusion or reordering.  The file
 * is compiled with -ffp-contract=off so a*b+c is two roundings everywhere
 * (the k-means decisions depend on that).
 *
 * Parity pins (tests marked "not gpu"): library softmax/matmul on small
 * shapes, hand-worked examples, closed forms, the k = H and identical-Q/K
 * reductions to dense attention, brute-force k-means over all partitions,
 * an independent Lloyd implementation with the same start, index gathers,
 * the shared-value ablation against dense attention of the representative,
 * the nearest-to-mean representative against hand-worked cases and numpy,
 * the representatives' projections against a library contraction, the
 * 8-bit floating point codes against the format's published values, a
 * library's conversion and brute-force nearest search, quantised attention
 * against a library softmax/matmul on dequantised tensors.
 * Unpinned: no function of this file.  (How well clustered attention
 * approximates dense attention on trained models is not computed here at
 * all; it needs weights and datasets.)
 *
 * All pointers are HOST pointers.  dtype: 0 = fp32, 1 = bf16 (raw uint16
 * bit patterns, converted exactly by placing them in the top half of an
 * fp32 word).  Return value 0 = ok, non-zero = bad argument.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_F32 0
#define ORC_BF16 1

int chai_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* exact widening of one stored element to double */
static double load_elem(const void *base, int64_t idx, int dtype)
{
    if (dtype == ORC_F32) {
        return (double)((const float *)base)[idx];
    } else {
        uint32_t w = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
        float f;
        memcpy(&f, &w, sizeof f);
        return (double)f;
    }
}

static size_t elem_size(int dtype) { return dtype == ORC_F32 ? 4u : 2u; }

/*
 * Softmax of n scores with the maximum subtracted first (the sigma of the
 * attention definition in Section 2; subtracting the maximum changes
 * nothing mathematically and keeps exp() in range).
 */
static void softmax_row(const double *s, int64_t n, double *p)
{
    double m = s[0];
    for (int64_t t = 1; t < n; ++t)
        if (s[t] > m) m = s[t];
    double z = 0.0;
    for (int64_t t = 0; t < n; ++t) {
        p[t] = exp(s[t] - m);
        z += p[t];
    }
    for (int64_t t = 0; t < n; ++t) p[t] = p[t] / z;
}

/*
 * One decode step of clustered-head attention for one layer (Sections 3.4
 * and 3.5 with the attention definition of Section 2):
 *
 *   for every batch row b and cluster j with representative head r = rep[b][j]
 *       s[t] = scale * sum_i q[b][r][i] * K[b][r][t][i]          t = 0..T-1
 *       p_j  = softmax(s)
 *   for every head h with cluster c = head_to_cluster[b][h]
 *       out[b][h][:] = sum_t p_c[t] * V[b][h][t][:]
 *
 * Only the representative's query and keys are used; every head keeps its
 * own values (only keys are pruned).  K is the FULL cache [B,H,T_cap,d] and
 * the representative is indexed in it, so a wrong compaction on the device
 * side shows up as an attention mismatch.
 *
 * q [B,H,d], k_full and v [B,H,T_cap,d] in `dtype`; out [B,H,d] double;
 * probs (nullable) [B,k,T] double.  T counts the current token too.
 */
int chai_oracle_clustered_decode(const void *q, const void *k_full, const void *v,
                                 const int32_t *head_to_cluster, const int32_t *rep_heads,
                                 int B, int H, int k, int T, int T_cap, int d, int dtype,
                                 double scale, double *out, double *probs)
{
    if (!q || !k_full || !v || !head_to_cluster || !rep_heads || !out) return 1;
    if (B < 0 || H < 1 || k < 1 || k > H || T < 1 || T > T_cap || d < 1) return 2;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return 3;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            int c = head_to_cluster[(int64_t)b * H + h];
            if (c < 0 || c >= k) return 2;
            /* a head may only point at a cluster slot that is in use */
            int r = rep_heads[(int64_t)b * k + c];
            if (r < 0 || r >= H) return 2;
        }

    double *p_all = (double *)malloc(sizeof(double) * (size_t)B * k * T + 8);
    if (!p_all) return 4;

#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        for (int j = 0; j < k; ++j) {
            double *p = p_all + ((int64_t)b * k + j) * T;
            int r = rep_heads[(int64_t)b * k + j];
            if (r < 0 || r >= H) {
                /* unused cluster slot (checked above: no head points at it) */
                for (int t = 0; t < T; ++t) p[t] = NAN;
                continue;
            }
            double *s = (double *)malloc(sizeof(double) * (size_t)T);
            int64_t qoff = ((int64_t)b * H + r) * d;
            int64_t koff = ((int64_t)b * H + r) * (int64_t)T_cap * d;
            for (int t = 0; t < T; ++t) {
                double acc = 0.0;
                for (int i = 0; i < d; ++i)
                    acc += load_elem(q, qoff + i, dtype) *
                           load_elem(k_full, koff + (int64_t)t * d + i, dtype);
                s[t] = scale * acc;
            }
            softmax_row(s, T, p);
            free(s);
        }
    }

#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            int c = head_to_cluster[(int64_t)b * H + h];
            const double *p = p_all + ((int64_t)b * k + c) * T;
            int64_t voff = ((int64_t)b * H + h) * (int64_t)T_cap * d;
            double *o = out + ((int64_t)b * H + h) * d;
            for (int i = 0; i < d; ++i) {
                double acc = 0.0;
                for (int t = 0; t < T; ++t)
                    acc += p[t] * load_elem(v, voff + (int64_t)t * d + i, dtype);
                o[i] = acc;
            }
        }
    }
    if (probs) memcpy(probs, p_all, sizeof(double) * (size_t)B * k * T);
    free(p_all);
    return 0;
}

/*
 * Clustered-head attention over a block of prompt positions (Section 3.5 and
 * its inference figure: once membership is fixed, clustered attention takes
 * the place of multi-head attention for the rest of the request, i.e. also
 * for the remaining prompt tokens whose cost the time-to-first-token figure
 * of Section 4.4 includes; attention
 * definition of Section 2 with the causal mask of a decoder-only model).
 *
 * Query row i (i = 0..Tq-1) sits at sequence position q_start + i and sees the
 * keys and values of positions 0 .. q_start + i:
 *   for cluster j with representative r:
 *       s[t]   = scale * q[b][r][i] . K[b][r][t]          t <= q_start + i
 *       p_j,i  = softmax(s)
 *   for head h in cluster c:
 *       out[b][h][i][:] = sum_t p_c,i[t] * V[b][h][t][:]
 *
 * q [B,H,Tq,d]; k_full, v [B,H,T_cap,d] (positions 0 .. q_start+Tq-1 valid);
 * out [B,H,Tq,d] double.
 */
int chai_oracle_clustered_prefill(const void *q, const void *k_full, const void *v,
                                  const int32_t *head_to_cluster, const int32_t *rep_heads,
                                  int B, int H, int k, int Tq, int q_start, int T_cap, int d, int dtype,
                                  double scale, double *out)
{
    if (!q || !k_full || !v || !head_to_cluster || !rep_heads || !out) return 1;
    if (B < 0 || H < 1 || k < 1 || k > H || Tq < 1 || q_start < 0 || q_start + Tq > T_cap || d < 1) return 2;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return 3;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            int c = head_to_cluster[(int64_t)b * H + h];
            if (c < 0 || c >= k) return 2;
            int r = rep_heads[(int64_t)b * k + c];
            if (r < 0 || r >= H) return 2;
        }

#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        for (int i = 0; i < Tq; ++i) {
            const int n = q_start + i + 1;               /* keys this row sees */
            double *s = (double *)malloc(sizeof(double) * (size_t)n);
            double *p = (double *)malloc(sizeof(double) * (size_t)n * (size_t)k);
            for (int j = 0; j < k; ++j) {
                int r = rep_heads[(int64_t)b * k + j];
                if (r < 0 || r >= H) continue;
                int64_t qoff = (((int64_t)b * H + r) * Tq + i) * d;
                int64_t koff = ((int64_t)b * H + r) * (int64_t)T_cap * d;
                for (int t = 0; t < n; ++t) {
                    double acc = 0.0;
                    for (int c = 0; c < d; ++c)
                        acc += load_elem(q, qoff + c, dtype) * load_elem(k_full, koff + (int64_t)t * d + c, dtype);
                    s[t] = scale * acc;
                }
                softmax_row(s, n, p + (size_t)j * n);
            }
            for (int h = 0; h < H; ++h) {
                const double *pc = p + (size_t)head_to_cluster[(int64_t)b * H + h] * n;
                int64_t voff = ((int64_t)b * H + h) * (int64_t)T_cap * d;
                double *o = out + (((int64_t)b * H + h) * Tq + i) * d;
                for (int c = 0; c < d; ++c) {
                    double acc = 0.0;
                    for (int t = 0; t < n; ++t) acc += pc[t] * load_elem(v, voff + (int64_t)t * d + c, dtype);
                    o[c] = acc;
                }
            }
            free(s);
            free(p);
        }
    }
    return 0;
}

/*
 * Dense multi-head decode attention, the textbook definition of Section 2:
 * every head h uses its own q, K and V.
 *   out[b][h][:] = softmax_t(scale * q[b][h] . K[b][h][t]) applied to V[b][h]
 * probs (nullable) [B,H,T] double.
 * Written out on its own (not through the clustered routine) so that the
 * "one head per cluster equals dense attention" test compares two separate
 * pieces of code.
 */
int chai_oracle_dense_decode(const void *q, const void *k_cache, const void *v,
                             int B, int H, int T, int T_cap, int d, int dtype,
                             double scale, double *out, double *probs)
{
    if (!q || !k_cache || !v || !out) return 1;
    if (B < 0 || H < 1 || T < 1 || T > T_cap || d < 1) return 2;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return 3;

#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            double *s = (double *)malloc(sizeof(double) * (size_t)T);
            double *p = (double *)malloc(sizeof(double) * (size_t)T);
            int64_t qoff = ((int64_t)b * H + h) * d;
            int64_t coff = ((int64_t)b * H + h) * (int64_t)T_cap * d;
            for (int t = 0; t < T; ++t) {
                double acc = 0.0;
                for (int i = 0; i < d; ++i)
                    acc += load_elem(q, qoff + i, dtype) *
                           load_elem(k_cache, coff + (int64_t)t * d + i, dtype);
                s[t] = scale * acc;
            }
            softmax_row(s, T, p);
            double *o = out + ((int64_t)b * H + h) * d;
            for (int i = 0; i < d; ++i) {
                double acc = 0.0;
                for (int t = 0; t < T; ++t)
                    acc += p[t] * load_elem(v, coff + (int64_t)t * d + i, dtype);
                o[i] = acc;
            }
            if (probs) memcpy(probs + ((int64_t)b * H + h) * T, p, sizeof(double) * (size_t)T);
            free(s);
            free(p);
        }
    }
    return 0;
}

/*
 * Ablation of Section 4.5 (pruning values as well): every head of a cluster
 * also takes the VALUES of the representative, i.e. the whole head is
 * replaced by the representative,
 *     out[b][h][:] = sum_t p_c[t] * V[b][rep[b][c]][t][:],   c = cluster of h,
 * with p_c as in chai_oracle_clustered_decode.  Layouts as there.
 */
int chai_oracle_shared_v_decode(const void *q, const void *k_full, const void *v,
                                const int32_t *head_to_cluster, const int32_t *rep_heads,
                                int B, int H, int k, int T, int T_cap, int d, int dtype,
                                double scale, double *out)
{
    if (!q || !k_full || !v || !head_to_cluster || !rep_heads || !out) return 1;
    if (B < 0 || H < 1 || k < 1 || k > H || T < 1 || T > T_cap || d < 1) return 2;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return 3;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            int c = head_to_cluster[(int64_t)b * H + h];
            if (c < 0 || c >= k) return 2;
            int r = rep_heads[(int64_t)b * k + c];
            if (r < 0 || r >= H) return 2;
        }

#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            int r = rep_heads[(int64_t)b * k + head_to_cluster[(int64_t)b * H + h]];
            double *s = (double *)malloc(sizeof(double) * (size_t)T);
            double *p = (double *)malloc(sizeof(double) * (size_t)T);
            int64_t qoff = ((int64_t)b * H + r) * d;
            int64_t roff = ((int64_t)b * H + r) * (int64_t)T_cap * d;
            for (int t = 0; t < T; ++t) {
                double acc = 0.0;
                for (int i = 0; i < d; ++i)
                    acc += load_elem(q, qoff + i, dtype) *
                           load_elem(k_full, roff + (int64_t)t * d + i, dtype);
                s[t] = scale * acc;
            }
            softmax_row(s, T, p);
            double *o = out + ((int64_t)b * H + h) * d;
            for (int i = 0; i < d; ++i) {
                double acc = 0.0;
                for (int t = 0; t < T; ++t)
                    acc += p[t] * load_elem(v, roff + (int64_t)t * d + i, dtype);
                o[i] = acc;
            }
            free(s);
            free(p);
        }
    }
    return 0;
}

/*
 * Clustering features (Section 3.3: the attention scores a head produces on
 * the first few tokens of a request; Section 3.1 defines the compared
 * quantity as the softmax of Q K^T).  For every (b,h) the n_tok x n_tok
 * causal attention matrix of the first n_tok positions,
 *     A[i][j] = softmax_j( scale * q_i . k_j ),  j <= i,   A[i][j] = 0, j > i,
 * flattened row-major to feat[b][h][i*n_tok + j], rounded to fp32.
 *
 * q5 element (b,h,i,c) sits at (b*H+h)*q_head_stride + i*d + c, likewise k5
 * with k_head_stride, so the keys may be read in place from a cache with
 * head stride T_cap*d.
 */
int chai_oracle_score_features(const void *q5, const void *k5, int B, int H, int n_tok, int d,
                               int dtype, int64_t q_head_stride, int64_t k_head_stride,
                               double scale, float *feat)
{
    if (!q5 || !k5 || !feat) return 1;
    if (B < 0 || H < 1 || n_tok < 1 || n_tok > 64 || d < 1) return 2;
    if (q_head_stride < (int64_t)n_tok * d || k_head_stride < (int64_t)n_tok * d) return 2;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return 3;

    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            int64_t qo = ((int64_t)b * H + h) * q_head_stride;
            int64_t ko = ((int64_t)b * H + h) * k_head_stride;
            float *f = feat + ((int64_t)b * H + h) * n_tok * n_tok;
            for (int i = 0; i < n_tok; ++i) {
                double s[64], p[64];
                for (int j = 0; j <= i; ++j) {
                    double acc = 0.0;
                    for (int c = 0; c < d; ++c)
                        acc += load_elem(q5, qo + (int64_t)i * d + c, dtype) *
                               load_elem(k5, ko + (int64_t)j * d + c, dtype);
                    s[j] = scale * acc;
                }
                softmax_row(s, i + 1, p);
                for (int j = 0; j < n_tok; ++j)
                    f[i * n_tok + j] = (j <= i) ? (float)p[j] : 0.0f;
            }
        }
    }
    return 0;
}

/* squared Euclidean distance, coordinates ascending, multiply and add
 * rounded separately */
static double sqdist(const float *x, const double *c, int F)
{
    double acc = 0.0;
    for (int f = 0; f < F; ++f) {
        double diff = (double)x[f] - c[f];
        double sq = diff * diff;
        acc = acc + sq;
    }
    return acc;
}

/*
 * Clustering error of a partition (Section 3.2: sum of squared distances of
 * the points to the centre of their cluster), with every non-empty
 * cluster's centre at the mean of its members.  `mean` is scratch of F
 * doubles.  Clusters in label order, members in head order, one running sum.
 */
static double partition_error(const float *X, const int32_t *label_of, int H, int F, int k, double *mean)
{
    double total = 0.0;
    for (int j = 0; j < k; ++j) {
        int cnt = 0;
        for (int h = 0; h < H; ++h)
            if (label_of[h] == j) ++cnt;
        if (cnt == 0) continue;
        for (int f = 0; f < F; ++f) {
            double acc = 0.0;
            for (int h = 0; h < H; ++h)
                if (label_of[h] == j) acc = acc + (double)X[(int64_t)h * F + f];
            mean[f] = acc / (double)cnt;
        }
        for (int h = 0; h < H; ++h)
            if (label_of[h] == j) total += sqdist(X + (int64_t)h * F, mean, F);
    }
    return total;
}

int chai_oracle_cluster_error(const float *feat, const int32_t *head_to_cluster, int B, int H, int F, int k,
                              double *sse)
{
    if (!feat || !head_to_cluster || !sse) return 1;
    if (B < 0 || H < 1 || F < 1 || k < 1 || k > H) return 2;
    double *mean = (double *)malloc(sizeof(double) * (size_t)F);
    for (int b = 0; b < B; ++b)
        sse[b] = partition_error(feat + (int64_t)b * H * F, head_to_cluster + (int64_t)b * H, H, F, k, mean);
    free(mean);
    return 0;
}

/*
 * Alternative choice of the head that stands for a cluster (the paper speaks
 * of one representative head per cluster without fixing which one): the
 * member whose features lie closest (squared Euclidean distance) to the mean
 * of the cluster's members; equal distances -> the lowest head index.
 * Empty cluster slots get -1.  rep_out [B,k].
 */
int chai_oracle_closest_representatives(const float *feat, const int32_t *head_to_cluster, int B, int H, int F,
                                        int k, int32_t *rep_out)
{
    if (!feat || !head_to_cluster || !rep_out) return 1;
    if (B < 0 || H < 1 || F < 1 || k < 1 || k > H) return 2;
    double *mean = (double *)malloc(sizeof(double) * (size_t)F);
    for (int b = 0; b < B; ++b) {
        const float *X = feat + (int64_t)b * H * F;
        const int32_t *lab = head_to_cluster + (int64_t)b * H;
        for (int j = 0; j < k; ++j) {
            int cnt = 0;
            for (int h = 0; h < H; ++h)
                if (lab[h] == j) ++cnt;
            int best = -1;
            double best_d = 0.0;
            if (cnt > 0) {
                for (int f = 0; f < F; ++f) {
                    double acc = 0.0;
                    for (int h = 0; h < H; ++h)
                        if (lab[h] == j) acc = acc + (double)X[(int64_t)h * F + f];
                    mean[f] = acc / (double)cnt;
                }
                for (int h = 0; h < H; ++h) {
                    if (lab[h] != j) continue;
                    double dist = sqdist(X + (int64_t)h * F, mean, F);
                    if (best < 0 || dist < best_d) {
                        best = h;
                        best_d = dist;
                    }
                }
            }
            rep_out[(int64_t)b * k + j] = best;
        }
    }
    free(mean);
    return 0;
}

/*
 * Number of clusters from the error curve (Section 3.2: the count is taken
 * where the error curve flattens; the paper reads the elbow plot by eye).  Reading used here: with err[i] the mean clustering error at ks[i]
 * (ks ascending), pick the smallest ks[i] whose error has come down to
 * within a fraction `tol` of the whole drop,
 *     err[i] - err[n-1] <= tol * (err[0] - err[n-1]).
 */
int chai_oracle_pick_cluster_count(const double *err, const int32_t *ks, int n, double tol, int32_t *k_out)
{
    if (!err || !ks || !k_out) return 1;
    if (n < 1 || !(tol >= 0.0)) return 2;
    double drop = err[0] - err[n - 1];
    for (int i = 0; i < n; ++i)
        if (err[i] - err[n - 1] <= tol * drop) { *k_out = ks[i]; return 0; }
    *k_out = ks[n - 1];
    return 0;
}

/*
 * Cluster membership by K-Means (Section 3.5: K-Means on the observed
 * activations once five tokens are processed; Section 3.2: the clustering
 * error is the sum of squared distances to the closest centre, i.e. the
 * Euclidean k-means objective).  The paper names the algorithm only; the
 * rules below complete it and are what the device kernel must reproduce
 * bit for bit.  One independent problem per batch row b (membership is
 * decided per request):
 *
 *  1. centre j starts at the feature vector of head init_heads[b][j].
 *  2. assignment pass: every head, in index order, goes to the centre with
 *     the smallest squared distance (ties: lowest j).
 *  3. repair: for each centre j, ascending, that received no head, take the
 *     head with the largest distance to its own centre among heads whose
 *     cluster holds at least two heads (ties: lowest head; a largest
 *     distance of zero leaves j empty) and move it to j.  (The "at least two
 *     heads" condition keeps a repair from emptying another cluster behind
 *     the scan: a lone head can be the farthest on the board, because its
 *     distance is measured to the centre of the previous pass; hand-worked
 *     examples of exactly that pin the condition.)
 *  4. if this is not the first pass and no head changed cluster: stop.
 *  5. update: each non-empty centre becomes the mean of its heads (summed
 *     in head order, then divided by the count); an empty centre stays.
 *  6. at most max_iter passes; iters[b] = passes run.
 *  7. canonical labels: non-empty clusters are numbered by their lowest
 *     member head; that head is the representative.  rep_heads[b][j] = -1
 *     for j >= n_clusters[b].
 *
 * feat [B,H,F] fp32; init_heads [B,k] distinct, in [0,H); outputs
 * head_to_cluster [B,H], rep_heads [B,k], n_clusters [B], iters [B]
 * (nullable), sse [B] (nullable; the clustering error of the returned
 * partition measured to the means of its clusters).
 */
int chai_oracle_kmeans(const float *feat, int B, int H, int F, int k, const int32_t *init_heads,
                       int max_iter, int32_t *head_to_cluster, int32_t *rep_heads,
                       int32_t *n_clusters, int32_t *iters, double *sse)
{
    if (!feat || !init_heads || !head_to_cluster || !rep_heads || !n_clusters) return 1;
    if (B < 0 || H < 1 || F < 1 || k < 1 || k > H || max_iter < 1) return 2;
    for (int64_t i = 0; i < (int64_t)B * k; ++i)
        if (init_heads[i] < 0 || init_heads[i] >= H) return 2;

    double *centre = (double *)malloc(sizeof(double) * (size_t)k * F);
    double *dmin = (double *)malloc(sizeof(double) * (size_t)H);
    int *assign = (int *)malloc(sizeof(int) * (size_t)H);
    int *prev = (int *)malloc(sizeof(int) * (size_t)H);
    int *count = (int *)malloc(sizeof(int) * (size_t)k);
    int *label = (int *)malloc(sizeof(int) * (size_t)k);

    for (int b = 0; b < B; ++b) {
        const float *X = feat + (int64_t)b * H * F;
        for (int j = 0; j < k; ++j)
            for (int f = 0; f < F; ++f)
                centre[j * F + f] = (double)X[(int64_t)init_heads[(int64_t)b * k + j] * F + f];
        for (int h = 0; h < H; ++h) prev[h] = -1;

        int it = 0;
        for (;;) {
            ++it;
            /* 2. assignment */
            for (int j = 0; j < k; ++j) count[j] = 0;
            for (int h = 0; h < H; ++h) {
                int best = 0;
                double bd = sqdist(X + (int64_t)h * F, centre, F);
                for (int j = 1; j < k; ++j) {
                    double dj = sqdist(X + (int64_t)h * F, centre + j * F, F);
                    if (dj < bd) { bd = dj; best = j; }
                }
                assign[h] = best;
                dmin[h] = bd;
                count[best]++;
            }
            /* 3. repair empty centres */
            for (int j = 0; j < k; ++j) {
                if (count[j] != 0) continue;
                int pick = -1;
                double far = 0.0;
                for (int h = 0; h < H; ++h)
                    if (count[assign[h]] >= 2 && dmin[h] > far) { far = dmin[h]; pick = h; }
                if (pick < 0) continue;
                count[assign[pick]]--;
                assign[pick] = j;
                count[j] = 1;
                dmin[pick] = 0.0;
            }
            /* 4. converged? */
            int changed = 0;
            for (int h = 0; h < H; ++h)
                if (assign[h] != prev[h]) changed = 1;
            for (int h = 0; h < H; ++h) prev[h] = assign[h];
            if (!changed || it >= max_iter) break;
            /* 5. update */
            for (int j = 0; j < k; ++j) {
                if (count[j] == 0) continue;
                for (int f = 0; f < F; ++f) {
                    double acc = 0.0;
                    for (int h = 0; h < H; ++h)
                        if (assign[h] == j) acc = acc + (double)X[(int64_t)h * F + f];
                    centre[j * F + f] = acc / (double)count[j];
                }
            }
        }

        /* 7. canonical labels */
        for (int j = 0; j < k; ++j) { label[j] = -1; rep_heads[(int64_t)b * k + j] = -1; }
        int n = 0;
        for (int h = 0; h < H; ++h) {
            int a = assign[h];
            if (label[a] < 0) {
                label[a] = n;
                rep_heads[(int64_t)b * k + n] = h;
                ++n;
            }
            head_to_cluster[(int64_t)b * H + h] = label[a];
        }
        n_clusters[b] = n;
        if (iters) iters[b] = it;

        if (sse) sse[b] = partition_error(X, head_to_cluster + (int64_t)b * H, H, F, k, centre);
    }
    free(centre); free(dmin); free(assign); free(prev); free(count); free(label);
    return 0;
}

/*
 * ---------------------------------------------------------------------
 * Quantised key/value caches (Section 2, related work: quantisation of
 * the K,V cache is orthogonal to clustering heads and can be combined with
 * it).  The paper gives no format; the reading used here:
 *
 *  - elements are 8-bit floating point E4M3 as defined by the OCP 8-bit
 *    floating point specification: 1 sign, 4 exponent bits (bias 7),
 *    3 mantissa bits, subnormals, no infinities, S.1111.111 = NaN, largest
 *    finite magnitude 448;
 *  - one fp32 scale per cached row (one token of one key or value stream):
 *    amax = max_i |x_i|, scale = amax / 448, code_i = nearest E4M3 value
 *    (ties to even) of x_i * (448 / amax), computed in fp32 -- the
 *    precision the device uses, because these steps decide integer codes;
 *    an all-zero row has scale 0 and codes 0;
 *  - the dequantised element is decode(code_i) * scale, and attention over a
 *    quantised cache is, by definition, the plain attention over the
 *    dequantised cache ("dequantise, then attend").
 * ---------------------------------------------------------------------
 */

/* value of one E4M3 code (NaN for 0x7f / 0xff) */
double chai_oracle_e4m3_decode(int code)
{
    int sign = (code >> 7) & 1, e = (code >> 3) & 15, m = code & 7;
    double mag;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) mag = ldexp((double)m / 8.0, 1 - 7);          /* subnormal: 0.mmm * 2^(1-bias) */
    else mag = ldexp(1.0 + (double)m / 8.0, e - 7);          /* normal: 1.mmm * 2^(e-bias)    */
    return sign ? -mag : mag;
}

/*
 * nearest E4M3 code of a finite y, ties to the even mantissa, magnitudes
 * above 448 saturate to 448 (NaN gives the NaN code)
 */
int chai_oracle_e4m3_encode(float y)
{
    if (isnan(y)) return 0x7f;
    int sign = signbit(y) ? 0x80 : 0;
    double a = fabs((double)y);
    if (a >= 448.0) return sign | 0x7e;
    if (a == 0.0) return sign;
    int ex;
    frexp(a, &ex);                       /* a = f * 2^ex, 0.5 <= f < 1  ->  floor(log2 a) = ex - 1 */
    int e = ex - 1;
    if (e < -6) e = -6;                  /* below the smallest normal the spacing stays 2^-9 */
    double step = ldexp(1.0, e - 3);     /* spacing of representable values around a */
    double r = nearbyint(a / step);      /* default rounding mode: to nearest, ties to even */
    double val = r * step;               /* may have moved up into the next binade: still representable */
    if (val == 0.0) return sign;
    int code;
    if (val < ldexp(1.0, -6)) {
        code = (int)(val / ldexp(1.0, -9));              /* subnormal: mantissa counts steps of 2^-9 */
    } else {
        frexp(val, &ex);
        int E = ex - 1 + 7;
        int M = (int)(val / ldexp(1.0, ex - 1) * 8.0) - 8;
        code = (E << 3) | M;
    }
    return sign | code;
}

/*
 * Quantise n_rows rows of d elements (dtype fp32 or bf16) to E4M3 codes with
 * one fp32 scale per row, by the rule in the header above.  The three fp32
 * operations (amax / 448, 448 / amax, x * that) are single IEEE operations.
 */
int chai_oracle_quantize_rows(const void *x, int64_t n_rows, int d, int dtype, uint8_t *codes, float *scales)
{
    if (!x || !codes || !scales) return 1;
    if (n_rows < 0 || d < 1) return 2;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return 3;
    for (int64_t r = 0; r < n_rows; ++r) {
        float amax = 0.0f;
        for (int i = 0; i < d; ++i) {
            float v = fabsf((float)load_elem(x, r * d + i, dtype));
            if (v > amax) amax = v;
        }
        if (amax == 0.0f) {
            scales[r] = 0.0f;
            for (int i = 0; i < d; ++i) codes[r * d + i] = 0;
            continue;
        }
        float scale = amax / 448.0f;
        float inv = 448.0f / amax;
        scales[r] = scale;
        for (int i = 0; i < d; ++i) {
            float yc = (float)load_elem(x, r * d + i, dtype) * inv;
            if (yc > 448.0f) yc = 448.0f;
            if (yc < -448.0f) yc = -448.0f;
            codes[r * d + i] = (uint8_t)chai_oracle_e4m3_encode(yc);
        }
    }
    return 0;
}

/* dequantised rows in double: decode(code) * scale, exactly */
int chai_oracle_dequantize_rows(const uint8_t *codes, const float *scales, int64_t n_rows, int d, double *x)
{
    if (!codes || !scales || !x) return 1;
    if (n_rows < 0 || d < 1) return 2;
    for (int64_t r = 0; r < n_rows; ++r)
        for (int i = 0; i < d; ++i)
            x[r * d + i] = chai_oracle_e4m3_decode(codes[r * d + i]) * (double)scales[r];
    return 0;
}

/*
 * One decode step of clustered-head attention over quantised caches: the
 * definition of chai_oracle_clustered_decode with every key and value
 * element replaced by its dequantised value decode(code) * scale_of_its_row
 * (dequantise, then attend).  k8, v8 [B,H,T_cap,d] codes of the FULL caches,
 * kscale, vscale [B,H,T_cap]; q [B,H,d] in `dtype`.
 */
int chai_oracle_clustered_decode_q8(const void *q, const uint8_t *k8, const float *kscale, const uint8_t *v8,
                                    const float *vscale, const int32_t *head_to_cluster,
                                    const int32_t *rep_heads, int B, int H, int k, int T, int T_cap, int d,
                                    int dtype, double scale, double *out, double *probs)
{
    if (!q || !k8 || !kscale || !v8 || !vscale || !head_to_cluster || !rep_heads || !out) return 1;
    if (B < 0 || H < 1 || k < 1 || k > H || T < 1 || T > T_cap || d < 1) return 2;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return 3;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            int c = head_to_cluster[(int64_t)b * H + h];
            if (c < 0 || c >= k) return 2;
            int r = rep_heads[(int64_t)b * k + c];
            if (r < 0 || r >= H) return 2;
        }
    double *p_all = (double *)malloc(sizeof(double) * (size_t)B * k * T + 8);
    if (!p_all) return 4;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        for (int j = 0; j < k; ++j) {
            double *p = p_all + ((int64_t)b * k + j) * T;
            int r = rep_heads[(int64_t)b * k + j];
            if (r < 0 || r >= H) {
                for (int t = 0; t < T; ++t) p[t] = NAN;
                continue;
            }
            double *s = (double *)malloc(sizeof(double) * (size_t)T);
            int64_t qoff = ((int64_t)b * H + r) * d;
            int64_t row0 = ((int64_t)b * H + r) * (int64_t)T_cap;
            for (int t = 0; t < T; ++t) {
                double acc = 0.0;
                for (int i = 0; i < d; ++i) {
                    double kd = chai_oracle_e4m3_decode(k8[(row0 + t) * d + i]) * (double)kscale[row0 + t];
                    acc += load_elem(q, qoff + i, dtype) * kd;
                }
                s[t] = scale * acc;
            }
            softmax_row(s, T, p);
            free(s);
        }
    }
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            int c = head_to_cluster[(int64_t)b * H + h];
            const double *p = p_all + ((int64_t)b * k + c) * T;
            int64_t row0 = ((int64_t)b * H + h) * (int64_t)T_cap;
            for (int i = 0; i < d; ++i) {
                double acc = 0.0;
                for (int t = 0; t < T; ++t) {
                    double vd = chai_oracle_e4m3_decode(v8[(row0 + t) * d + i]) * (double)vscale[row0 + t];
                    acc += p[t] * vd;
                }
                out[((int64_t)b * H + h) * d + i] = acc;
            }
        }
    }
    if (probs) memcpy(probs, p_all, sizeof(double) * (size_t)B * k * T);
    free(p_all);
    return 0;
}

/*
 * Query / key projections of the representatives only (Fig. 3 and Section
 * 3.5: in clustered attention the query and key vectors of the other heads
 * are not needed, so their share of the projection is not computed; the
 * keys go straight into the pruned cache).  For every batch row b, cluster
 * slot j with representative r = rep_heads[b][j] >= 0, token i < Tn and
 * coordinate c < d:
 *     q_rep[b][j][i][c] = sum_e x[b][i][e] * w_q[r*d + c][e]
 *     k_rep[b][j][i][c] = sum_e x[b][i][e] * w_k[r*d + c][e]
 * x [B,Tn,D]; w_q, w_k [H*d, D] (one row per output feature, the layout of
 * a linear layer's weight); outputs [B,k,Tn,d] in double, unrounded (slots
 * with rep_heads = -1 are filled with NaN).  No bias (LLaMa has none; a
 * model with one adds it afterwards).
 */
int chai_oracle_project_qk(const void *x, const void *w_q, const void *w_k, const int32_t *rep_heads,
                           int B, int H, int k, int Tn, int D, int d, int dtype,
                           double *q_rep, double *k_rep)
{
    if (!x || !w_q || !w_k || !rep_heads || !q_rep || !k_rep) return 1;
    if (B < 0 || H < 1 || k < 1 || k > H || Tn < 1 || D < 1 || d < 1) return 2;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return 3;
    for (int64_t i = 0; i < (int64_t)B * k; ++i)
        if (rep_heads[i] >= H) return 2;

#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        for (int j = 0; j < k; ++j) {
            int r = rep_heads[(int64_t)b * k + j];
            for (int i = 0; i < Tn; ++i) {
                int64_t xoff = ((int64_t)b * Tn + i) * D;
                int64_t ooff = (((int64_t)b * k + j) * Tn + i) * d;
                for (int c = 0; c < d; ++c) {
                    if (r < 0) {
                        q_rep[ooff + c] = NAN;
                        k_rep[ooff + c] = NAN;
                        continue;
                    }
                    int64_t woff = ((int64_t)r * d + c) * D;
                    double aq = 0.0, ak = 0.0;
                    for (int e = 0; e < D; ++e) {
                        double xe = load_elem(x, xoff + e, dtype);
                        aq += xe * load_elem(w_q, woff + e, dtype);
                        ak += xe * load_elem(w_k, woff + e, dtype);
                    }
                    q_rep[ooff + c] = aq;
                    k_rep[ooff + c] = ak;
                }
            }
        }
    }
    return 0;
}

/*
 * K-cache pruning (Section 3.5: once membership is fixed the keys of the
 * pruned heads are removed; values are all kept).  The compact cache holds
 * one key stream per cluster, the representative's:
 *     k_compact[b][j][t][:] = k_full[b][rep_heads[b][j]][t][:],  t < T.
 * Slots with rep_heads = -1 and rows t >= T are left untouched.
 * src_rows (nullable) [B,k,T] int64 receives the flat source row index
 * (b*H + rep)*T_cap + t of every copied row, or -1 for unused slots.
 */
int chai_oracle_compact_kcache(const void *k_full, const int32_t *rep_heads, void *k_compact,
                               int B, int H, int k, int T, int T_cap, int Tc_cap, int d, int dtype,
                               int64_t *src_rows)
{
    if (!k_full || !rep_heads || !k_compact) return 1;
    if (B < 0 || H < 1 || k < 1 || k > H || T < 0 || T > T_cap || T > Tc_cap || d < 1) return 2;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return 3;
    size_t row = (size_t)d * elem_size(dtype);
    for (int b = 0; b < B; ++b)
        for (int j = 0; j < k; ++j) {
            int r = rep_heads[(int64_t)b * k + j];
            for (int t = 0; t < T; ++t) {
                int64_t dst = ((int64_t)b * k + j) * Tc_cap + t;
                if (r < 0) {
                    if (src_rows) src_rows[((int64_t)b * k + j) * T + t] = -1;
                    continue;
                }
                if (r >= H) return 2;
                int64_t src = ((int64_t)b * H + r) * T_cap + t;
                memcpy((char *)k_compact + (size_t)dst * row, (const char *)k_full + (size_t)src * row, row);
                if (src_rows) src_rows[((int64_t)b * k + j) * T + t] = src;
            }
        }
    return 0;
}

/*
 * Cache growth by one token at position pos (Section 2: keys and values of
 * prior tokens are cached; Section 3.5: pruned heads' keys are not stored):
 *     k_compact[b][j][pos][:] = k_new[b][rep_heads[b][j]][:]
 *     v_cache[b][h][pos][:]   = v_new[b][h][:]
 */
int chai_oracle_append_kv(const void *k_new, const void *v_new, const int32_t *rep_heads,
                          void *k_compact, void *v_cache, int B, int H, int k, int pos,
                          int Tc_cap, int T_cap, int d, int dtype)
{
    if (!k_new || !v_new || !rep_heads || !k_compact || !v_cache) return 1;
    if (B < 0 || H < 1 || k < 1 || k > H || pos < 0 || pos >= T_cap || pos >= Tc_cap || d < 1) return 2;
    if (dtype != ORC_F32 && dtype != ORC_BF16) return 3;
    size_t row = (size_t)d * elem_size(dtype);
    for (int b = 0; b < B; ++b) {
        for (int j = 0; j < k; ++j) {
            int r = rep_heads[(int64_t)b * k + j];
            if (r < 0) continue;
            if (r >= H) return 2;
            memcpy((char *)k_compact + (((size_t)b * k + j) * Tc_cap + pos) * row,
                   (const char *)k_new + ((size_t)b * H + r) * row, row);
        }
        for (int h = 0; h < H; ++h)
            memcpy((char *)v_cache + (((size_t)b * H + h) * T_cap + pos) * row,
                   (const char *)v_new + ((size_t)b * H + h) * row, row);
    }
    return 0;
}
