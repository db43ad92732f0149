/*
 * chai.h -- C ABI of the MI355X (gfx950) clustered-head decode attention library.
 *
 * CHAI (Clustered Head Attention): per layer and per request the attention
 * heads are grouped into clusters by k-means over the attention scores they
 * produce on the first few tokens; afterwards only one representative head
 * per cluster computes softmax(q K^T), the keys of the other heads are
 * dropped from the cache, and every head applies its cluster's probabilities
 * to its own values.
 *
 * Conventions for every entry point
 *  - All tensor pointers are DEVICE pointers owned by the caller.  The
 *    library allocates nothing, frees nothing and keeps no pointer after the
 *    call returns.  Its only process-wide state is bookkeeping that does not
 *    affect results: per-device "attribute already set" flags of the kernels
 *    with large LDS, and the fixed scratch array of
 *    chai_decode_attention_static with its per-device address table.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue work on it: no synchronisation, no host read-back.
 *    Cluster maps produced by one call are consumed by the next on the device.
 *  - Tensors are dense, row-major, last index fastest, in the shapes written
 *    next to each argument.  `dtype` (CHAI_F32 or CHAI_BF16) is the storage
 *    type of q, K and V; bf16 is the upper half of an IEEE fp32 word.  All
 *    arithmetic accumulates in fp32 (fp64 in chai_assign_clusters and
 *    chai_score_features); outputs are fp32.
 *  - q/K/V base pointers must be 16-byte aligned; d must be 128.
 *  - Arguments are checked on the host before anything is launched; on an
 *    argument error nothing is enqueued and outputs are untouched.  Contents
 *    of device maps (cluster ids, representative ids) cannot be checked on
 *    the host; kernels clamp them into range instead of faulting, and the
 *    result for an out-of-range map entry is unspecified.
 *  - One call handles one layer.  B = batch rows (independent requests),
 *    H = heads, k = cluster slots of this layer, T = cached tokens attended
 *    to (the current token included), d = head dimension.
 *  - Return value: CHAI_OK or one of the error codes below.
 */
#ifndef CHAI_H
#define CHAI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    CHAI_OK = 0,
    CHAI_ERR_NULL = 1,        /* a required pointer is NULL                          */
    CHAI_ERR_SHAPE = 2,       /* a size is out of range or inconsistent              */
    CHAI_ERR_DTYPE = 3,       /* dtype is neither CHAI_F32 nor CHAI_BF16             */
    CHAI_ERR_WORKSPACE = 4,   /* workspace NULL, misaligned or smaller than required */
    CHAI_ERR_UNSUPPORTED = 5, /* valid request this build does not implement (d != 128, ...) */
    CHAI_ERR_HIP = 6,         /* the HIP runtime reported an error at launch         */
    CHAI_ERR_ALIGN = 7,       /* a tensor pointer is not 16-byte aligned             */
    CHAI_ERR_STATIC_LIMIT = 8 /* chai_decode_attention_static: sizes need more than CHAI_STATIC_SCRATCH_BYTES */
};

/* Size of the scratch array built into the library for chai_decode_attention_static. */
#define CHAI_STATIC_SCRATCH_BYTES (32u << 20)

enum { CHAI_F32 = 0, CHAI_BF16 = 1 };

/* Library version, major * 100 + minor. */
int chai_version(void);

/* Static string for a status code (never NULL). */
const char *chai_status_string(int status);

/*
 * Clustering features (Section 3.3: the attention scores of the first tokens
 * of a request predict cluster membership; Section 3.1: the compared
 * quantity is f(Q,K) = softmax(Q K^T); Section 2: decoder-only, so causal).
 *
 * For every (b,h): the n_tok x n_tok causal attention matrix of the first
 * n_tok positions, A[i][j] = softmax_j(scale * q_i . k_j) for j <= i and 0
 * for j > i, flattened row-major into feat[b][h][i*n_tok + j] (fp32).
 *
 *   q5    [B,H,*,d]  element (b,h,i,c) at (b*H+h)*q_head_stride + i*d + c
 *   k5    [B,H,*,d]  element (b,h,j,c) at (b*H+h)*k_head_stride + j*d + c
 *                    (strides in elements, >= n_tok*d, multiples of 8; lets
 *                    the keys be read in place from a cache with stride
 *                    T_cap*d)
 *   feat  [B,H,n_tok*n_tok] fp32, written
 * 1 <= n_tok <= 8.  Scores and the softmax are evaluated in fp64 and rounded
 * once to fp32.
 */
int chai_score_features(const void *q5, const void *k5, int B, int H, int n_tok, int d, int dtype,
                        int64_t q_head_stride, int64_t k_head_stride, float scale, float *feat,
                        void *stream);

/*
 * Cluster membership by K-Means (Section 3.5: K-Means on the observed
 * activations once five tokens are processed, then fixed for the request;
 * Section 3.2: clustering error = sum of squared distances to the closest
 * centre).  One independent problem per batch row.  Lloyd iterations in
 * fp64 with separately rounded multiplies and adds:
 *   1. centre j starts at feat[b][init_heads[b][j]];
 *   2. every head goes to the centre at the smallest squared Euclidean
 *      distance (ties: lowest j);
 *   3. each centre left without heads, in ascending j, takes the head that is
 *      farthest from its own centre among heads of clusters holding at least
 *      two heads (ties: lowest head; if that distance is 0 the centre stays
 *      empty);
 *   4. stop if no head changed cluster (never after the first pass);
 *   5. non-empty centres move to the mean of their heads (summed in head
 *      order, divided by the count);
 *   6. at most max_iter passes;
 *   7. clusters are numbered by their lowest member head, which is the
 *      cluster's representative.
 *
 *   feat            [B,H,F] fp32
 *   init_heads      [B,k] int32, distinct head ids in [0,H) (the caller's
 *                   seeded choice; the library draws no random numbers)
 *   head_to_cluster [B,H] int32, written: canonical cluster id of each head
 *   rep_heads       [B,k] int32, written: representative of cluster j, -1 for
 *                   j >= n_clusters[b]
 *   n_clusters      [B] int32, written: number of non-empty clusters
 *   iters           [B] int32, written if not NULL: assignment passes run
 * Limits: 1 <= k <= H <= 256, 1 <= F <= 64, k*F <= 7168, 1 <= max_iter
 * (beyond them: CHAI_ERR_UNSUPPORTED).  The outputs are bit-identical to the
 * sequential algorithm above for the same feat bits.
 */
int chai_assign_clusters(const float *feat, int B, int H, int F, int k, const int32_t *init_heads,
                         int max_iter, int32_t *head_to_cluster, int32_t *rep_heads,
                         int32_t *n_clusters, int32_t *iters, void *stream);

/*
 * Offline choice of the number of clusters (Section 3.2: clustering error =
 * sum of squared distances to the closest centre, plotted against the number
 * of clusters; the count is taken where the error plateaus).
 *
 * chai_cluster_error: for each batch row (one sample) the error of the given
 * partition, every non-empty cluster's centre at the mean of its members;
 * fp64, clusters in label order, heads ascending, one running sum (bit-
 * identical to the sequential evaluation).
 *   feat [B,H,F] fp32; head_to_cluster [B,H] int32 with labels in [0,k) (any
 *   labelling, labels may be unused); sse [B] fp64 on the device, written.
 *   Limits as for chai_assign_clusters.
 * A sweep is the caller's loop: for each candidate k, chai_assign_clusters
 * then chai_cluster_error over the samples.
 *
 * chai_pick_cluster_count (HOST pointers, runs on the host, no GPU work):
 * mean_error[i] is the error averaged over the samples at ks[i], ks strictly
 * ascending.  The paper reads the elbow by eye; the rule here returns the
 * smallest ks[i] with  mean_error[i] - mean_error[n-1] <= tol * (mean_error[0]
 * - mean_error[n-1]),  i.e. whose error has come within a fraction tol of the
 * whole drop.
 */
int chai_cluster_error(const float *feat, const int32_t *head_to_cluster, int B, int H, int F, int k,
                       double *sse, void *stream);
int chai_pick_cluster_count(const double *mean_error, const int32_t *ks, int n, double tol, int32_t *k_out);

/*
 * Variant of the choice of representative.  Sections 3.4-3.5 and Fig. 3 let
 * one head stand for its cluster without fixing which member; the default
 * everywhere in this library is the lowest-numbered member (what
 * chai_assign_clusters returns).  This call returns instead, for every
 * cluster of a given partition, the member whose features lie nearest
 * (squared Euclidean distance, fp64) to the mean of the cluster's members;
 * equal distances -> the lowest head; unused labels -> -1.  Bit-identical to
 * the sequential evaluation (means and distances as in chai_cluster_error).
 *   feat [B,H,F] fp32; head_to_cluster [B,H] int32, labels in [0,k);
 *   rep_heads [B,k] int32, written.  Limits as for chai_assign_clusters.
 * The maps it returns can be passed to every other entry point (they accept
 * any member as representative).
 */
int chai_closest_representatives(const float *feat, const int32_t *head_to_cluster, int B, int H, int F, int k,
                                 int32_t *rep_heads, void *stream);

/*
 * K-cache pruning (Section 3.5: once membership is fixed, the keys of the
 * pruned heads are removed; Section 4.3 / Fig. 3: all values are kept).
 *   k_compact[b][j][t][:] = k_full[b][rep_heads[b][j]][t][:]   for t < T.
 * Cluster slots with rep_heads[b][j] < 0 and rows t >= T are not written.
 *
 *   k_full    [B,H,T_cap,d]   read
 *   rep_heads [B,k] int32     read on the device
 *   k_compact [B,k,Tc_cap,d]  written; must not overlap k_full
 * 0 <= T <= min(T_cap, Tc_cap), 1 <= k <= H.
 */
int chai_compact_kcache(const void *k_full, const int32_t *rep_heads, void *k_compact, int B, int H,
                        int k, int T, int T_cap, int Tc_cap, int d, int dtype, void *stream);

/*
 * Cache growth by one token (Section 2: keys and values of prior tokens are
 * cached; Section 3.5: keys of pruned heads are not stored).
 *   k_compact[b][j][pos][:] = k_new[b][rep_heads[b][j]][:]   (rep >= 0)
 *   v_cache[b][h][pos][:]   = v_new[b][h][:]
 *
 *   k_new, v_new [B,H,d]; k_compact [B,k,Tc_cap,d]; v_cache [B,H,T_cap,d]
 * 0 <= pos < min(T_cap, Tc_cap).
 */
int chai_append_kv(const void *k_new, const void *v_new, const int32_t *rep_heads, void *k_compact,
                   void *v_cache, int B, int H, int k, int pos, int Tc_cap, int T_cap, int d,
                   int dtype, void *stream);

/*
 * Bytes of scratch chai_decode_attention / chai_dense_decode_attention need
 * for these sizes (0 on invalid sizes).  For the dense call pass k = H.  The
 * value never decreases when B, H, k or T grows, so a workspace sized for the
 * cache capacity serves every shorter context.
 */
size_t chai_decode_workspace_bytes(int B, int H, int k, int T, int d, int dtype);

/*
 * One decode step of clustered-head attention for one layer (Sections 3.4
 * and 3.5 with the attention definition of Section 2):
 *   for every cluster j of row b with representative r = rep_heads[b][j] >= 0
 *       s[t]   = scale * sum_i q[b][r][i] * k_compact[b][j][t][i]    t < T
 *       p_j[t] = exp(s[t] - max s) / sum_t exp(s[t] - max s)
 *   for every head h, c = head_to_cluster[b][h]
 *       out[b][h][:] = sum_t p_c[t] * v_cache[b][h][t][:]
 * Long contexts are processed in token chunks whose partial softmax
 * statistics and partial outputs are merged exactly; the result is the
 * one-pass definition above up to fp32 rounding order.
 *
 *   q               [B,H,d]           only representatives' rows are read
 *   k_compact       [B,k,Tc_cap,d]
 *   v_cache         [B,H,T_cap,d]
 *   head_to_cluster [B,H] int32, values in [0,k), pointing at used slots
 *   rep_heads       [B,k] int32, head ids in [0,H) or -1 for unused slots
 *   out             [B,H,d] fp32, written
 *   probs_out       NULL, or [B,k,T] fp32: receives p_j (unused slots are
 *                   not written); for tests and inspection
 *   workspace       at least chai_decode_workspace_bytes(...) bytes, 256-byte
 *                   aligned; contents need not be initialised and are
 *                   undefined afterwards.  Two calls that run concurrently
 *                   need separate workspaces.
 * 1 <= T <= min(T_cap, Tc_cap), 1 <= k <= H, B >= 0 (B = 0 is a no-op).
 */
int chai_decode_attention(const void *q, const void *k_compact, const void *v_cache,
                          const int32_t *head_to_cluster, const int32_t *rep_heads, int B, int H,
                          int k, int T, int Tc_cap, int T_cap, int d, int dtype, float scale,
                          float *out, float *probs_out, void *workspace, size_t workspace_bytes,
                          void *stream);

/*
 * chai_decode_attention for callers that cannot allocate device memory or
 * carry a workspace around: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * same results as chai_decode_attention, minus the workspace: scores, chunk
 * statistics and partial rows live in a fixed array of
 * CHAI_STATIC_SCRATCH_BYTES (32 MiB) that is part of the library's code
 * object; every GPU the library runs on holds its own copy until the process
 * ends.  The call allocates and frees nothing (its first call on a device
 * looks up the array's address once).
 *   - Sizes whose chai_decode_workspace_bytes(B, H, k, T, d, dtype) exceeds
 *     CHAI_STATIC_SCRATCH_BYTES are refused with CHAI_ERR_STATIC_LIMIT
 *     before anything is launched (use chai_decode_attention then).
 *   - Nothing in the array has to start at zero: every location a call reads
 *     it has written first, so stale contents of an earlier, larger call are
 *     harmless.
 *   - All calls on one GPU share that GPU's array: calls that overlap in
 *     time on one GPU (two streams, two threads) race.  Serialise them, or
 *     give the overlapping ones chai_decode_attention with workspaces.
 */
int chai_decode_attention_static(const void *q, const void *k_compact, const void *v_cache,
                                 const int32_t *head_to_cluster, const int32_t *rep_heads, int B,
                                 int H, int k, int T, int Tc_cap, int T_cap, int d, int dtype,
                                 float scale, float *out, float *probs_out, void *stream);

/*
 * The two phases of chai_decode_attention as separate calls (same arguments,
 * same workspace, same results): chai_decode_scores computes the scaled
 * scores of every cluster and their per-chunk softmax statistics into the
 * workspace (scores of Section 2, one per cluster as in Section 3.4);
 * chai_decode_values turns them into probabilities and applies them to every
 * head's own values (Section 3.5, Fig. 3).  chai_decode_values must follow
 * chai_decode_scores on the same stream with the same sizes and workspace.
 * Meant for callers that time or overlap the phases; chai_decode_attention
 * is exactly the two in sequence.
 */
int chai_decode_scores(const void *q, const void *k_compact, const int32_t *rep_heads, int B, int H, int k,
                       int T, int Tc_cap, int d, int dtype, float scale, void *workspace,
                       size_t workspace_bytes, void *stream);
int chai_decode_values(const void *v_cache, const int32_t *head_to_cluster, const int32_t *rep_heads, int B,
                       int H, int k, int T, int T_cap, int d, int dtype, float *out, float *probs_out,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * One decode step with the cache growth folded in (Section 2: the keys and
 * values of the token being decoded join the cache, then it attends over
 * all T positions; Section 3.5: only the representatives' keys are kept).
 * Same result as chai_append_kv at position T-1 followed by
 * chai_decode_attention over T positions, without the extra launch: the
 * kernels that stream the caches take row T-1 from k_new / v_new and write
 * it to the caches themselves.
 *
 *   k_new, v_new [B,H,d]   the new token's key and value rows (keys of
 *                          representatives are read, values of all heads)
 *   k_compact, v_cache     read for positions 0 .. T-2, row T-1 written
 *   T                      context length INCLUDING the new token, >= 1
 * Other arguments, limits and errors as chai_decode_attention (no
 * probs_out).  The accumulation order of the new row differs from the
 * two-call sequence, so outputs agree to rounding, not bit for bit.
 */
int chai_decode_step(const void *q, const void *k_new, const void *v_new, void *k_compact, void *v_cache,
                     const int32_t *head_to_cluster, const int32_t *rep_heads, int B, int H, int k, int T,
                     int Tc_cap, int T_cap, int d, int dtype, float scale, float *out, void *workspace,
                     size_t workspace_bytes, void *stream);

/*
 * For callers that profile the two kernels: the same calls with two more
 * arguments, hipEvent_t handles passed as void* that the caller created with
 * timing enabled (either may be NULL).  The runtime stamps start_event when
 * the phase's kernel begins executing and stop_event when it has finished, so
 * hipEventElapsedTime(start, stop) is the duration of the kernel itself,
 * without launch gaps.  (When the value phase runs a combine kernel after the
 * value kernel, the events cover the value kernel only.)
 */
int chai_decode_scores_timed(const void *q, const void *k_compact, const int32_t *rep_heads, int B, int H,
                             int k, int T, int Tc_cap, int d, int dtype, float scale, void *workspace,
                             size_t workspace_bytes, void *stream, void *start_event, void *stop_event);
int chai_decode_values_timed(const void *v_cache, const int32_t *head_to_cluster, const int32_t *rep_heads,
                             int B, int H, int k, int T, int T_cap, int d, int dtype, float *out,
                             float *probs_out, void *workspace, size_t workspace_bytes, void *stream,
                             void *start_event, void *stop_event);

/*
 * Ablation of Section 4.5 (values pruned as well): every head of a cluster
 * takes the representative's values too, so only the representatives' K and
 * V are cached.  The paper reports that this costs accuracy; it is here to
 * price the variant.
 *   out[b][h][:] = sum_t p_c[t] * v_compact[b][c][t][:],  c = head_to_cluster[b][h]
 * with p_c the probabilities of chai_decode_attention.
 *
 *   v_compact [B,k,Tv_cap,d]  slot j = values of head rep_heads[b][j]; build it
 *                             with chai_compact_kcache (a plain gather that
 *                             serves V as well) and grow it with
 *                             chai_append_kv_shared_v
 *   out       [B,H,d] fp32    rows of heads whose label is outside [0,k) are
 *                             left untouched
 *   workspace chai_decode_workspace_bytes(B,H,k,T,...) bytes suffice
 * Other arguments, limits and errors as chai_decode_attention.
 *
 * chai_append_kv_shared_v: position `pos` of both compact caches takes the
 * new token's K and V rows of the representatives (k_new, v_new [B,H,d]).
 */
int chai_decode_attention_shared_v(const void *q, const void *k_compact, const void *v_compact,
                                   const int32_t *head_to_cluster, const int32_t *rep_heads, int B, int H,
                                   int k, int T, int Tc_cap, int Tv_cap, int d, int dtype, float scale,
                                   float *out, void *workspace, size_t workspace_bytes, void *stream);
int chai_append_kv_shared_v(const void *k_new, const void *v_new, const int32_t *rep_heads, void *k_compact,
                            void *v_compact, int B, int H, int k, int pos, int Tc_cap, int Tv_cap, int d,
                            int dtype, void *stream);

/*
 * Quantised K,V caches (Section 2, related work: quantising the K,V cache is
 * orthogonal to clustering heads and composes with it; the paper fixes no
 * format).  Format used here: elements are 8-bit floating point E4M3 of the
 * OCP 8-bit floating point specification (1 sign, 4 exponent bits with bias
 * 7, 3 mantissa bits, subnormals, no infinities, largest finite value 448),
 * with ONE fp32 scale per cached row (one token of one key or value stream):
 *     scale = max_i |x_i| / 448,   code_i = nearest E4M3 (ties to even) of
 *     x_i * (448 / max_i |x_i|),   all three operations in fp32;
 * an all-zero row has scale 0 and codes 0.  The dequantised element is
 * decode(code_i) * scale, and attention over quantised caches is attention
 * over the dequantised caches.  A cache stream is then 132 bytes per token
 * instead of 256.
 *
 * chai_quantize_rows: n_rows rows of d = 128 elements (dtype fp32 or bf16,
 *   dense, 16-byte aligned) -> codes [n_rows,128] uint8 and scales [n_rows].
 *   A whole cache [B,S,T_cap,128] is n_rows = B*S*T_cap rows.
 * chai_append_kv_q8: cache growth by one token, quantising on the way in:
 *     k8[b][j][pos], kscale[b][j][pos] <- quantised k_new[b][rep_heads[b][j]]
 *     v8[b][h][pos], vscale[b][h][pos] <- quantised v_new[b][h]
 *   k_new, v_new [B,H,d] in `dtype`; k8 [B,k,Tc_cap,d], kscale [B,k,Tc_cap];
 *   v8 [B,H,T_cap,d], vscale [B,H,T_cap].
 * chai_decode_attention_q8: chai_decode_attention over such caches.  q stays
 *   unquantised ([B,H,d] in q_dtype); out, probs_out, maps, limits and errors
 *   as chai_decode_attention; workspace of chai_decode_q8_workspace_bytes
 *   bytes (monotone in T).  The _timed form also takes two pairs of HIP
 *   events (any of them NULL) that the runtime stamps with the begin and the
 *   end of the score kernel and of the value kernel.
 */
int chai_quantize_rows(const void *x, int dtype, long long n_rows, int d, uint8_t *codes, float *scales,
                       void *stream);
int chai_append_kv_q8(const void *k_new, const void *v_new, const int32_t *rep_heads, uint8_t *k8,
                      float *kscale, uint8_t *v8, float *vscale, int B, int H, int k, int pos, int Tc_cap,
                      int T_cap, int d, int dtype, void *stream);
size_t chai_decode_q8_workspace_bytes(int B, int H, int k, int T, int d);
int chai_decode_attention_q8(const void *q, const uint8_t *k8, const float *kscale, const uint8_t *v8,
                             const float *vscale, const int32_t *head_to_cluster, const int32_t *rep_heads,
                             int B, int H, int k, int T, int Tc_cap, int T_cap, int d, int q_dtype,
                             float scale, float *out, float *probs_out, void *workspace,
                             size_t workspace_bytes, void *stream);
int chai_decode_attention_q8_timed(const void *q, const uint8_t *k8, const float *kscale, const uint8_t *v8,
                                   const float *vscale, const int32_t *head_to_cluster,
                                   const int32_t *rep_heads, int B, int H, int k, int T, int Tc_cap, int T_cap,
                                   int d, int q_dtype, float scale, float *out, float *probs_out,
                                   void *workspace, size_t workspace_bytes, void *stream, void *score_start,
                                   void *score_stop, void *value_start, void *value_stop);

/*
 * Dense multi-head decode attention, the definition of Section 2
 * (A_h = softmax(q_h K_h^T / sqrt(d)), y = A_0 V_0 (+) A_1 V_1 ...): the
 * baseline clustered attention is compared against.  Runs the same kernels
 * with every head its own cluster and K read in place.
 *
 *   q [B,H,d]; k_cache, v_cache [B,H,T_cap,d]; out [B,H,d] fp32
 *   workspace: chai_decode_workspace_bytes(B,H,H,T,d,dtype) bytes.
 */
int chai_dense_decode_attention(const void *q, const void *k_cache, const void *v_cache, int B, int H,
                                int T, int T_cap, int d, int dtype, float scale, float *out,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * Clustered-head attention over a block of prompt positions: the prefill that
 * follows the membership decision (Section 3.5: after the cluster membership
 * is fixed, multi-head attention is replaced by clustered-head attention for
 * the rest of the request; Section 4.4 prices it in the time to first token;
 * attention definition of Section 2, causal).
 *
 * Query row i (0 <= i < Tq) sits at sequence position q_start + i and sees
 * positions 0 .. q_start + i:
 *   for cluster j with representative r = rep_heads[b][j] >= 0
 *       p_j,i = softmax_t( scale * q[b][r][i] . k_compact[b][j][t] ),  t <= q_start + i
 *   for head h in cluster c:  out[b][h][i][:] = sum_t p_c,i[t] * v_cache[b][h][t][:]
 * The scores of a cluster are computed once and applied to the values of its
 * member heads.  bf16 inputs only and scale > 0 (otherwise
 * CHAI_ERR_UNSUPPORTED).  Scores
 * accumulate in fp32 from exact bf16 products; probabilities are rounded to
 * fp16 and values converted to fp16 for the second product (fp32
 * accumulation): the conversion is exact for 2^-14 <= |v| <= 65504, loses
 * low bits below that, and |v| must not exceed 65504.
 *
 *   q         [B,H,Tq,d]        only representatives' rows are read
 *   k_compact [B,k,Tc_cap,d]    keys of positions 0 .. q_start+Tq-1 present
 *   v_cache   [B,H,T_cap,d]     values of positions 0 .. q_start+Tq-1 present
 *   out       [B,H,Tq,d] fp32, written for heads whose cluster slot is in use
 *   workspace chai_prefill_workspace_bytes(B,H,k,q_start+Tq) bytes, 256-byte
 *             aligned (holds the work list and a transposed fp16 copy of the
 *             values, B*H*d*roundup(q_start+Tq,64)*2 bytes)
 * q_start + Tq <= min(T_cap, Tc_cap), Tq >= 1, q_start >= 0, H <= 4096, q_start + Tq <= 2^23 - 64 (one head's
 * keys are addressed with 32-bit byte offsets; beyond that CHAI_ERR_UNSUPPORTED).
 *
 * chai_dense_prefill_attention: the dense baseline (every head its own
 * cluster, K read in place), same kernel.
 *
 * chai_prefill_attention_timed: the same call with two hipEvent_t handles
 * passed as void* (timing enabled, either may be NULL) that the runtime
 * stamps with the begin and the end of the main kernel; the V^T pre-pass and
 * the work-list kernel that run before it are outside the pair.
 */
size_t chai_prefill_workspace_bytes(int B, int H, int k, int n_keys);
int chai_prefill_attention(const void *q, const void *k_compact, const void *v_cache,
                           const int32_t *head_to_cluster, const int32_t *rep_heads, int B, int H, int k,
                           int Tq, int q_start, int Tc_cap, int T_cap, int d, int dtype, float scale,
                           float *out, void *workspace, size_t workspace_bytes, void *stream);
int chai_prefill_attention_timed(const void *q, const void *k_compact, const void *v_cache,
                                 const int32_t *head_to_cluster, const int32_t *rep_heads, int B, int H, int k,
                                 int Tq, int q_start, int Tc_cap, int T_cap, int d, int dtype, float scale,
                                 float *out, void *workspace, size_t workspace_bytes, void *stream,
                                 void *start_event, void *stop_event);
int chai_dense_prefill_attention(const void *q, const void *k_cache, const void *v_cache, int B, int H, int Tq,
                                 int q_start, int T_cap, int d, int dtype, float scale, float *out,
                                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * Query and key projections of the representative heads only (Fig. 3 and
 * Section 3.5: clustered attention needs the query and key vectors of one
 * head per cluster, so the share of W_Q and W_K that belongs to the other
 * heads is never multiplied; the new keys go straight into the pruned K
 * cache).  For batch row b, slot j with r = rep_heads[b][j] >= 0, token
 * i < Tn:
 *   q_out[b][r][i][:]            = x[b][i][:] . w_q[r*d .. r*d+d-1][:]^T
 *   k_compact[b][j][pos0 + i][:] = x[b][i][:] . w_k[r*d .. r*d+d-1][:]^T
 * fp32 accumulation of exact bf16 products, one rounding (to nearest even)
 * to bf16.  No bias term.
 *
 *   x         [B,Tn,D] bf16      activations of Tn tokens per batch row (a
 *                                prompt block, or Tn = 1 for a decode step)
 *   w_q, w_k  [H*d, D] bf16      one row per output feature (the layout of a
 *                                linear layer's weight)
 *   q_out     [B,H,Tn,d] bf16    rows of representatives written, others
 *                                untouched (the layout chai_prefill_attention
 *                                and, with Tn = 1, chai_decode_attention read)
 *   k_compact [B,k,Tc_cap,d]     rows pos0 .. pos0+Tn-1 of used slots written
 * bf16 only, d = 128, D a multiple of 64, Tn*D < 2^31 (otherwise
 * CHAI_ERR_UNSUPPORTED); pos0 + Tn <= Tc_cap.  The saving is in flops (a
 * fraction k/H of the dense projections); at Tn = 1 the call is bound by
 * reading the representatives' weights.
 *
 * chai_project_qk_timed: two more arguments, hipEvent_t handles as void*
 * that the runtime stamps with the kernel's begin and end (either may be
 * NULL).
 */
int chai_project_qk(const void *x, const void *w_q, const void *w_k, const int32_t *rep_heads, int B, int H, int k,
                    int Tn, int D, int d, int dtype, void *q_out, void *k_compact, int pos0, int Tc_cap,
                    void *stream);
int chai_project_qk_timed(const void *x, const void *w_q, const void *w_k, const int32_t *rep_heads, int B, int H,
                          int k, int Tn, int D, int d, int dtype, void *q_out, void *k_compact, int pos0,
                          int Tc_cap, void *stream, void *start_event, void *stop_event);

#ifdef __cplusplus
}
#endif
#endif /* CHAI_H */
