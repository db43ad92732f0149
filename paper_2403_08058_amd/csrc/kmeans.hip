// Cluster-membership kernels: the 5-token attention-score features (Section 3.3, with f(Q,K) = softmax(Q K^T)
// of Section 3.1) and K-Means over them (Section 3.5; clustering error of Section 3.2).
//
// The k-means result must be bit-identical to the sequential statement of the algorithm for the same feature
// bits, so every fp64 multiply, add, subtract and divide below is rounded on its own: this file is compiled
// with -ffp-contract=off, the pragma repeats it, and each sum runs in the stated index order inside ONE
// thread (threads split independent sums, never one sum).
#include "chai_internal.h"

#pragma clang fp contract(off)

namespace chai {

namespace {

// ---------------------------------------------------------------------------------------------------------
// Features: grid (H, B), one wave per head.  Lane p < n_tok*(n_tok+1)/2 owns one causal (i, j) pair and runs
// its 128-term dot product in element order in fp64; lane i < n_tok then normalises row i.
// ---------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void feature_kernel(const void *__restrict__ q5, const void *__restrict__ k5,
                                                     int H, int n_tok, int bf16, long long qs, long long ks,
                                                     double scale, float *__restrict__ feat)
{
    __shared__ double s[8][8];
    const int h = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    const size_t head = (size_t)b * H + h;

    // lane -> (i, j) with j <= i, row by row
    int i = 0, j = lane;
    while (i < n_tok && j > i) { j -= i + 1; ++i; }
    if (i < n_tok) {
        const size_t qo = head * (size_t)qs + (size_t)i * kHeadDim;
        const size_t ko = head * (size_t)ks + (size_t)j * kHeadDim;
        // 16-byte loads (rows start on 16-byte boundaries: the strides are multiples of 8 elements); the products
        // are still added one by one in element order
        double acc = 0.0;
        if (bf16) {
            const uint4 *qv = reinterpret_cast<const uint4 *>(static_cast<const unsigned short *>(q5) + qo);
            const uint4 *kv = reinterpret_cast<const uint4 *>(static_cast<const unsigned short *>(k5) + ko);
#pragma unroll 4
            for (int c8 = 0; c8 < kHeadDim / 8; ++c8) {
                const uint4 a = qv[c8], bb = kv[c8];
                const unsigned int aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {bb.x, bb.y, bb.z, bb.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const unsigned int abits = (e & 1) ? (aw[e >> 1] & 0xffff0000u) : (aw[e >> 1] << 16);
                    const unsigned int bbits = (e & 1) ? (bw[e >> 1] & 0xffff0000u) : (bw[e >> 1] << 16);
                    const double prod = (double)__uint_as_float(abits) * (double)__uint_as_float(bbits);
                    acc = acc + prod;
                }
            }
        } else {
            const float4 *qv = reinterpret_cast<const float4 *>(static_cast<const float *>(q5) + qo);
            const float4 *kv = reinterpret_cast<const float4 *>(static_cast<const float *>(k5) + ko);
#pragma unroll 4
            for (int c4 = 0; c4 < kHeadDim / 4; ++c4) {
                const float4 a = qv[c4], bb = kv[c4];
                const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {bb.x, bb.y, bb.z, bb.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const double prod = (double)av[e] * (double)bv[e];
                    acc = acc + prod;
                }
            }
        }
        s[i][j] = scale * acc;
    }
    __syncthreads();
    if (lane < n_tok) {
        const int row = lane;
        double m = s[row][0];
        for (int c = 1; c <= row; ++c) m = fmax(m, s[row][c]);
        double e[8];
        double z = 0.0;
        for (int c = 0; c <= row; ++c) { e[c] = exp(s[row][c] - m); z = z + e[c]; }
        float *f = feat + head * (size_t)(n_tok * n_tok) + (size_t)row * n_tok;
        for (int c = 0; c < n_tok; ++c) f[c] = c <= row ? (float)(e[c] / z) : 0.0f;
    }
}

// ---------------------------------------------------------------------------------------------------------
// K-Means: grid (B), one workgroup of 512 threads per batch row.  Dynamic LDS: centres [k][F] fp64, per-head
// distance [H] fp64, slice winners [H][slices], assignment/previous assignment/member order [H],
// counts/labels/list starts [k], and a copy of the features when it fits.
// ---------------------------------------------------------------------------------------------------------
__device__ __forceinline__ double sqdist(const float *__restrict__ x, const double *c, int F)
{
    double acc = 0.0;
    for (int f = 0; f < F; ++f) {
        const double diff = (double)x[f] - c[f];
        const double sq = diff * diff;
        acc = acc + sq;
    }
    return acc;
}

// The same sum with the head's coordinates in registers: every term in index order, terms past F left out.  Fully
// unrolled, so the loads of the centre's coordinates are all in flight together instead of one per iteration.
constexpr int kRegF = 32;
constexpr int kHeadWaves = 4;         // waves that own a head each (H <= 256)
constexpr int kKmBlock = 512;        // threads of the k-means workgroup: more slices per head, one round for the update
__device__ __forceinline__ double sqdist_regs(const double (&x)[kRegF], const double *c, int F)
{
    double acc = 0.0;
#pragma unroll
    for (int f = 0; f < kRegF; ++f) {
        if (f < F) {
            const double diff = x[f] - c[f];
            const double sq = diff * diff;
            acc = acc + sq;
        }
    }
    return acc;
}

__global__ __launch_bounds__(kKmBlock) void kmeans_kernel(const float *__restrict__ feat, int H, int F, int k,
                                                        const int32_t *__restrict__ init_heads, int max_iter,
                                                        int slices, int stage_x, int32_t *__restrict__ h2c,
                                                        int32_t *__restrict__ rep, int32_t *__restrict__ ncl,
                                                        int32_t *__restrict__ iters)
{
    extern __shared__ double lds[];
    double *centre = lds;                                   // [k][F]
    double *dmin = centre + (size_t)k * F;                  // [H]      distance of a head to its centre
    double *cand_d = dmin + H;                              // [H][slices] best distance found by a slice
    int *cand_j = reinterpret_cast<int *>(cand_d + (size_t)H * slices);   // [H][slices] and its centre
    int *assign = cand_j + (size_t)H * slices;              // [H]
    int *prev = assign + H;                                 // [H]
    int *count = prev + H;                                  // [k]
    int *label = count + k;                                 // [k]
    int *order = label + k;                                 // [H] heads sorted by centre, ascending inside a centre
    int *first = order + H;                                 // [k] where a centre's heads start in `order`
    int *wave_count = first + k;                            // [kHeadWaves][k] heads of a centre inside one wave
    float *x_lds = reinterpret_cast<float *>(wave_count + kHeadWaves * k);   // [H][F] copy of the features, when it fits

    const int b = blockIdx.x, tid = threadIdx.x;
    const float *Xg = feat + (size_t)b * H * F;
    if (stage_x)
        for (int i = tid; i < H * F; i += kKmBlock) x_lds[i] = Xg[i];
    const float *X = stage_x ? x_lds : Xg;                  // same values either way

    for (int i = tid; i < k * F; i += kKmBlock) {
        const int j = i / F, f = i - j * F;
        const int h0 = min(max(init_heads[(size_t)b * k + j], 0), H - 1);
        centre[i] = (double)Xg[(size_t)h0 * F + f];
    }
    for (int h = tid; h < H; h += kKmBlock) prev[h] = -1;
    __syncthreads();

    // H * slices <= kKmBlock: a thread keeps the same (head, slice) in every pass, so the head's coordinates are
    // converted once and stay in registers when there are few enough of them
    const bool in_regs = F <= kRegF && tid < H * slices;
    double xr[kRegF];
#pragma unroll
    for (int f = 0; f < kRegF; ++f) xr[f] = (in_regs && f < F) ? (double)Xg[(size_t)(tid / slices) * F + f] : 0.0;

    int it = 0;
    for (;;) {
        ++it;
        // Assignment.  The centres of a head are dealt to `slices` threads (slice s scans s, s+slices, ... in
        // ascending order and keeps the first smallest), then one thread per head picks the smallest of the
        // slice winners, the lowest centre on ties: the same centre a single ascending scan would pick.  Each
        // distance is one sequential fp64 sum inside one thread.
        for (int p = tid; p < H * slices; p += kKmBlock) {
            const int h = p / slices, sl = p - h * slices;
            const float *x = X + (size_t)h * F;
            int best = -1;
            double bd = 0.0;
            for (int j = sl; j < k; j += slices) {
                const double dj = in_regs ? sqdist_regs(xr, centre + (size_t)j * F, F) : sqdist(x, centre + (size_t)j * F, F);
                if (best < 0 || dj < bd) { bd = dj; best = j; }
            }
            cand_d[p] = bd;
            cand_j[p] = best;
        }
        __syncthreads();
        for (int h = tid; h < H; h += kKmBlock) {
            int best = cand_j[(size_t)h * slices];
            double bd = cand_d[(size_t)h * slices];
            for (int sl = 1; sl < slices; ++sl) {
                const int j = cand_j[(size_t)h * slices + sl];
                const double dj = cand_d[(size_t)h * slices + sl];
                if (j >= 0 && (dj < bd || (dj == bd && j < best))) { bd = dj; best = j; }
            }
            assign[h] = best;
            dmin[h] = bd;
        }
        for (int j = tid; j < k; j += kKmBlock) count[j] = 0;
        __syncthreads();
        // members per centre: every head adds one to its centre's counter (integers: any order gives the
        // sequential result)
        for (int h = tid; h < H; h += kKmBlock) atomicAdd(&count[assign[h]], 1);
        __syncthreads();
        int empty = 0;
        for (int j = tid; j < k; j += kKmBlock) empty |= count[j] == 0;
        // Centres that received no head take, in ascending order, the farthest head of a cluster that can spare
        // one.  Sequential by nature, but needed only when some centre is empty.
        if (__syncthreads_or(empty)) {
            if (tid == 0) {
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
            }
            __syncthreads();
        }
        int moved = 0;
        for (int h = tid; h < H; h += kKmBlock) {
            moved |= assign[h] != prev[h];
            prev[h] = assign[h];
        }
        const int changed = __syncthreads_or(moved);        // same value in every thread
        if (!changed || it >= max_iter) break;
        // member lists: the heads of centre j in ascending order, behind those of the centres before it.  Thread h
        // owns head h (H <= 256: the first four waves); its place is the number of lower heads of the same centre,
        // counted with one wave vote per centre plus the totals of the waves before it.
        {
            const int wv = tid >> 6, ln = tid & 63;
            const int a = tid < H ? assign[tid] : -1;
            int below = 0;
            if (wv < kHeadWaves) {
                for (int j = 0; j < k; ++j) {
                    const unsigned long long votes = __ballot(a == j);
                    if (a == j) below = __popcll(votes & ((1ull << ln) - 1ull));
                    if (ln == 0) wave_count[wv * k + j] = __popcll(votes);
                }
            }
            for (int j = tid; j < k; j += kKmBlock) {
                int at = 0;
                for (int i = 0; i < j; ++i) at += count[i];
                first[j] = at;
            }
            __syncthreads();
            if (tid < H) {
                int at = first[a] + below;
                for (int i = 0; i < wv; ++i) at += wave_count[i * k + a];
                order[at] = tid;
            }
        }
        __syncthreads();
        // update: one thread per (centre, coordinate), members added in head order
        for (int i = tid; i < k * F; i += kKmBlock) {
            const int j = i / F, f = i - j * F;
            const int n = count[j];
            if (n == 0) continue;
            const int *mem = order + first[j];
            double acc = 0.0;
#pragma unroll 4
            for (int m = 0; m < n; ++m) acc = acc + (double)X[(size_t)mem[m] * F + f];
            centre[i] = acc / (double)n;
        }
        __syncthreads();
    }
    __syncthreads();

    // canonical labels: clusters numbered by their lowest member, which represents them
    if (tid == 0) {
        for (int j = 0; j < k; ++j) { label[j] = -1; rep[(size_t)b * k + j] = -1; }
        int n = 0;
        for (int h = 0; h < H; ++h) {
            const int a = assign[h];
            if (label[a] < 0) {
                label[a] = n;
                rep[(size_t)b * k + n] = h;
                ++n;
            }
            h2c[(size_t)b * H + h] = label[a];
        }
        ncl[b] = n;
        if (iters) iters[b] = it;
    }
}

// ---------------------------------------------------------------------------------------------------------
// Clustering error of a given partition (Section 3.2): grid (B), 256 threads.  Means per (cluster, coordinate)
// by one thread each (members in head order), distance of every head to its cluster's mean by one thread each,
// then thread 0 adds the distances cluster by cluster, heads ascending: the order of the sequential statement.
// With rep_out, thread j also picks the member of cluster j nearest its mean (first of equals = lowest head,
// -1 for an empty slot).  Either output may be NULL.
// Dynamic LDS: means [k][F] fp64, distances [H] fp64, counts [k].
// ---------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void cluster_error_kernel(const float *__restrict__ feat,
                                                               const int32_t *__restrict__ h2c, int H, int F, int k,
                                                               double *__restrict__ sse,
                                                               int32_t *__restrict__ rep_out)
{
    extern __shared__ double lds[];
    double *mean = lds;                          // [k][F]
    double *dist = mean + (size_t)k * F;         // [H]
    int *count = reinterpret_cast<int *>(dist + H);   // [k]
    const int b = blockIdx.x, tid = threadIdx.x;
    const float *X = feat + (size_t)b * H * F;
    const int32_t *lab = h2c + (size_t)b * H;

    for (int j = tid; j < k; j += kBlock) {
        int c = 0;
        for (int h = 0; h < H; ++h) c += lab[h] == j;
        count[j] = c;
    }
    __syncthreads();
    for (int i = tid; i < k * F; i += kBlock) {
        const int j = i / F, f = i - j * F;
        if (count[j] == 0) continue;
        double acc = 0.0;
        for (int h = 0; h < H; ++h)
            if (lab[h] == j) acc = acc + (double)X[(size_t)h * F + f];
        mean[i] = acc / (double)count[j];
    }
    __syncthreads();
    for (int h = tid; h < H; h += kBlock) {
        const int j = lab[h];
        dist[h] = (j >= 0 && j < k) ? sqdist(X + (size_t)h * F, mean + (size_t)j * F, F) : 0.0;
    }
    __syncthreads();
    if (rep_out != nullptr) {
        for (int j = tid; j < k; j += kBlock) {
            int best = -1;
            double best_d = 0.0;
            for (int h = 0; h < H; ++h)
                if (lab[h] == j && (best < 0 || dist[h] < best_d)) {
                    best = h;
                    best_d = dist[h];
                }
            rep_out[(size_t)b * k + j] = best;
        }
    }
    if (sse != nullptr && tid == 0) {
        double total = 0.0;
        for (int j = 0; j < k; ++j)
            for (int h = 0; h < H; ++h)
                if (lab[h] == j) total += dist[h];
        sse[b] = total;
    }
}

// threads that share the centres of one head: as many as fit the workgroup, at most one per centre
int assignment_slices(int H, int k)
{
    int s = kKmBlock / H;
    if (s > k) s = k;
    return s < 1 ? 1 : s;
}

}  // namespace

int launch_score_features(const void *q5, const void *k5, int B, int H, int n_tok, int dtype, int64_t qs, int64_t ks,
                          float scale, float *feat, hipStream_t stream)
{
    return (int)launch_kernel(feature_kernel, dim3(H, B), dim3(64), 0, stream, KernelEvents(), q5, k5, H, n_tok,
                              dtype == CHAI_BF16 ? 1 : 0, (long long)qs, (long long)ks, (double)scale, feat);
}

size_t assign_clusters_lds_bytes(int H, int F, int k)
{
    const size_t sl = (size_t)assignment_slices(H, k);
    return sizeof(double) * ((size_t)k * F + H + H * sl) +
           sizeof(int) * (H * sl + 3 * (size_t)H + (3 + kHeadWaves) * (size_t)k);
}

// the features are copied to LDS too when that still fits the 64 KB a workgroup may ask for
constexpr size_t kKmeansLdsLimit = 64 * 1024 - 64;
size_t kmeans_feature_copy_bytes(int H, int F, int k)
{
    const size_t extra = sizeof(float) * (size_t)H * F;
    return assign_clusters_lds_bytes(H, F, k) + extra <= kKmeansLdsLimit ? extra : 0;
}

int launch_assign_clusters(const float *feat, int B, int H, int F, int k, const int32_t *init_heads, int max_iter,
                           int32_t *h2c, int32_t *rep, int32_t *ncl, int32_t *iters, hipStream_t stream)
{
    const size_t copy = kmeans_feature_copy_bytes(H, F, k);
    return (int)launch_kernel(kmeans_kernel, dim3(B), dim3(kKmBlock), assign_clusters_lds_bytes(H, F, k) + copy, stream,
                              KernelEvents(), feat, H, F, k, init_heads, max_iter, assignment_slices(H, k),
                              copy != 0 ? 1 : 0, h2c, rep, ncl, iters);
}

size_t cluster_error_lds_bytes(int H, int F, int k)
{
    return sizeof(double) * ((size_t)k * F + H) + sizeof(int) * (size_t)k;
}

int launch_cluster_error(const float *feat, const int32_t *h2c, int B, int H, int F, int k, double *sse,
                         int32_t *rep_out, hipStream_t stream)
{
    return (int)launch_kernel(cluster_error_kernel, dim3(B), dim3(kBlock), cluster_error_lds_bytes(H, F, k), stream,
                              KernelEvents(), feat, h2c, H, F, k, sse, rep_out);
}

}  // namespace chai
