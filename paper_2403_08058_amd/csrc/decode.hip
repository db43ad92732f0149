// Clustered-head decode attention for gfx950 (MI355X): the score kernel streams the compact K cache once per
// cluster, the value kernel streams the full V cache once per head.  Both are HBM-bandwidth kernels: every
// lane issues 16-byte loads, 16 lanes (bf16) or 32 lanes (fp32) cover one 128-element row, a wave64 load
// instruction covers 1 KiB of consecutive rows, and the four waves of a workgroup walk a contiguous region.
//
// Method: attention definition of Section 2; one score computation per cluster with the representative's
// query and keys, shared by the member heads, each applying it to its own values (Sections 3.4-3.5, Fig. 3).
#include "chai_internal.h"

namespace chai {

namespace {

constexpr int kUnroll = 8;        // independent 16-byte loads in flight per lane
constexpr int kMaxCs = 256;       // largest score chunk (= workgroup size: one thread per score)
constexpr int kMaxCp = 1024;      // largest value chunk (probabilities staged in LDS)

template <bool BF16>
struct Tile {
    static constexpr int EPL = BF16 ? 8 : 4;               // elements per lane per load (16 bytes)
    static constexpr int LPR = kHeadDim / EPL;             // lanes per row: 16 (bf16) / 32 (fp32)
    static constexpr int RPW = 64 / LPR;                   // rows per wave load: 4 / 2
    static constexpr int RPB = RPW * (kBlock / 64);        // rows per workgroup iteration: 16 / 8
    static constexpr int ROW_BYTES = kHeadDim * (BF16 ? 2 : 4);
};

__device__ __forceinline__ void unpack(const uint4 &raw, float (&f)[8])
{
    // bf16 pairs: the low half-word is the even element; a bf16 is the top half of an fp32
    f[0] = __uint_as_float(raw.x << 16); f[1] = __uint_as_float(raw.x & 0xffff0000u);
    f[2] = __uint_as_float(raw.y << 16); f[3] = __uint_as_float(raw.y & 0xffff0000u);
    f[4] = __uint_as_float(raw.z << 16); f[5] = __uint_as_float(raw.z & 0xffff0000u);
    f[6] = __uint_as_float(raw.w << 16); f[7] = __uint_as_float(raw.w & 0xffff0000u);
}

__device__ __forceinline__ void unpack(const uint4 &raw, float (&f)[4])
{
    f[0] = __uint_as_float(raw.x); f[1] = __uint_as_float(raw.y);
    f[2] = __uint_as_float(raw.z); f[3] = __uint_as_float(raw.w);
}

__device__ __forceinline__ uint4 load16(const char *p)
{
    return *reinterpret_cast<const uint4 *>(p);
}

// x + (x of the lane selected by a DPP control) -- cross-lane adds inside a 16-lane DPP row
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x)
{
    int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false);
    return x + __int_as_float(y);
}

// Sum over the lanes that share a row; every one of them ends up with the total.
template <bool BF16>
__device__ __forceinline__ float row_sum(float x)
{
    x = dpp_add<0xB1>(x);    // quad_perm [1,0,3,2]: lane ^ 1
    x = dpp_add<0x4E>(x);    // quad_perm [2,3,0,1]: lane ^ 2
    x = dpp_add<0x141>(x);   // row_half_mirror: other quad of the same 8 lanes
    x = dpp_add<0x140>(x);   // row_mirror: other half of the same 16 lanes
    if (!BF16) x += __shfl_xor(x, 16);   // fp32 rows span 32 lanes
    return x;
}

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// Workgroup-wide reductions over 4 waves; `red` is 4 floats of LDS, reusable right after return.
__device__ __forceinline__ float block_max(float x, float *red)
{
    x = wave_max(x);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
    __syncthreads();
    x = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    return x;
}

__device__ __forceinline__ float block_sum(float x, float *red)
{
    x = wave_sum(x);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
    __syncthreads();
    x = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
    return x;
}

// ---------------------------------------------------------------------------------------------------------
// Score kernel: s[b][j][t] = scale * q[b][rep(b,j)] . Kc[b][j][t], plus (max, sum of exp) per chunk.
// grid = (n_cs, k, B).  Also clears the split counters the value kernel uses.
// ---------------------------------------------------------------------------------------------------------
template <bool BF16, bool IDENT>
__global__ __launch_bounds__(kBlock) void score_kernel(const char *__restrict__ q, const char *__restrict__ kc,
                                                       const int32_t *__restrict__ rep, int H, int k, int T,
                                                       int Tc_cap, float scale, int cs, int n_cs,
                                                       float *__restrict__ scores, float2 *__restrict__ stats,
                                                       unsigned int *__restrict__ counters)
{
    using TL = Tile<BF16>;
    __shared__ float s_lds[kMaxCs];
    __shared__ float red[4];

    const int tid = threadIdx.x;
    const int chunk = blockIdx.x, j = blockIdx.y, b = blockIdx.z;

    if (chunk == 0 && j == 0)
        for (int i = tid; i < H; i += kBlock) counters[(size_t)b * H + i] = 0u;

    int r = IDENT ? j : rep[(size_t)b * k + j];
    if (r < 0) return;                       // unused cluster slot (same decision for the whole workgroup)
    r = min(r, H - 1);

    const int lane = tid & 63, w = tid >> 6;
    const int cg = lane % TL::LPR, rg = lane / TL::LPR;
    const int t0 = chunk * cs;
    const int n = min(T, t0 + cs) - t0;      // >= 1 by construction of n_cs

    float qf[TL::EPL];
    unpack(load16(q + ((size_t)b * H + r) * TL::ROW_BYTES + cg * 16), qf);

    const char *kbase = kc + (((size_t)b * k + j) * Tc_cap + t0) * TL::ROW_BYTES + cg * 16;
    const int n_iter = (n + TL::RPB - 1) / TL::RPB;
    for (int i0 = 0; i0 < n_iter; i0 += kUnroll) {
        uint4 raw[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int tl = (i0 + u) * TL::RPB + w * TL::RPW + rg;
            raw[u] = load16(kbase + (size_t)min(tl, n - 1) * TL::ROW_BYTES);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int tl = (i0 + u) * TL::RPB + w * TL::RPW + rg;
            float f[TL::EPL];
            unpack(raw[u], f);
            float dot = 0.f;
#pragma unroll
            for (int e = 0; e < TL::EPL; ++e) dot = fmaf(qf[e], f[e], dot);
            dot = row_sum<BF16>(dot);
            if (cg == 0 && tl < n) s_lds[tl] = scale * dot;
        }
    }
    __syncthreads();

    const float sv = tid < n ? s_lds[tid] : -INFINITY;
    const float m = block_max(sv, red);
    const float l = block_sum(tid < n ? expf(sv - m) : 0.f, red);
    const size_t row = (size_t)b * k + j;
    if (tid < n) scores[row * T + t0 + tid] = sv;
    if (tid == 0) stats[row * n_cs + chunk] = make_float2(m, l);
}

// ---------------------------------------------------------------------------------------------------------
// Value kernel: out[b][h] = sum_t p_c[t] * V[b][h][t], c = cluster of h.  grid = (n_cp, H, B).
// Each workgroup merges the chunk statistics of its cluster into the global (max, denominator), turns its
// chunk of scores into final probabilities in LDS, streams its chunk of V, and writes a partial output; the
// workgroup that finishes last for a head adds the partials in chunk order.
// ---------------------------------------------------------------------------------------------------------
template <bool BF16, bool IDENT>
__global__ __launch_bounds__(kBlock) void value_kernel(const char *__restrict__ v, const int32_t *__restrict__ h2c,
                                                       const int32_t *__restrict__ rep, int H, int k, int T,
                                                       int T_cap, int n_cs, int cp, int n_cp,
                                                       const float *__restrict__ scores,
                                                       const float2 *__restrict__ stats, float *partial,
                                                       unsigned int *counters, float *__restrict__ out,
                                                       float *__restrict__ probs_out)
{
    using TL = Tile<BF16>;
    __shared__ float p_lds[kMaxCp];
    __shared__ float red[4];
    __shared__ float acc_lds[kBlock / 64][kHeadDim];
    __shared__ int last_flag;

    const int tid = threadIdx.x;
    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int c = IDENT ? h : min(max(h2c[(size_t)b * H + h], 0), k - 1);
    const size_t crow = (size_t)b * k + c;
    const int t0 = split * cp;
    const int n = min(T, t0 + cp) - t0;

    // softmax statistics of the whole row from the per-chunk records (exact merge of the chunks)
    const float2 *st = stats + crow * n_cs;
    float m = -INFINITY;
    for (int i = tid; i < n_cs; i += kBlock) m = fmaxf(m, st[i].x);
    const float M = block_max(m, red);
    float l = 0.f;
    for (int i = tid; i < n_cs; i += kBlock) l += st[i].y * expf(st[i].x - M);
    const float inv = 1.0f / block_sum(l, red);

    const bool write_p = probs_out != nullptr && (IDENT || rep[crow] == h);
    for (int i = tid; i < n; i += kBlock) {
        const float p = expf(scores[crow * T + t0 + i] - M) * inv;
        p_lds[i] = p;
        if (write_p) probs_out[crow * T + t0 + i] = p;
    }
    __syncthreads();

    const int lane = tid & 63, w = tid >> 6;
    const int cg = lane % TL::LPR, rg = lane / TL::LPR;
    const char *vbase = v + (((size_t)b * H + h) * T_cap + t0) * TL::ROW_BYTES + cg * 16;

    float acc[TL::EPL];
#pragma unroll
    for (int e = 0; e < TL::EPL; ++e) acc[e] = 0.f;

    const int n_iter = (n + TL::RPB - 1) / TL::RPB;
    for (int i0 = 0; i0 < n_iter; i0 += kUnroll) {
        uint4 raw[kUnroll];
        float pv[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int tl = (i0 + u) * TL::RPB + w * TL::RPW + rg;
            raw[u] = load16(vbase + (size_t)min(tl, n - 1) * TL::ROW_BYTES);
            pv[u] = tl < n ? p_lds[tl] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            float f[TL::EPL];
            unpack(raw[u], f);
#pragma unroll
            for (int e = 0; e < TL::EPL; ++e) acc[e] = fmaf(pv[u], f[e], acc[e]);
        }
    }

    // rows of one wave load, then the four waves
#pragma unroll
    for (int e = 0; e < TL::EPL; ++e) {
        if (BF16) acc[e] += __shfl_xor(acc[e], 16);
        acc[e] += __shfl_xor(acc[e], 32);
    }
    if (rg == 0) {
#pragma unroll
        for (int e = 0; e < TL::EPL; ++e) acc_lds[w][cg * TL::EPL + e] = acc[e];
    }
    __syncthreads();
    float val = 0.f;
    if (tid < kHeadDim) val = (acc_lds[0][tid] + acc_lds[1][tid]) + (acc_lds[2][tid] + acc_lds[3][tid]);

    const size_t orow = (size_t)b * H + h;
    if (n_cp == 1) {
        if (tid < kHeadDim) out[orow * kHeadDim + tid] = val;
        return;
    }

    if (tid < kHeadDim) partial[(orow * n_cp + split) * kHeadDim + tid] = val;
    __threadfence();                                   // partials visible device-wide before the count
    __syncthreads();
    if (tid == 0) last_flag = (atomicAdd(&counters[orow], 1u) == (unsigned int)(n_cp - 1));
    __syncthreads();
    if (!last_flag) return;
    __threadfence();                                   // see the other workgroups' partials
    if (tid < kHeadDim) {
        float sum = 0.f;
        for (int s = 0; s < n_cp; ++s)
            sum += __hip_atomic_load(&partial[(orow * n_cp + s) * kHeadDim + tid], __ATOMIC_RELAXED,
                                     __HIP_MEMORY_SCOPE_AGENT);
        out[orow * kHeadDim + tid] = sum;
    }
}

struct Workspace {
    float *scores;
    float2 *stats;
    float *partial;
    unsigned int *counters;
    Workspace(void *base, const DecodePlan &pl)
    {
        char *ws = static_cast<char *>(base);
        scores = reinterpret_cast<float *>(ws + pl.off_scores);
        stats = reinterpret_cast<float2 *>(ws + pl.off_stats);
        partial = reinterpret_cast<float *>(ws + pl.off_partial);
        counters = reinterpret_cast<unsigned int *>(ws + pl.off_counter);
    }
};

template <bool BF16, bool IDENT>
int scores_typed(const void *q, const void *kc, const int32_t *rep, int B, int H, int k, int T, int Tc_cap,
                 float scale, const Workspace &w, const DecodePlan &pl, hipStream_t stream)
{
    score_kernel<BF16, IDENT><<<dim3(pl.n_cs, k, B), kBlock, 0, stream>>>(
        static_cast<const char *>(q), static_cast<const char *>(kc), rep, H, k, T, Tc_cap, scale, pl.cs, pl.n_cs,
        w.scores, w.stats, w.counters);
    return (int)hipGetLastError();
}

template <bool BF16, bool IDENT>
int values_typed(const void *v, const int32_t *h2c, const int32_t *rep, int B, int H, int k, int T, int T_cap,
                 float *out, float *probs_out, const Workspace &w, const DecodePlan &pl, hipStream_t stream)
{
    value_kernel<BF16, IDENT><<<dim3(pl.n_cp, H, B), kBlock, 0, stream>>>(
        static_cast<const char *>(v), h2c, rep, H, k, T, T_cap, pl.n_cs, pl.cp, pl.n_cp, w.scores, w.stats,
        w.partial, w.counters, out, probs_out);
    return (int)hipGetLastError();
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

DecodePlan make_decode_plan(int B, int H, int k, int T)
{
    DecodePlan pl;
    // score chunk: the largest of 256/128/64 tokens that still gives >= 1024 workgroups (4 per CU)
    pl.cs = 64;
    for (int c : {256, 128}) {
        if ((long long)B * k * ((T + c - 1) / c) >= 1024) { pl.cs = c; break; }
    }
    pl.n_cs = (T + pl.cs - 1) / pl.cs;
    // value chunk: the largest of 1024/512/256 tokens that still gives >= 2048 workgroups (8 per CU)
    pl.cp = 128;
    for (int c : {1024, 512, 256}) {
        if ((long long)B * H * ((T + c - 1) / c) >= 2048) { pl.cp = c; break; }
    }
    pl.n_cp = (T + pl.cp - 1) / pl.cp;

    // Region sizes are upper bounds over every chunking the rules above can pick (smallest chunks), so the
    // total grows monotonically with T: a workspace sized for the cache capacity serves every shorter context.
    const size_t max_n_cs = (size_t)(T + 63) / 64, max_n_cp = (size_t)(T + 127) / 128;
    size_t off = 0;
    pl.off_scores = off;  off = align_up(off + (size_t)B * k * T * sizeof(float), 256);
    pl.off_stats = off;   off = align_up(off + (size_t)B * k * max_n_cs * sizeof(float2), 256);
    pl.off_partial = off; off = align_up(off + (size_t)B * H * max_n_cp * kHeadDim * sizeof(float), 256);
    pl.off_counter = off; off = align_up(off + (size_t)B * H * sizeof(unsigned int), 256);
    pl.bytes = off;
    return pl;
}

int launch_scores(const void *q, const void *kc, const int32_t *rep, int B, int H, int k, int T, int Tc_cap, int dtype,
                  float scale, void *workspace, const DecodePlan &plan, bool identity, hipStream_t stream)
{
    const Workspace w(workspace, plan);
    if (dtype == CHAI_BF16)
        return identity ? scores_typed<true, true>(q, kc, rep, B, H, k, T, Tc_cap, scale, w, plan, stream)
                        : scores_typed<true, false>(q, kc, rep, B, H, k, T, Tc_cap, scale, w, plan, stream);
    return identity ? scores_typed<false, true>(q, kc, rep, B, H, k, T, Tc_cap, scale, w, plan, stream)
                    : scores_typed<false, false>(q, kc, rep, B, H, k, T, Tc_cap, scale, w, plan, stream);
}

int launch_values(const void *v, const int32_t *h2c, const int32_t *rep, int B, int H, int k, int T, int T_cap,
                  int dtype, float *out, float *probs_out, void *workspace, const DecodePlan &plan, bool identity,
                  hipStream_t stream)
{
    const Workspace w(workspace, plan);
    if (dtype == CHAI_BF16)
        return identity ? values_typed<true, true>(v, h2c, rep, B, H, k, T, T_cap, out, probs_out, w, plan, stream)
                        : values_typed<true, false>(v, h2c, rep, B, H, k, T, T_cap, out, probs_out, w, plan, stream);
    return identity ? values_typed<false, true>(v, h2c, rep, B, H, k, T, T_cap, out, probs_out, w, plan, stream)
                    : values_typed<false, false>(v, h2c, rep, B, H, k, T, T_cap, out, probs_out, w, plan, stream);
}

}  // namespace chai
