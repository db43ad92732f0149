// Clustered-head decode attention for gfx950 (MI355X): the score kernel streams the compact K cache once per
// cluster, the value kernel streams the full V cache once per head.  Both are HBM-bandwidth kernels: every
// lane issues 16-byte non-temporal loads, 8 lanes (8-bit codes), 16 lanes (bf16) or 32 lanes (fp32) cover one
// 128-element row, a wave64 load instruction covers 1 KiB of consecutive rows, a wave keeps 8 KiB (one batch) or
// more in flight and the waves of a workgroup walk neighbouring batches of one contiguous region.  Caches of
// 8-bit floating point codes (E4M3, one fp32 scale per row) go through the same kernels: the codes are widened
// by the hardware conversion, the row's scale is folded into the row's score (keys) or probability (values).
//
// Method: attention definition of Section 2; one score computation per cluster with the representative's
// query and keys, shared by the member heads, each applying it to its own values (Sections 3.4-3.5, Fig. 3).
#include "chai_internal.h"

#include <hip/hip_ext.h>

namespace chai {

namespace {

constexpr int kUnroll = 8;        // 16-byte loads per lane in one batch
constexpr int kScoreWaves = 4;    // waves per workgroup of the score kernel ...
constexpr int kScoreBatches = 2;  // ... each with this many batches in flight

// storage types of the caches inside this file: CHAI_F32, CHAI_BF16, and 8-bit E4M3 codes with per-row scales
constexpr int DT_F32 = CHAI_F32, DT_BF16 = CHAI_BF16, DT_E4M3 = 2;
template <int DT>
struct Elem {
    static constexpr int BYTES = DT == DT_F32 ? 4 : (DT == DT_BF16 ? 2 : 1);
    static constexpr int EPL = 16 / BYTES;                 // elements per lane per load (16 bytes)
};

template <int DT>
struct Tile {
    static constexpr int EPL = Elem<DT>::EPL;
    static constexpr int LPR = kHeadDim / EPL;             // lanes per row: 32 (fp32) / 16 (bf16) / 8 (codes)
    static constexpr int RPW = 64 / LPR;                   // rows per wave load: 2 / 4 / 8
    static constexpr int BATCH = RPW * kUnroll;            // rows per wave batch: 16 / 32 / 64
    static constexpr int ROW_BYTES = kHeadDim * Elem<DT>::BYTES;
};

// Value kernel: a workgroup may take only one of DS column parts of its head's rows (DS = 1: whole rows).
template <int DT, int DS>
struct VTile {
    static constexpr int EPL = Elem<DT>::EPL;
    static constexpr int COLS = kHeadDim / DS;             // columns of this workgroup
    static constexpr int LPR = COLS / EPL;                 // lanes per (part of a) row
    static constexpr int RPW = 64 / LPR;                   // rows per wave load
    static constexpr int BATCH = RPW * kUnroll;            // rows per wave batch (at most 64)
    static constexpr int ROW_BYTES = kHeadDim * Elem<DT>::BYTES;
    static constexpr int PART_BYTES = ROW_BYTES / DS;
    static_assert(BATCH <= 64, "one lane per row of a batch turns its score into a probability");
};

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void unpack(const u32x4 &raw, float (&f)[8])
{
    // bf16 pairs: the low half-word is the even element; a bf16 is the top half of an fp32
    f[0] = __uint_as_float(raw.x << 16); f[1] = __uint_as_float(raw.x & 0xffff0000u);
    f[2] = __uint_as_float(raw.y << 16); f[3] = __uint_as_float(raw.y & 0xffff0000u);
    f[4] = __uint_as_float(raw.z << 16); f[5] = __uint_as_float(raw.z & 0xffff0000u);
    f[6] = __uint_as_float(raw.w << 16); f[7] = __uint_as_float(raw.w & 0xffff0000u);
}

// sixteen E4M3 codes: the hardware conversion widens two bytes of a word at a time (exact)
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void unpack(const u32x4 &raw, float (&f)[16])
{
    const unsigned int w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], false);
        const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], true);
        f[4 * i + 0] = lo.x; f[4 * i + 1] = lo.y; f[4 * i + 2] = hi.x; f[4 * i + 3] = hi.y;
    }
}

__device__ __forceinline__ void unpack(const u32x4 &raw, float (&f)[4])
{
    f[0] = __uint_as_float(raw.x); f[1] = __uint_as_float(raw.y);
    f[2] = __uint_as_float(raw.z); f[3] = __uint_as_float(raw.w);
}

// The caches are read exactly once per call: non-temporal loads keep them from displacing the small,
// re-read score and statistics buffers in L2 (and measure ~10% faster than plain loads on a pure stream).
__device__ __forceinline__ u32x4 stream16(const char *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}

// x + (x of the lane selected by a DPP control) -- cross-lane adds inside a 16-lane DPP row
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x)
{
    int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false);
    return x + __int_as_float(y);
}

// Sum over the lanes that share a row; every one of them ends up with the total.
template <int DT>
__device__ __forceinline__ float row_sum(float x)
{
    x = dpp_add<0xB1>(x);    // quad_perm [1,0,3,2]: lane ^ 1
    x = dpp_add<0x4E>(x);    // quad_perm [2,3,0,1]: lane ^ 2
    x = dpp_add<0x141>(x);   // row_half_mirror: other quad of the same 8 lanes (rows of 8-bit codes end here)
    if (DT != DT_E4M3) x = dpp_add<0x140>(x);   // row_mirror: other half of the same 16 lanes
    if (DT == DT_F32) x += __shfl_xor(x, 16);   // fp32 rows span 32 lanes
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

// ---------------------------------------------------------------------------------------------------------
// Value kernel: out[b][h] = sum_t p_c[t] * V[b][h][t], c = cluster of h.  grid = (n_cp, H, B).
//
// Every wave works on its own: it merges the chunk statistics of its cluster into the row maximum M and the
// denominator (exact merge of the chunks), and then, batch by batch, its first BATCH lanes turn one score
// each into a final probability exp(s - M) / denominator, hand them to the other lanes through a private
// LDS strip, and all lanes accumulate p * V for the rows they loaded.  Each wave keeps NB batches (V rows and
// scores) in flight -- a buffer is refilled right after it is consumed -- and the first ones are requested
// before the statistics are merged; with NW independent waves per workgroup the stream never drains.  The
// only workgroup barrier is the one that adds up the waves at the end.  With one chunk per head the sum goes to `out`, otherwise to a partial row that
// combine_kernel adds up in chunk order.
// ---------------------------------------------------------------------------------------------------------
// APPEND: position T-1 is the token being decoded; the workgroup whose chunk ends there takes its value row from
// v_new [B,H,d], weighs it like any other row and writes it to the cache.
// DS = 2: two workgroups per head, each with half of the columns of every row (128-byte pieces, whole cache
// lines): twice the workgroups without partial rows to add up afterwards -- for head counts that are too small
// for one workgroup per head and would otherwise pay a combine launch.  grid = (n_cp, H * DS, B).
template <int DT, bool IDENT, int NW, int NB, bool WRITE_P, bool APPEND, int DS>
__device__ __forceinline__ void value_block(const char *__restrict__ v, const int32_t *__restrict__ h2c,
                                            const int32_t *__restrict__ rep, int H, int k, int T, int T_cap,
                                            int n_rec, int cp, int n_cp,
                                            const float *__restrict__ scores, const float2 *__restrict__ stats,
                                            float *__restrict__ partial, float *__restrict__ out,
                                            float *__restrict__ probs_out, const char *__restrict__ v_new,
                                            const float *__restrict__ vscale, int split, int hy, int b)
{
    using TL = VTile<DT, DS>;
    __shared__ float p_lds[NW][TL::BATCH];
    __shared__ float acc_lds[NW][TL::COLS];

    const int tid = threadIdx.x;
    const int lane = tid & 63, w = tid >> 6;
    const int cg = lane % TL::LPR, rg = lane / TL::LPR;
    const int h = hy / DS, dpart = hy % DS;
    const int t0 = split * cp;
    const int n_all = min(T, t0 + cp) - t0;
    const bool has_new = APPEND && split == n_cp - 1;        // this chunk ends with the token being decoded
    const int n = has_new ? n_all - 1 : n_all;               // rows that are in the cache already (may be 0)
    const int n_batches = (n + TL::BATCH - 1) / TL::BATCH;
    const int n_it = n_batches > w ? (n_batches - w + NW - 1) / NW : 0;     // batches of this wave

    // uniform base of the chunk + a 32-bit per-lane byte offset (a chunk is far below 4 GiB)
    const char *vbase = v + (((size_t)b * H + h) * T_cap + t0) * TL::ROW_BYTES;
    const unsigned int lane_off = dpart * TL::PART_BYTES + cg * 16;

    // one batch: the 16-byte pieces of kUnroll * RPW consecutive rows, and (lanes < BATCH) one row's score
    // (rows of 8-bit codes: also the row's scale)
    struct Batch {
        u32x4 v[kUnroll];
        float s;
        float vs;
    };
    const float *vsrow = DT == DT_E4M3 ? vscale + ((size_t)b * H + h) * T_cap + t0 : nullptr;
    Batch buf[NB];

    // Rows of batch `it` of this wave start at (it * NW + w) * BATCH within the chunk.  Every batch issues the
    // same number of loads whatever `it` is -- rows past the end are clamped to the last row and later
    // multiplied by p = 0 -- so the compiler can wait for exactly the batch it consumes and leave the younger
    // ones in flight (loads under a condition would force it to drain the whole queue at every merge point).
    // last cached row of the chunk for rows past it (with APPEND a chunk may hold no cached row at all: row 0 then)
    auto clamp_row = [&](int row) { return APPEND ? max(min(row, n - 1), 0) : min(row, n - 1); };
    auto request_v = [&](Batch &bt, int it) {
        const int r0 = (it * NW + w) * TL::BATCH + rg;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            bt.v[u] = stream16(vbase + ((unsigned int)clamp_row(r0 + u * TL::RPW) * TL::ROW_BYTES + lane_off));
    };
#pragma unroll
    for (int j = 0; j < NB; ++j) request_v(buf[j], j);

    const int c = IDENT ? h : min(max(h2c[(size_t)b * H + h], 0), k - 1);
    const size_t crow = (size_t)b * k + c;
    const float *srow = scores + crow * T + t0;
    float *prow = nullptr;
    if (WRITE_P) prow = (probs_out != nullptr && dpart == 0 && (IDENT || rep[crow] == h)) ? probs_out + crow * T + t0 : nullptr;

    // the score this lane turns into a probability for batch `it` (lanes >= BATCH and rows past the end: none;
    // they still issue the load, of the last score, to keep the count fixed)
    auto request_s = [&](Batch &bt, int it) {
        const int tl = (it * NW + w) * TL::BATCH + lane;
        bt.s = srow[clamp_row(tl)];           // masked when it is consumed
        if (DT == DT_E4M3) bt.vs = vsrow[clamp_row(tl)];
    };
#pragma unroll
    for (int j = 0; j < NB; ++j) request_s(buf[j], j);

    const float2 *st = stats + crow * n_rec;
    float m = -INFINITY;
    for (int i = lane; i < n_rec; i += 64) m = fmaxf(m, st[i].x);
    const float M = wave_max(m);
    float l = 0.f;
    for (int i = lane; i < n_rec; i += 64) l += st[i].y * expf(st[i].x - M);
    const float inv = 1.0f / wave_sum(l);

    float acc[TL::EPL];
#pragma unroll
    for (int e = 0; e < TL::EPL; ++e) acc[e] = 0.f;

    auto consume = [&](const Batch &bt, int it) {
        // probabilities of this batch: lane i < BATCH owns row i of the batch; slot rg*kUnroll + u holds the
        // row that lane group rg multiplies with its load u, so a lane reads kUnroll consecutive floats
        const int tl = (it * NW + w) * TL::BATCH + lane;
        const float p = tl < n ? expf(bt.s - M) * inv : 0.f;          // rows past the end weigh nothing
        if (lane < TL::BATCH) {
            // a quantised row's scale rides on its probability: p * (scale * code) = (p * scale) * code
            p_lds[w][(lane % TL::RPW) * kUnroll + lane / TL::RPW] = DT == DT_E4M3 ? p * bt.vs : p;
            if (WRITE_P) {
                if (prow != nullptr && tl < n) prow[tl] = p;
            }
        }
        __builtin_amdgcn_wave_barrier();
        float pv[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) pv[u] = p_lds[w][rg * kUnroll + u];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            float f[TL::EPL];
            unpack(bt.v[u], f);
#pragma unroll
            for (int e = 0; e < TL::EPL; ++e) acc[e] = fmaf(pv[u], f[e], acc[e]);
        }
    };

    // NB batches are in flight; a buffer is refilled as soon as it has been consumed.  The trip count is
    // rounded up to a multiple of NB: the surplus batches lie past the end and contribute p = 0.
    for (int it0 = 0; it0 < n_it; it0 += NB) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            consume(buf[j], it0 + j);
            request_v(buf[j], it0 + j + NB);
            request_s(buf[j], it0 + j + NB);
        }
    }

    if (APPEND) {
        if (has_new && w == 0 && rg == 0) {      // one lane group: the new value row of this head
            const u32x4 nraw = *reinterpret_cast<const u32x4 *>(v_new + ((size_t)b * H + h) * TL::ROW_BYTES + lane_off);
            const float p = expf(srow[n] - M) * inv;
            float f[TL::EPL];
            unpack(nraw, f);
#pragma unroll
            for (int e = 0; e < TL::EPL; ++e) acc[e] = fmaf(p, f[e], acc[e]);
            *reinterpret_cast<u32x4 *>(const_cast<char *>(vbase) + ((unsigned int)n * TL::ROW_BYTES + lane_off)) = nraw;
        }
    }

    // lane groups of a wave, then the waves
#pragma unroll
    for (int e = 0; e < TL::EPL; ++e) {
#pragma unroll
        for (int o = TL::LPR; o < 64; o <<= 1) acc[e] += __shfl_xor(acc[e], o);
    }
    if (rg == 0) {
#pragma unroll
        for (int e = 0; e < TL::EPL; ++e) acc_lds[w][cg * TL::EPL + e] = acc[e];
    }
    __syncthreads();
    if (tid < TL::COLS) {
        float val = 0.f;
#pragma unroll
        for (int i = 0; i < NW; ++i) val += acc_lds[i][tid];
        const size_t orow = (size_t)b * H + h;
        const int col = dpart * TL::COLS + tid;
        if (n_cp == 1) out[orow * kHeadDim + col] = val;
        else partial[(orow * n_cp + split) * kHeadDim + col] = val;     // combine_kernel adds the rows up
    }
}

template <int DT, bool IDENT, int NW, int NB, bool WRITE_P, bool APPEND, int DS>
__global__ __launch_bounds__(NW * 64) void value_kernel(const char *__restrict__ v,
                                                        const int32_t *__restrict__ h2c,
                                                        const int32_t *__restrict__ rep, int H, int k, int T,
                                                        int T_cap, int n_rec, int cp, int n_cp,
                                                        const float *__restrict__ scores,
                                                        const float2 *__restrict__ stats,
                                                        float *__restrict__ partial, float *__restrict__ out,
                                                        float *__restrict__ probs_out,
                                                        const char *__restrict__ v_new,
                                                        const float *__restrict__ vscale)
{
    value_block<DT, IDENT, NW, NB, WRITE_P, APPEND, DS>(v, h2c, rep, H, k, T, T_cap, n_rec, cp, n_cp, scores, stats,
                                                        partial, out, probs_out, v_new, vscale, blockIdx.x, blockIdx.y,
                                                        blockIdx.z);
}

// ---------------------------------------------------------------------------------------------------------
// Score kernel: s[b][j][t] = scale * q[b][rep(b,j)] . Kc[b][j][t], plus (max, sum of exp) records for the value
// kernel's exact merge.  grid = (n_cs, k, B): a workgroup takes a chunk of cs tokens of one cluster's key stream.
//
// A wave owns every NW-th batch of BATCH consecutive rows of its chunk, keeps NB batches in flight and refills a
// buffer right after it has consumed it.  After the 16-lane row sums every lane of a lane group holds the dot
// products of the group's kUnroll rows; lane cg < kUnroll keeps the one of load u = cg, so the first kUnroll lanes
// of every group own one score each (row rg + cg * RPW of the batch): BATCH scores per wave, written as one
// 128-byte (bf16 rows) piece of the score row.  The softmax statistics are carried per lane (running maximum and
// sum of exponentials over the scores the lane has seen) and reduced once over the wave at the end: one
// (max, sum-exp) record per wave (n_cs * NW per cluster), no workgroup barrier anywhere, no LDS.
// APPEND: the last position, T-1, is the token being decoded: its key is not in the cache yet.  The workgroup of
// the last chunk takes it from k_new [B,H,d] (row of the representative), scores it, and writes it to the cache,
// so that growing the cache costs no launch of its own.
// ---------------------------------------------------------------------------------------------------------
template <int DT, bool IDENT, bool APPEND, int NW, int NB>
__global__ __launch_bounds__(NW * 64) void score_kernel(const char *__restrict__ q, const char *__restrict__ kc,
                                                        const int32_t *__restrict__ rep, int H, int k, int T,
                                                        int Tc_cap, float scale, int cs, int n_cs,
                                                        float *__restrict__ scores, float2 *__restrict__ stats,
                                                        const char *__restrict__ k_new,
                                                        const float *__restrict__ kscale, int q_dtype)
{
    using TL = Tile<DT>;
    static_assert(!(APPEND && DT == DT_E4M3), "quantised caches grow through their own append kernel");
    const int chunk = blockIdx.x, j = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x;
    const int lane = tid & 63, w = tid >> 6;
    const int cg = lane % TL::LPR, rg = lane / TL::LPR;
    const int t0 = chunk * cs;
    const int n_all = min(T, t0 + cs) - t0;                   // >= 1 by construction of n_cs
    const bool has_new = APPEND && chunk == n_cs - 1;         // this chunk ends with the token being decoded
    const int n = has_new ? n_all - 1 : n_all;                // rows that are in the cache already (may be 0)
    const int n_batches = (n + TL::BATCH - 1) / TL::BATCH;
    const int n_it = n_batches > w ? (n_batches - w + NW - 1) / NW : 0;

    const char *kbase = kc + (((size_t)b * k + j) * Tc_cap + t0) * TL::ROW_BYTES;
    const unsigned int lane_off = cg * 16;
    u32x4 buf[NB][kUnroll];
    float ks_buf[NB];                        // rows of 8-bit codes: the scale of the row this lane will own
    const float *ksrow = DT == DT_E4M3 ? kscale + ((size_t)b * k + j) * Tc_cap + t0 : nullptr;
    auto clamp_row = [&](int row) { return APPEND ? max(min(row, n - 1), 0) : min(row, n - 1); };
    auto request = [&](u32x4 (&bt)[kUnroll], float &ks, int it) {
        const int r0 = (it * NW + w) * TL::BATCH + rg;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
            bt[u] = stream16(kbase + ((unsigned int)clamp_row(r0 + u * TL::RPW) * TL::ROW_BYTES + lane_off));
        if (DT == DT_E4M3) ks = ksrow[clamp_row(r0 + cg * TL::RPW)];
    };
#pragma unroll
    for (int i = 0; i < NB; ++i) request(buf[i], ks_buf[i], i);

    int r = IDENT ? j : rep[(size_t)b * k + j];
    if (r < 0) return;                       // unused cluster slot (same decision for every wave of the chunk)
    r = min(r, H - 1);
    float qf[TL::EPL];
    if (DT == DT_E4M3) {
        // the query is not quantised: fp32 or bf16 (q_dtype), elements cg*16 .. cg*16+15 for this lane
        const char *qrow = q + ((size_t)b * H + r) * (size_t)(kHeadDim * (q_dtype == CHAI_BF16 ? 2 : 4));
        if (q_dtype == CHAI_BF16) {
#pragma unroll
            for (int part = 0; part < 2; ++part) {
                float f8[8];
                unpack(*reinterpret_cast<const u32x4 *>(qrow + cg * 32 + part * 16), f8);
#pragma unroll
                for (int e = 0; e < 8; ++e) qf[(part * 8 + e) % TL::EPL] = f8[e];
            }
        } else {
#pragma unroll
            for (int part = 0; part < 4; ++part) {
                float f4[4];
                unpack(*reinterpret_cast<const u32x4 *>(qrow + cg * 64 + part * 16), f4);
#pragma unroll
                for (int e = 0; e < 4; ++e) qf[(part * 4 + e) % TL::EPL] = f4[e];
            }
        }
    } else {
        const u32x4 qraw = *reinterpret_cast<const u32x4 *>(q + ((size_t)b * H + r) * TL::ROW_BYTES + lane_off);
        unpack(qraw, qf);
    }
    float *srow = scores + ((size_t)b * k + j) * T + t0;
    float m_run = -INFINITY, l_run = 0.f;
    // The stored score is the ROUNDED product: the statistics below and the value kernel must both start from
    // that value (a multiply fused into the subtraction of the running maximum would use the unrounded one,
    // and with scores of magnitude 10^3 the difference reaches 1e-4 of a probability).
    auto scaled = [&](float x, float row_scale) {
#pragma clang fp contract(off)
        return DT == DT_E4M3 ? (scale * row_scale) * x : scale * x;
    };
    auto see = [&](float sv) {               // running softmax statistics of this lane
        const float m_new = fmaxf(m_run, sv);
        l_run = l_run * __expf(m_run - m_new) + __expf(sv - m_new);
        m_run = m_new;
    };

    for (int it0 = 0; it0 < n_it; it0 += NB) {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int it = it0 + i;
            float mine = 0.f;
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                float f[TL::EPL];
                unpack(buf[i][u], f);
                float dot = 0.f;
#pragma unroll
                for (int e = 0; e < TL::EPL; ++e) dot = fmaf(qf[e], f[e], dot);
                dot = row_sum<DT>(dot);
                mine = cg == u ? dot : mine;
            }
            const float ks = DT == DT_E4M3 ? ks_buf[i] : 1.f;
            request(buf[i], ks_buf[i], it + NB);
            const int tl = (it * NW + w) * TL::BATCH + rg + cg * TL::RPW;
            if (cg < kUnroll && tl < n) {
                const float sv = scaled(mine, ks);
                srow[tl] = sv;
                see(sv);
            }
        }
    }
    if (APPEND) {
        if (has_new && w == 0 && rg == 0) {      // one lane group: the new key row of the representative
            const u32x4 nraw = *reinterpret_cast<const u32x4 *>(k_new + ((size_t)b * H + r) * TL::ROW_BYTES + lane_off);
            float f[TL::EPL];
            unpack(nraw, f);
            float dot = 0.f;
#pragma unroll
            for (int e = 0; e < TL::EPL; ++e) dot = fmaf(qf[e], f[e], dot);
            dot = row_sum<DT>(dot);
            if (cg == 0) {
                const float sv = scaled(dot, 1.f);
                srow[n] = sv;
                see(sv);
            }
            *reinterpret_cast<u32x4 *>(const_cast<char *>(kbase) + ((unsigned int)n * TL::ROW_BYTES + lane_off)) = nraw;
        }
    }
    // one record per wave: lanes without scores carry (-inf, 0) and drop out of the merge
    const float M = wave_max(m_run);
    const float L = wave_sum(m_run == -INFINITY ? 0.f : l_run * __expf(m_run - M));
    if (lane == 0) {
        stats[((size_t)b * k + j) * ((size_t)n_cs * NW) + (size_t)chunk * NW + w] = make_float2(M, L);
    }
}

// Sum of the partial rows of every head in chunk order.  grid = (B*H), 128 threads.
__global__ __launch_bounds__(kHeadDim) void combine_kernel(const float *__restrict__ partial, int n_cp,
                                                           float *__restrict__ out)
{
    const size_t orow = blockIdx.x;
    float sum = 0.f;
    for (int s = 0; s < n_cp; ++s) sum += partial[(orow * n_cp + s) * kHeadDim + threadIdx.x];
    out[orow * kHeadDim + threadIdx.x] = sum;
}

// Shared-value variant: the streams are compact (one per cluster); head h of n_heads takes the sum of the
// partial rows of its cluster's stream.  grid = (n_heads, B), 128 threads.
__global__ __launch_bounds__(kHeadDim) void combine_members_kernel(const float *__restrict__ partial, int n_cp,
                                                                   const int32_t *__restrict__ h2c, int n_heads, int k,
                                                                   float *__restrict__ out)
{
    const int h = blockIdx.x, b = blockIdx.y;
    const int c = h2c[(size_t)b * n_heads + h];
    if (c < 0 || c >= k) return;
    const size_t srow = (size_t)b * k + c;
    float sum = 0.f;
    for (int s = 0; s < n_cp; ++s) sum += partial[(srow * n_cp + s) * kHeadDim + threadIdx.x];
    out[((size_t)b * n_heads + h) * kHeadDim + threadIdx.x] = sum;
}

struct Workspace {
    float *scores;
    float2 *stats;
    float *partial;
    Workspace(void *base, const DecodePlan &pl)
    {
        char *ws = static_cast<char *>(base);
        scores = reinterpret_cast<float *>(ws + pl.off_scores);
        stats = reinterpret_cast<float2 *>(ws + pl.off_stats);
        partial = reinterpret_cast<float *>(ws + pl.off_partial);
    }
};

// Launches carry the optional pair of events that the runtime stamps with the begin and the end of the kernel
// itself (both NULL for an ordinary launch), for callers who profile.
template <int DT, bool IDENT>
int scores_typed(const void *q, const void *kc, const int32_t *rep, int B, int H, int k, int T, int Tc_cap,
                 float scale, const Workspace &w, const DecodePlan &pl, const KernelEvents &ev, hipStream_t stream,
                 const void *k_new, const float *kscale = nullptr, int q_dtype = DT)
{
    const dim3 grid(pl.n_cs, k, B), block(kScoreWaves * 64);
    const char *qc = static_cast<const char *>(q), *kcc = static_cast<const char *>(kc);
    if constexpr (DT != DT_E4M3) {
        if (!IDENT && k_new != nullptr)
            return (int)launch_kernel(score_kernel<DT, false, true, kScoreWaves, kScoreBatches>, grid, block, 0, stream,
                                      ev, qc, kcc, rep, H, k, T, Tc_cap, scale, pl.cs, pl.n_cs, w.scores, w.stats,
                                      static_cast<const char *>(k_new), nullptr, q_dtype);
    }
    return (int)launch_kernel(score_kernel<DT, IDENT, false, kScoreWaves, kScoreBatches>, grid, block, 0, stream, ev, qc,
                              kcc, rep, H, k, T, Tc_cap, scale, pl.cs, pl.n_cs, w.scores, w.stats, nullptr, kscale,
                              q_dtype);
}

// A merge of the partial rows inside the value kernel (last workgroup of a head, found through a device-scope
// arrival counter) was measured and dropped: with __threadfence() in every workgroup the kernel ran 10x slower
// (L2 write-back + invalidate per fence across 8 XCDs), and with fence-free device-scope stores/loads it was
// still slower than the separate combine launch at every chunk count tried.  So was a single launch of both
// phases (score workgroups first in the grid, value workgroups prefetching V and waiting on per-cluster
// device-scope counters): 67 us against 55 us per LLaMa-7B layer -- cross-XCD flag traffic costs more than the
// 2.5 us of a second launch.  A third design -- one workgroup per (cluster, chunk of 128 tokens) that scores the
// chunk, keeps exp(s - chunk max) in LDS and streams the chunk of every member's values, with a rescaling merge of
// per-chunk partial rows as the only second launch -- needs no cross-workgroup wait at all and was slower still
// (71 against 55 us per LLaMa-7B layer, 306 against 181 us at 32k tokens): thousands of short workgroups, each
// with a dependent start-up chain (membership row -> member list -> values; keys -> scores -> two barriers), do
// not stream like one long workgroup per head.
template <int DT, bool IDENT, int NW, int NB, int DS>
int values_launch(const void *v, const int32_t *h2c, const int32_t *rep, int B, int H, int k, int T, int T_cap,
                  float *out, float *probs_out, const Workspace &w, const DecodePlan &pl, const KernelEvents &ev,
                  hipStream_t stream, const MemberRows *members, const void *v_new, const float *vscale = nullptr)
{
    // the copy of the probabilities (tests, inspection) lives in an instantiation of its own so that the
    // production kernel has no store inside its streaming loop; so does the variant that appends the new token
    const dim3 grid(pl.n_cp, H * DS, B), block(NW * 64);
    const char *vc = static_cast<const char *>(v);
    hipError_t e = hipSuccess;
    bool launched = false;
    if constexpr (DT != DT_E4M3) {
        if (!IDENT && v_new != nullptr) {
            e = launch_kernel(value_kernel<DT, false, NW, NB, false, true, DS>, grid, block, 0, stream, ev, vc, h2c, rep, H,
                              k, T, T_cap, pl.n_rec, pl.cp, pl.n_cp, w.scores, w.stats, w.partial, out, probs_out,
                              static_cast<const char *>(v_new), nullptr);
            launched = true;
        }
    }
    if (launched) {
    } else if (probs_out != nullptr)
        e = launch_kernel(value_kernel<DT, IDENT, NW, NB, true, false, DS>, grid, block, 0, stream, ev, vc, h2c, rep, H, k,
                          T, T_cap, pl.n_rec, pl.cp, pl.n_cp, w.scores, w.stats, w.partial, out, probs_out, nullptr,
                          vscale);
    else
        e = launch_kernel(value_kernel<DT, IDENT, NW, NB, false, false, DS>, grid, block, 0, stream, ev, vc, h2c, rep, H,
                          k, T, T_cap, pl.n_rec, pl.cp, pl.n_cp, w.scores, w.stats, w.partial, out, probs_out, nullptr,
                          vscale);
    if (e != hipSuccess) return (int)e;
    if (members != nullptr)
        // one launch both adds the partial rows (n_cp = 1: the staged row itself) and hands them to the members
        return (int)launch_kernel(combine_members_kernel, dim3(members->n_heads, B), dim3(kHeadDim), 0, stream,
                                  KernelEvents(), pl.n_cp == 1 ? out : w.partial, pl.n_cp, members->head_to_cluster,
                                  members->n_heads, H, members->out_members);
    if (pl.n_cp == 1) return (int)hipSuccess;
    return (int)launch_kernel(combine_kernel, dim3(B * H), dim3(kHeadDim), 0, stream, KernelEvents(), w.partial, pl.n_cp,
                              out);
}

template <int DT, bool IDENT>
int values_typed(const void *v, const int32_t *h2c, const int32_t *rep, int B, int H, int k, int T, int T_cap,
                 float *out, float *probs_out, const Workspace &w, const DecodePlan &pl, const KernelEvents &ev,
                 hipStream_t stream, const MemberRows *members, const void *v_new, const float *vscale = nullptr)
{
    if constexpr (DT == DT_E4M3) {
        // rows of 8-bit codes are one cache line: no column split (the plan is made without it)
        if (pl.cp >= 4096)
            return values_launch<DT, IDENT, 4, 2, 1>(v, h2c, rep, B, H, k, T, T_cap, out, probs_out, w, pl, ev, stream, members, v_new, vscale);
        return values_launch<DT, IDENT, 8, 1, 1>(v, h2c, rep, B, H, k, T, T_cap, out, probs_out, w, pl, ev, stream, members, v_new, vscale);
    } else {
    // Workgroup shape (measured on MI355X): eight waves with one batch in flight each are 1-6 % faster than
    // four waves with two batches up to a few thousand tokens per workgroup; on long chunks four waves with
    // two batches are ~1.5 % ahead.
    const bool long_chunks = pl.cp >= 4096;
    if (pl.ds == 2) {
        if (long_chunks)
            return values_launch<DT, IDENT, 4, 2, 2>(v, h2c, rep, B, H, k, T, T_cap, out, probs_out, w, pl, ev, stream, members, v_new);
        return values_launch<DT, IDENT, 8, 1, 2>(v, h2c, rep, B, H, k, T, T_cap, out, probs_out, w, pl, ev, stream, members, v_new);
    }
    if (long_chunks)
        return values_launch<DT, IDENT, 4, 2, 1>(v, h2c, rep, B, H, k, T, T_cap, out, probs_out, w, pl, ev, stream, members, v_new);
    return values_launch<DT, IDENT, 8, 1, 1>(v, h2c, rep, B, H, k, T, T_cap, out, probs_out, w, pl, ev, stream, members, v_new);
    }
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

DecodePlan make_decode_plan(int B, int H, int k, int T, bool column_split)
{
    DecodePlan pl;
    // Score chunk (measured on MI355X on the LLaMa-7B/33B, OPT-66B and 32k-context shapes): the largest of
    // 2048/1024/512 tokens that still gives one workgroup per CU; smaller problems take 256 (one round of the
    // workgroup's waves with both batches in flight).
    pl.cs = 256;
    for (int c : {2048, 1024, 512}) {
        if ((long long)B * k * ((T + c - 1) / c) >= 256) { pl.cs = c; break; }
    }
    // value chunk (measured on MI355X at T = 2048): with >= 384 heads one workgroup per head -- whole row of
    // the cache, no partial rows, no combine launch -- is fastest (416 heads: 39 us against 41-44 us split);
    // with fewer heads the single workgroups become latency-bound and the tokens are split into >= 1024
    // workgroups whose partial rows a combine launch adds up (288 heads: 30 us with 4 chunks against 34 us
    // unsplit).  Between 192 and 383 heads and up to 1536 tokens, two workgroups per head that take half of the
    // columns each do better still: enough workgroups without partial rows and without the combine launch
    // (288 heads: 18.6 against 21.7 us at 640 tokens, 23.0 against 24.3 at 1024, 30.3 against 30.8 at 1536; at
    // 2048 the token split is 3 % ahead again).
    {
        const long long heads = (long long)B * H > 0 ? (long long)B * H : 1;
        pl.ds = (column_split && heads >= 192 && heads < 384 && T <= 1536) ? 2 : 1;
        const long long groups = heads * pl.ds;
        long long want = groups >= 384 ? 1 : (1024 + groups - 1) / groups;
        const long long most = (T + 127) / 128;
        if (want > most) want = most;
        pl.cp = (int)(((T + want - 1) / want + 127) / 128 * 128);
    }
    pl.n_cs = (T + pl.cs - 1) / pl.cs;
    pl.n_rec = pl.n_cs * kScoreWaves;
    pl.n_cp = (T + pl.cp - 1) / pl.cp;

    // Region sizes are upper bounds over every chunking the rules above can pick (smallest chunks), so the
    // total grows monotonically with T: a workspace sized for the cache capacity serves every shorter context.
    const size_t max_n_rec = (size_t)(T + 255) / 256 * kScoreWaves, max_n_cp = (size_t)(T + 127) / 128;
    size_t off = 0;
    pl.off_scores = off;  off = align_up(off + (size_t)B * k * T * sizeof(float), 256);
    pl.off_stats = off;   off = align_up(off + (size_t)B * k * max_n_rec * sizeof(float2), 256);
    pl.off_partial = off; off = align_up(off + (size_t)B * H * max_n_cp * kHeadDim * sizeof(float), 256);
    pl.off_rows = off;    off = align_up(off + (size_t)B * H * kHeadDim * sizeof(float), 256);
    pl.bytes = off;
    return pl;
}

int launch_scores(const void *q, const void *kc, const int32_t *rep, int B, int H, int k, int T, int Tc_cap, int dtype,
                  float scale, void *workspace, const DecodePlan &plan, bool identity, const KernelEvents &ev,
                  hipStream_t stream, const void *k_new)
{
    const Workspace w(workspace, plan);
    if (dtype == CHAI_BF16)
        return identity ? scores_typed<DT_BF16, true>(q, kc, rep, B, H, k, T, Tc_cap, scale, w, plan, ev, stream, k_new)
                        : scores_typed<DT_BF16, false>(q, kc, rep, B, H, k, T, Tc_cap, scale, w, plan, ev, stream, k_new);
    return identity ? scores_typed<DT_F32, true>(q, kc, rep, B, H, k, T, Tc_cap, scale, w, plan, ev, stream, k_new)
                    : scores_typed<DT_F32, false>(q, kc, rep, B, H, k, T, Tc_cap, scale, w, plan, ev, stream, k_new);
}

int launch_values(const void *v, const int32_t *h2c, const int32_t *rep, int B, int H, int k, int T, int T_cap,
                  int dtype, float *out, float *probs_out, void *workspace, const DecodePlan &plan, bool identity,
                  const KernelEvents &ev, hipStream_t stream, const MemberRows *members, const void *v_new)
{
    const Workspace w(workspace, plan);
    if (dtype == CHAI_BF16)
        return identity ? values_typed<DT_BF16, true>(v, h2c, rep, B, H, k, T, T_cap, out, probs_out, w, plan, ev, stream,
                                                      members, v_new)
                        : values_typed<DT_BF16, false>(v, h2c, rep, B, H, k, T, T_cap, out, probs_out, w, plan, ev,
                                                       stream, members, v_new);
    return identity ? values_typed<DT_F32, true>(v, h2c, rep, B, H, k, T, T_cap, out, probs_out, w, plan, ev, stream,
                                                 members, v_new)
                    : values_typed<DT_F32, false>(v, h2c, rep, B, H, k, T, T_cap, out, probs_out, w, plan, ev, stream,
                                                  members, v_new);
}

int launch_scores_q8(const void *q, int q_dtype, const void *k8, const float *kscale, const int32_t *rep, int B, int H,
                     int k, int T, int Tc_cap, float scale, void *workspace, const DecodePlan &plan,
                     const KernelEvents &ev, hipStream_t stream)
{
    const Workspace w(workspace, plan);
    return scores_typed<DT_E4M3, false>(q, k8, rep, B, H, k, T, Tc_cap, scale, w, plan, ev, stream, nullptr, kscale,
                                        q_dtype);
}

int launch_values_q8(const void *v8, const float *vscale, const int32_t *h2c, const int32_t *rep, int B, int H, int k,
                     int T, int T_cap, float *out, float *probs_out, void *workspace, const DecodePlan &plan,
                     const KernelEvents &ev, hipStream_t stream)
{
    const Workspace w(workspace, plan);
    return values_typed<DT_E4M3, false>(v8, h2c, rep, B, H, k, T, T_cap, out, probs_out, w, plan, ev, stream, nullptr,
                                        nullptr, vscale);
}

}  // namespace chai
