// Clustered-head attention over a block of prompt positions (the prefill that follows the membership decision;
// Section 3.5, attention definition of Section 2 with the causal mask of a decoder-only model).  Many query rows
// per key make this the one compute-bound step of the method, so it runs on the matrix cores: a flash-style
// kernel (scores, online softmax and output accumulation tile by tile, nothing T x T ever leaves the chip) in
// which the score tile of a cluster is computed ONCE from the representative's queries and keys and then applied
// to the values of up to kGroup member heads -- the saving the method is about.
//
// MFMA tiles (v_mfma_f32_32x32x16, wave64), lane l = (r = l % 32, hl = l / 32):
//   A[32][16]: lane holds A[r][8*hl .. 8*hl+7]     B[16][32]: lane holds B[8*hl .. 8*hl+7][r]
//   D[32][32]: lane holds D[(v/4)*8 + hl*4 + v%4][r] for v = 0..15
// Scores are computed transposed, S^T = K_tile Q^T (bf16 inputs): a lane then owns ONE query column and 16 of
// the 32 keys of the tile, so row maxima and sums are in-lane plus one exchange with lane l^32, and the tile of
// probabilities is already in the B-operand layout of O^T += V^T P^T.  That second product runs in fp16 (P in
// [0,1] keeps 11 bits instead of bf16's 8; V is widened exactly from bf16 while it is transposed into LDS, so
// values must stay inside the fp16 range, |v| <= 65504).
#include "chai_internal.h"

namespace chai {

namespace {

constexpr int kGroup = 2;          // member heads that share one score tile inside a workgroup
constexpr int kQWave = 32;         // query rows per wave
constexpr int kPWaves = 4;         // waves per workgroup
constexpr int kQTile = kQWave * kPWaves;   // 128 query rows per workgroup
constexpr int kKTile = 32;         // keys per tile
constexpr int kVtStride = 40;      // halves per row of the transposed V tile in LDS (32 + 8 of padding)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

union Frag16 {            // 16 bytes seen as a raw load, bf16 x 8 or fp16 x 8
    u32x4 raw;
    bf16x8 bf;
    f16x8 h;
};

// position inside a 32-key LDS row of key jj, so that lane half hl finds the 8 keys of MFMA step s that match
// its probability registers (keys 16s + (e/4)*8 + hl*4 + e%4, e = 0..7) in 8 consecutive halves
__device__ __forceinline__ int key_slot(int jj)
{
    const int s = jj >> 4, r = jj & 15;
    return 16 * s + 8 * ((r & 7) >> 2) + 4 * (r >> 3) + (r & 3);
}

// ---------------------------------------------------------------------------------------------------------
// Work list: the heads of every cluster, in ascending order, cut into groups of at most kGroup.  One thread
// per batch row (H <= a few hundred).  groups[b][g] = {cluster, n, head_0 .. head_{kGroup-1}}.
// ---------------------------------------------------------------------------------------------------------
__global__ void prefill_plan_kernel(const int32_t *__restrict__ h2c, const int32_t *__restrict__ rep, int H, int k,
                                    int max_groups, int32_t *__restrict__ groups, int32_t *__restrict__ n_groups)
{
    const int b = blockIdx.x;
    if (threadIdx.x != 0) return;
    int32_t *g = groups + (size_t)b * max_groups * (2 + kGroup);
    int ng = 0;
    for (int j = 0; j < k; ++j) {
        if (rep[(size_t)b * k + j] < 0) continue;
        int n = 0;
        for (int h = 0; h < H; ++h) {
            if (h2c[(size_t)b * H + h] != j) continue;
            if (n == 0 && ng < max_groups) { g[ng * (2 + kGroup)] = j; }
            if (ng < max_groups) g[ng * (2 + kGroup) + 2 + n] = h;
            if (++n == kGroup) {
                if (ng < max_groups) g[ng * (2 + kGroup) + 1] = n;
                ++ng;
                n = 0;
            }
        }
        if (n > 0) {
            if (ng < max_groups) g[ng * (2 + kGroup) + 1] = n;
            ++ng;
        }
    }
    n_groups[b] = ng < max_groups ? ng : max_groups;
}

// ---------------------------------------------------------------------------------------------------------
// grid (query tiles [largest first], max_groups, B), 256 threads.  IDENT: every head is its own cluster
// (dense attention); the work list is not read.
// ---------------------------------------------------------------------------------------------------------
template <bool IDENT>
__global__ __launch_bounds__(kPWaves * 64) void prefill_kernel(const char *__restrict__ q, const char *__restrict__ kc,
                                                               const char *__restrict__ v,
                                                               const int32_t *__restrict__ rep,
                                                               const int32_t *__restrict__ groups,
                                                               const int32_t *__restrict__ n_groups, int H, int k,
                                                               int Tq, int q_start, int Tc_cap, int T_cap,
                                                               int max_groups, float scale, float *__restrict__ out)
{
    __shared__ _Float16 vt[kGroup][kHeadDim][kVtStride];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r = lane & 31, hl = lane >> 5;
    const int qt = gridDim.x - 1 - blockIdx.x, gi = blockIdx.y, b = blockIdx.z;

    int cluster, n_mem, heads[kGroup];
    if (IDENT) {
        if (gi >= H) return;
        cluster = gi; n_mem = 1; heads[0] = gi;
#pragma unroll
        for (int g = 1; g < kGroup; ++g) heads[g] = gi;
    } else {
        if (gi >= n_groups[b]) return;
        const int32_t *gr = groups + ((size_t)b * max_groups + gi) * (2 + kGroup);
        cluster = gr[0];
        n_mem = min(max(gr[1], 1), kGroup);
#pragma unroll
        for (int g = 0; g < kGroup; ++g) heads[g] = min(max(gr[2 + min(g, n_mem - 1)], 0), H - 1);
    }
    const int rhead = IDENT ? cluster : min(max(rep[(size_t)b * k + cluster], 0), H - 1);

    const int i0 = qt * kQTile + w * kQWave;                 // first query row of this wave (relative)
    const int my_i = i0 + r;                                 // this lane's query row
    const int q_abs = q_start + min(my_i, Tq - 1);           // its sequence position (clamped for padding rows)
    const int wave_last = q_start + min(i0 + kQWave - 1, Tq - 1);     // last position any lane of the wave sees
    const int wg_last = q_start + min(qt * kQTile + kQTile - 1, Tq - 1);
    const int n_tiles = wg_last / kKTile + 1;                // key tiles 0 .. n_tiles-1 cover positions <= wg_last
    const bool wave_active = i0 < Tq;

    // query fragments (B operand of S^T = K Q^T): Q[my_i][16*ks + 8*hl .. +7]
    Frag16 qf[kHeadDim / 16];
    {
        const char *qrow = q + (((size_t)b * H + rhead) * Tq + min(my_i, Tq - 1)) * (kHeadDim * 2) + hl * 16;
#pragma unroll
        for (int ks = 0; ks < kHeadDim / 16; ++ks) qf[ks].raw = *reinterpret_cast<const u32x4 *>(qrow + ks * 32);
    }
    const char *kbase = kc + ((size_t)b * k + cluster) * (size_t)Tc_cap * (kHeadDim * 2) + hl * 16;

    f32x16 acc[kGroup][kHeadDim / 32];
#pragma unroll
    for (int g = 0; g < kGroup; ++g)
#pragma unroll
        for (int blk = 0; blk < kHeadDim / 32; ++blk)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[g][blk][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    for (int kt = 0; kt < n_tiles; ++kt) {
        const int key0 = kt * kKTile;
        __syncthreads();                        // everyone is done reading the previous V tile
        // V tiles of the member heads -> LDS, transposed, widened to fp16.  512 pieces of 16 bytes per head.
#pragma unroll
        for (int g = 0; g < kGroup; ++g) {
            if (g < n_mem) {
                const char *vhead = v + ((size_t)b * H + heads[g]) * (size_t)T_cap * (kHeadDim * 2);
#pragma unroll
                for (int pp = 0; pp < 2; ++pp) {
                    const int piece = tid + pp * 256, jj = piece >> 4, c8 = piece & 15;
                    Frag16 x;
                    x.raw = *reinterpret_cast<const u32x4 *>(vhead + (size_t)min(key0 + jj, wg_last) * (kHeadDim * 2) +
                                                             c8 * 16);
                    const int slot = key_slot(jj);
#pragma unroll
                    for (int e = 0; e < 8; ++e) vt[g][c8 * 8 + e][slot] = (_Float16)(float)x.bf[e];
                }
            }
        }
        __syncthreads();
        if (!wave_active || key0 > wave_last) continue;     // uniform per wave; barriers above are always reached

        // S^T tile: 32 keys x 32 queries
        f32x16 st;
#pragma unroll
        for (int e = 0; e < 16; ++e) st[e] = 0.f;
        {
            const char *krow = kbase + (size_t)min(key0 + r, wg_last) * (kHeadDim * 2);
#pragma unroll
            for (int ks = 0; ks < kHeadDim / 16; ++ks) {
                Frag16 kf;
                kf.raw = *reinterpret_cast<const u32x4 *>(krow + ks * 32);
                st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf.bf, qf[ks].bf, st, 0, 0, 0);
            }
        }
        // scale, causal mask, online softmax for this lane's query column
        float mx = -INFINITY;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int key = key0 + (e >> 2) * 8 + hl * 4 + (e & 3);
            const float sv = key <= q_abs ? st[e] * scale : -INFINITY;
            st[e] = sv;
            mx = fmaxf(mx, sv);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);               // finite: tile 0 always holds key 0 <= q_abs
        const float alpha = __expf(m_run - m_new);
        float rs = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float p = __expf(st[e] - m_new);
            st[e] = p;
            rs += p;
        }
        rs += __shfl_xor(rs, 32);
        l_run = l_run * alpha + rs;
        m_run = m_new;
        Frag16 pf[2];
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[s].h[e] = (_Float16)st[8 * s + e];

        // O^T[d][query] = alpha * O^T + V^T P^T for every member head
#pragma unroll
        for (int g = 0; g < kGroup; ++g) {
            if (g < n_mem) {
#pragma unroll
                for (int blk = 0; blk < kHeadDim / 32; ++blk) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[g][blk][e] *= alpha;
#pragma unroll
                    for (int s = 0; s < 2; ++s) {
                        Frag16 vf;
                        vf.raw = *reinterpret_cast<const u32x4 *>(&vt[g][blk * 32 + r][16 * s + 8 * hl]);
                        acc[g][blk] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf.h, pf[s].h, acc[g][blk], 0, 0, 0);
                    }
                }
            }
        }
    }

    if (!wave_active || my_i >= Tq) return;
    const float inv = 1.0f / l_run;
#pragma unroll
    for (int g = 0; g < kGroup; ++g) {
        if (g < n_mem) {
            float *orow = out + (((size_t)b * H + heads[g]) * Tq + my_i) * kHeadDim;
#pragma unroll
            for (int blk = 0; blk < kHeadDim / 32; ++blk)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    float4 o;
                    o.x = acc[g][blk][v4 * 4 + 0] * inv; o.y = acc[g][blk][v4 * 4 + 1] * inv;
                    o.z = acc[g][blk][v4 * 4 + 2] * inv; o.w = acc[g][blk][v4 * 4 + 3] * inv;
                    *reinterpret_cast<float4 *>(orow + blk * 32 + v4 * 8 + hl * 4) = o;
                }
        }
    }
}

}  // namespace

int prefill_max_groups(int H, int k) { return (H + kGroup - 1) / kGroup + k; }

size_t prefill_workspace_bytes(int B, int H, int k)
{
    const size_t groups = (size_t)B * prefill_max_groups(H, k) * (2 + kGroup) * sizeof(int32_t);
    return (groups + 255) / 256 * 256 + ((size_t)B * sizeof(int32_t) + 255) / 256 * 256;
}

int launch_prefill(const void *q, const void *kc, const void *v, const int32_t *h2c, const int32_t *rep, int B, int H,
                   int k, int Tq, int q_start, int Tc_cap, int T_cap, float scale, float *out, void *workspace,
                   bool identity, hipStream_t stream)
{
    const int max_groups = identity ? H : prefill_max_groups(H, k);
    int32_t *groups = static_cast<int32_t *>(workspace);
    const size_t goff = ((size_t)B * prefill_max_groups(H, k) * (2 + kGroup) * sizeof(int32_t) + 255) / 256 * 256;
    int32_t *n_groups = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + goff);
    const int n_qt = (Tq + kQTile - 1) / kQTile;
    if (identity) {
        prefill_kernel<true><<<dim3(n_qt, H, B), kPWaves * 64, 0, stream>>>(
            static_cast<const char *>(q), static_cast<const char *>(kc), static_cast<const char *>(v), nullptr, nullptr,
            nullptr, H, k, Tq, q_start, Tc_cap, T_cap, max_groups, scale, out);
        return (int)hipGetLastError();
    }
    prefill_plan_kernel<<<dim3(B), 64, 0, stream>>>(h2c, rep, H, k, max_groups, groups, n_groups);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
    prefill_kernel<false><<<dim3(n_qt, max_groups, B), kPWaves * 64, 0, stream>>>(
        static_cast<const char *>(q), static_cast<const char *>(kc), static_cast<const char *>(v), rep, groups, n_groups,
        H, k, Tq, q_start, Tc_cap, T_cap, max_groups, scale, out);
    return (int)hipGetLastError();
}

}  // namespace chai
