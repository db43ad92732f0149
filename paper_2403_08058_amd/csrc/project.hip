// Query / key projections of the representative heads only (Fig. 3, Section 3.5: clustered attention needs the
// query and key vectors of one head per cluster, so the columns of W_Q and W_K that belong to the other heads are
// never multiplied; the new keys go straight into the pruned K cache).  A dense contraction with reuse on both
// operands, so it runs on the matrix cores.
//
//   for batch row b, slot j, r = rep_heads[b][j] >= 0, token i < Tn:
//       q_out[b][r][i][:]            = bf16( x[b][i][:] . w_q[r*128 .. r*128+127][:]^T )
//       k_compact[b][j][pos0 + i][:] = bf16( x[b][i][:] . w_k[r*128 .. r*128+127][:]^T )
//
// One workgroup (8 waves) computes a 256-token x 256-column tile: the 128 query columns and the 128 key columns
// of one representative, which share the activation tile.  The product is formed transposed, C^T = W X^T, with
// v_mfma_f32_32x32x16_bf16: both operands are then read along the contraction axis (weights are stored one row
// per output feature), a lane owns one token and gets 4 consecutive output features per register quad, so rows
// are written in 8-byte pieces.  Operand tiles of 64 contraction steps go global -> registers -> LDS (double
// buffered, one barrier per step); fp32 accumulation, one rounding to bf16 at the end.
#include "chai_internal.h"

#include <hip/hip_ext.h>

namespace chai {

namespace {

constexpr int kJBlock = 512;                 // threads (8 waves: 4 along the tokens x 2 along the columns)
constexpr int kJTok = 256;                   // tokens per workgroup tile
constexpr int kJCol = 2 * kHeadDim;          // columns per workgroup tile: query + key columns of one head
constexpr int kJStep = 64;                   // contraction elements per LDS tile
constexpr int kJStride = kJStep + 8;         // halves per LDS row (144 B: rows land on different banks)
constexpr size_t kJTileBytes = (size_t)(kJTok + kJCol) * kJStride * 2;     // activations + weights, one stage
constexpr size_t kJLdsBytes = 2 * kJTileBytes;
constexpr int kJPieces = (kJTok + kJCol) * kJStep * 2 / 16 / kJBlock;      // 16-byte pieces per thread per stage (8)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

union Frag {
    u32x4 raw;
    bf16x8 bf;
};

// 1-D grid of n_mt * k * B workgroups, renumbered so that each XCD owns a contiguous range of (batch row, token
// tile) pairs with all their cluster slots: the slots of a pair read the same activations and find them in L2.
__global__ __launch_bounds__(kJBlock) void project_kernel(const char *__restrict__ x, const char *__restrict__ w_q,
                                                          const char *__restrict__ w_k,
                                                          const int32_t *__restrict__ rep, int H, int k, int Tn, int D,
                                                          int n_mt, char *__restrict__ q_out,
                                                          char *__restrict__ k_compact, int pos0, int Tc_cap)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r = lane & 31, hl = lane >> 5;
    const int wm = w & 3, wn = w >> 2;               // wave's 64-token strip, and query (0) or key (1) half

    int j, mt, b;
    {
        const unsigned n = blockIdx.x, N = gridDim.x;
        const unsigned xcd = n & 7u, per = N >> 3, rem = N & 7u;
        const unsigned item = xcd * per + min(xcd, rem) + (n >> 3);
        j = (int)(item % (unsigned)k);
        const unsigned rest = item / (unsigned)k;
        mt = (int)(rest % (unsigned)n_mt);
        b = (int)(rest / (unsigned)n_mt);
    }
    const int head = rep[(size_t)b * k + j];
    if (head < 0) return;
    const int rh = min(head, H - 1);
    const int t0 = mt * kJTok;

    // staging: a thread's piece i (of 8) is 16 bytes of row (tid >> 3) + 64 i of the stage, rows 0..255 being the
    // activation tile and rows 256..511 the weight tile (query rows, then key rows).  Uniform base pointers plus
    // 32-bit per-lane offsets (one batch row of activations and one head's weights are far below 4 GiB).
    const unsigned int row_bytes = (unsigned int)D * 2u;
    const int srow = tid >> 3, c = tid & 7;
    const char *xb = x + (size_t)b * Tn * row_bytes;
    const char *wqb = w_q + (size_t)rh * kHeadDim * row_bytes;
    const char *wkb = w_k + (size_t)rh * kHeadDim * row_bytes;
    unsigned int xoff[4], woff[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) xoff[i] = (unsigned int)min(t0 + srow + 64 * i, Tn - 1) * row_bytes + c * 16;
#pragma unroll
    for (int i = 0; i < 2; ++i) woff[i] = (unsigned int)(srow + 64 * i) * row_bytes + c * 16;
    const int dst0 = (srow * kJStride + c * 8) * 2;
    u32x4 regs[kJPieces];
    auto fetch = [&](int step) {
        const unsigned int so = (unsigned int)step * (kJStep * 2);
#pragma unroll
        for (int i = 0; i < 4; ++i) regs[i] = *reinterpret_cast<const u32x4 *>(xb + (xoff[i] + so));
#pragma unroll
        for (int i = 0; i < 2; ++i) regs[4 + i] = *reinterpret_cast<const u32x4 *>(wqb + (woff[i] + so));
#pragma unroll
        for (int i = 0; i < 2; ++i) regs[6 + i] = *reinterpret_cast<const u32x4 *>(wkb + (woff[i] + so));
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < kJPieces; ++i)
            *reinterpret_cast<u32x4 *>(lds + buf * kJTileBytes + dst0 + i * 64 * kJStride * 2) = regs[i];
    };

    f32x16 acc[4][2];                                // [column block of 32][token block of 32]
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[nb][tb][e] = 0.f;

    // fragment addresses inside a stage: weights (A operand) rows kJTok + wn*128 + nb*32 + r, activations
    // (B operand) rows wm*64 + tb*32 + r; 8 halves at 16*ks + 8*hl
    const int a_off = ((kJTok + wn * kHeadDim + r) * kJStride + hl * 8) * 2;
    const int b_off = ((wm * 64 + r) * kJStride + hl * 8) * 2;

    const int n_steps = D / kJStep;
    fetch(0);
    stage(0);
    if (n_steps > 1) fetch(1);
    __syncthreads();
    for (int s = 0; s < n_steps; ++s) {
        const int buf = s & 1;
        if (s + 1 < n_steps) stage(buf ^ 1);          // fetched one iteration ago
        if (s + 2 < n_steps) fetch(s + 2);
        const char *base = lds + buf * kJTileBytes;
        // scheduling hint: spread the LDS reads and the stage's global loads and LDS writes between the MFMAs of
        // the step instead of grouping them (measured: about 2 % faster)
        __builtin_amdgcn_iglp_opt(1);
#pragma unroll
        for (int ks = 0; ks < kJStep / 16; ++ks) {
            Frag af[4], bfr[2];
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
                af[nb].raw = *reinterpret_cast<const u32x4 *>(base + a_off + (nb * 32 * kJStride + ks * 16) * 2);
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
                bfr[tb].raw = *reinterpret_cast<const u32x4 *>(base + b_off + (tb * 32 * kJStride + ks * 16) * 2);
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
                    acc[nb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[nb].bf, bfr[tb].bf, acc[nb][tb], 0, 0, 0);
        }
        __syncthreads();
    }

    // D[(v/4)*8 + hl*4 + v%4][r]: this lane's token is t0 + wm*64 + tb*32 + r, its features nb*32 + (v/4)*8 + hl*4 ..+3
    char *orow_base = wn == 0 ? q_out + ((size_t)b * H + rh) * (size_t)Tn * (kHeadDim * 2)
                              : k_compact + (((size_t)b * k + j) * (size_t)Tc_cap + pos0) * (kHeadDim * 2);
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        const int t = t0 + wm * 64 + tb * 32 + r;
        if (t >= Tn) continue;
        char *orow = orow_base + (size_t)t * (kHeadDim * 2);
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[nb][tb][v4 * 4 + e];
                *reinterpret_cast<bf16x4 *>(orow + (nb * 32 + v4 * 8 + hl * 4) * 2) = o;
            }
    }
}

// Measurement aid: the matrix pipe alone.  Every wave (two per SIMD on every CU) loads six operand fragments from
// `buf` once and then issues rounds of eight independent v_mfma_f32_32x32x16_bf16 with nothing else in the loop.
// The rate depends on the operand VALUES (switching activity moves the clocks), hence operands from the caller's
// data rather than constants.
constexpr int kProbeBlocks = 512, kProbeMfmaPerRound = 8;
__global__ __launch_bounds__(kJBlock) void mfma_probe_kernel(const u32x4 *__restrict__ buf, unsigned long long n_pieces,
                                                             int rounds, float *__restrict__ sink)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    Frag a[2], b[4];
#pragma unroll
    for (int i = 0; i < 6; ++i) {
        const unsigned long long at = (((unsigned long long)blockIdx.x * 8 + w) * 6 + i) * 64 + lane;
        (i < 2 ? a[i] : b[i - 2]).raw = buf[at % n_pieces];
    }
    f32x16 acc[kProbeMfmaPerRound];
#pragma unroll
    for (int i = 0; i < kProbeMfmaPerRound; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    for (int it = 0; it < rounds; ++it) {
#pragma unroll
        for (int i = 0; i < kProbeMfmaPerRound; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 1].bf, b[i >> 1].bf, acc[i], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < kProbeMfmaPerRound; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) t += acc[i][e];
    if (t == 123.456f) sink[0] = t;              // practically never true: keeps the MFMAs alive
}

}  // namespace

double mfma_probe_flops(int rounds)
{
    return (double)kProbeBlocks * (kJBlock / 64) * (double)rounds * kProbeMfmaPerRound * (2.0 * 32 * 32 * 16);
}

int launch_mfma_probe(const void *buf, size_t bytes, int rounds, float *sink, const KernelEvents &ev, hipStream_t stream)
{
    return (int)launch_kernel(mfma_probe_kernel, dim3(kProbeBlocks), dim3(kJBlock), 0, stream, ev,
                              static_cast<const u32x4 *>(buf), (unsigned long long)(bytes / 16), rounds, sink);
}

int launch_project_qk(const void *x, const void *w_q, const void *w_k, const int32_t *rep, int B, int H, int k, int Tn,
                      int D, void *q_out, void *k_compact, int pos0, int Tc_cap, const KernelEvents &ev,
                      hipStream_t stream)
{
    static DeviceFlags lds_allowed;
    const hipError_t attr = allow_dynamic_lds(reinterpret_cast<const void *>(&project_kernel), kJLdsBytes, lds_allowed);
    if (attr != hipSuccess) return (int)attr;
    const int n_mt = (Tn + kJTok - 1) / kJTok;
    if ((long long)n_mt * k * B > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    return (int)launch_kernel(project_kernel, dim3((unsigned int)n_mt * k * B), dim3(kJBlock), kJLdsBytes, stream, ev,
                              static_cast<const char *>(x), static_cast<const char *>(w_q), static_cast<const char *>(w_k),
                              rep, H, k, Tn, D, n_mt, static_cast<char *>(q_out), static_cast<char *>(k_compact), pos0,
                              Tc_cap);
}

}  // namespace chai
