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
// Scores are computed transposed, S^T = K_tile Q^T (bf16 inputs): a lane then owns ONE query column and half of
// the keys of the tile, so row maxima and sums are in-lane plus one exchange with lane l^32, and the tile of
// probabilities is already in the B-operand layout of O^T += V^T P^T.  That second product runs in fp16 (P in
// [0,256] keeps 11 bits instead of bf16's 8).  Its A operand needs 8 keys of one value column per lane, which a
// row-major V cache cannot deliver, so a first kernel writes V^T once per call: fp16 (exact from bf16 inside
// the fp16 range, |v| <= 65504), in blocks of 32 keys x 128 columns, keys permuted inside every group of 16 into
// the order the probability registers have, zero beyond the last key.  The main kernel then stages K and V^T
// tiles in LDS with 16-byte direct loads and feeds every MFMA operand with one ds_read_b128.  (The LDS transpose
// reads of this chip could hand the operand over from a row-major bf16 tile and make the pre-pass unnecessary,
// but only as bf16: the probabilities would then be rounded to 8 bits as well, up to 2^-9 of relative error per
// element, which is the whole error budget of the 16-bit contract; converting the values to fp16 inside the
// main kernel instead would be paid by every workgroup that streams a tile, a dozen vector instructions per
// MFMA.)
#include "chai_internal.h"

#include <hip/hip_ext.h>

#include <type_traits>

namespace chai {

namespace {

constexpr int kGroup = 2;          // member heads that share one score tile
constexpr int kPairedRounds = 4;     // launches of fewer rounds of 256 paired workgroups send single tiles instead
constexpr int kRec = 2 + kGroup;   // ints per work-list record: cluster, member count, members
constexpr int kQWave = 32;         // query rows per wave
constexpr int kPWaves = 8;         // waves per workgroup (two per SIMD: one's MFMAs overlap the other's VALU work)
constexpr int kPBlock = kPWaves * 64;
constexpr int kQTile = kQWave * kPWaves;   // 256 query rows per workgroup
constexpr int kKTile = 64;         // keys per tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kRescaleSlack = 8.0f;      // log2 units a tile may exceed the running maximum before a rescale

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

union Frag16 {            // 16 bytes seen as a raw load, bf16 x 8 or fp16 x 8
    u32x4 raw;
    bf16x8 bf;
    f16x8 h;
};

// Both halves of a wave get x of lanes 0..31 and x of lanes 32..63 (lane l and lane l ^ 32 see the same pair, in
// the same order): one v_permlane32_swap instead of a round trip through the LDS crossbar.
__device__ __forceinline__ void both_halves(float x, float &lo, float &hi)
{
    const unsigned int bits = __float_as_uint(x);
    const auto sw = __builtin_amdgcn_permlane32_swap(bits, bits, false, false);
    lo = __uint_as_float(sw[0]);
    hi = __uint_as_float(sw[1]);
}

// Position of key jj (0..15) inside its group of 16 in V^T: lane half hl of MFMA step s multiplies its
// probability registers e = 0..7, which hold keys 16s + (e/4)*8 + hl*4 + e%4, with 8 consecutive halves.
__device__ __forceinline__ int key_slot16(int r16) { return 8 * ((r16 & 7) >> 2) + 4 * (r16 >> 3) + (r16 & 3); }

// ---------------------------------------------------------------------------------------------------------
// V^T in blocks of 32 keys: vt[b][h][t/32][dd][16*((t%32)/16) + key_slot16(t%16)] = fp16(V[b][h][t][dd]) for
// t < n_keys, 0 up to Tp (a multiple of 64).  A block is 8 KB of consecutive memory, so the main kernels stage it
// with fully coalesced 16-byte loads.  grid (Tp/64, H, B), 256 threads; a 64 x 128 tile goes through LDS.
// ---------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void vt_kernel(const char *__restrict__ v, int H, int T_cap, int n_keys, int Tp,
                                                 _Float16 *__restrict__ vt)
{
    __shared__ _Float16 tile[kHeadDim][kKTile + 2];
    const int tid = threadIdx.x, t0 = blockIdx.x * kKTile, h = blockIdx.y, b = blockIdx.z;
    const char *vhead = v + ((size_t)b * H + h) * (size_t)T_cap * (kHeadDim * 2);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int piece = tid + i * 256, jj = piece >> 4, c8 = piece & 15;       // key row, 8-column block
        Frag16 x;
        x.raw = u32x4{0u, 0u, 0u, 0u};
        if (t0 + jj < n_keys)
            x.raw = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(vhead + (size_t)(t0 + jj) * (kHeadDim * 2) + c8 * 16));
        const int slot = 16 * (jj >> 4) + key_slot16(jj & 15);
#pragma unroll
        for (int e = 0; e < 8; ++e) tile[c8 * 8 + e][slot] = (_Float16)(float)x.bf[e];
    }
    __syncthreads();
    _Float16 *dst = vt + (((size_t)b * H + h) * (Tp / 32) + t0 / 32) * (size_t)(kHeadDim * 32);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int idx = tid + i * 256, c8 = idx & 7, dd = (idx >> 3) & (kHeadDim - 1), blk = idx >> 10;   // 4 keys each
        const unsigned int lo = *reinterpret_cast<const unsigned int *>(&tile[dd][blk * 32 + c8 * 4]);
        const unsigned int hi = *reinterpret_cast<const unsigned int *>(&tile[dd][blk * 32 + c8 * 4 + 2]);
        *reinterpret_cast<uint2 *>(dst + ((size_t)blk * kHeadDim + dd) * 32 + c8 * 4) = make_uint2(lo, hi);
    }
}

// ---------------------------------------------------------------------------------------------------------
// Work list: the heads of every cluster, in ascending order, cut into groups of at most `gsize` (<= kGroup).
// groups[b][g] = {cluster, n, head_0 .. }, kRec ints per record; clusters in ascending order.  One workgroup per
// batch row: the membership row is copied to LDS, thread j counts cluster j, thread h ranks head h among the
// heads of its cluster, and every head writes its own slot.  Heads that name no live cluster are left out.
// Dynamic LDS: (H + 2k) ints.
// ---------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prefill_plan_kernel(const int32_t *__restrict__ h2c,
                                                           const int32_t *__restrict__ rep, int H, int k, int gsize,
                                                           int max_groups, int32_t *__restrict__ groups,
                                                           int32_t *__restrict__ n_groups)
{
    extern __shared__ int32_t plan_lds[];
    int32_t *member = plan_lds, *count = plan_lds + H, *base = count + k;
    const int b = blockIdx.x, tid = threadIdx.x;
    for (int h = tid; h < H; h += blockDim.x) {
        const int c = h2c[(size_t)b * H + h];
        member[h] = (c >= 0 && c < k && rep[(size_t)b * k + c] >= 0) ? c : -1;
    }
    __syncthreads();
    for (int j = tid; j < k; j += blockDim.x) {
        int n = 0;
        for (int h = 0; h < H; ++h) n += member[h] == j;
        count[j] = n;
    }
    __syncthreads();
    for (int j = tid; j < k; j += blockDim.x) {
        int first = 0;
        for (int i = 0; i < j; ++i) first += (count[i] + gsize - 1) / gsize;
        base[j] = first;
        if (j == k - 1) {
            const int ng = first + (count[j] + gsize - 1) / gsize;
            n_groups[b] = ng < max_groups ? ng : max_groups;
        }
    }
    __syncthreads();
    int32_t *g = groups + (size_t)b * max_groups * kRec;
    for (int h = tid; h < H; h += blockDim.x) {
        const int c = member[h];
        if (c < 0) continue;
        int rank = 0;
        for (int i = 0; i < h; ++i) rank += member[i] == c;
        const int gi = base[c] + rank / gsize, slot = rank % gsize;
        if (gi >= max_groups) continue;
        g[gi * kRec + 2 + slot] = h;
        if (slot == 0) {
            const int left = count[c] - rank;
            g[gi * kRec] = c;
            g[gi * kRec + 1] = left < gsize ? left : gsize;
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// Main kernel.  1-D grid of ceil(n_qt / 2) * n_slots * B workgroups of 512 threads; IDENT: every head is its own cluster
// (dense attention) and the work list is not read.
//
// A score block is shared by the TWO members whose accumulators one wave can hold.  Two wider schemes were built,
// passed the same parity tests and measured no faster on the LLaMa-7B shape, so neither is kept:
//  * four members through LDS -- the two waves of a SIMD own the same 32 query rows and two members each, take
//    turns producing the probabilities of a 32-key block and hand them over in the B-operand layout, one barrier
//    per block: 670-840 us per 8-cluster layer in three schedules against 578 us for pairs (128 query rows per
//    workgroup double the staging per flop, and the producer's chain scores -> softmax -> publish is not hidden
//    by its partner);
//  * three members in ONE wave -- four waves per workgroup, one per SIMD, 192 accumulation registers of
//    accumulators (a fourth member does not fit: the compiler keeps every MFMA result, the score block's
//    included, in the accumulation half), the loop software-pipelined by hand (value products of block i-1, score
//    product of block i+1 and softmax of block i interleaved instruction by instruction, LDS fragments four
//    MFMAs ahead, rings of three 32-key blocks): equal to pairs when every cluster has exactly three heads
//    (592 against 596 us), 630 us against 553 us on the benchmark's membership and 1000 against 730 us when
//    every head is its own cluster.  A single wave per SIMD issues about eight vector instructions per MFMA and
//    nothing else fills its waits.
//
// Workgroup -> work item: the hardware deals consecutive workgroup ids round-robin to the 8 XCDs, each with an L2
// of its own.  The ids are therefore re-numbered so that every XCD owns a contiguous range of (batch row, group)
// pairs with all their query tiles (largest first): the tiles of one group stream the same keys and values and
// now find them in the same L2.
//
// LDS (dynamic): three K tiles and two V^T tiles per member.  K runs one tile ahead of V^T because the scores of
// a 32-key block are issued one block before its softmax (the matrix pipe works on the next block's scores while
// the vector ALUs exponentiate this one), and the extra buffer of each kind lets tile t+2 / t+1 be written while
// tile t is read: ONE barrier per 64-key tile.
// ---------------------------------------------------------------------------------------------------------
constexpr int kKBufs = 3, kVBufs = 2;
constexpr size_t kKBufBytes = (size_t)kKTile * kHeadDim * 2;        // 64 rows of 256 B (16 pieces), swizzled
constexpr size_t kVBufBytes = (size_t)kHeadDim * kKTile * 2;        // one member: 128 rows of 128 B (8 pieces), swizzled
constexpr size_t prefill_lds_bytes(bool ident) { return kKBufs * kKBufBytes + kVBufs * (ident ? 1 : kGroup) * kVBufBytes; }

template <bool IDENT>
__global__ __launch_bounds__(kPBlock) void prefill_kernel(const char *__restrict__ q, const char *__restrict__ kc,
                                                          const _Float16 *__restrict__ vt,
                                                          const int32_t *__restrict__ rep,
                                                          const int32_t *__restrict__ groups,
                                                          const int32_t *__restrict__ n_groups, int H, int k, int Tq,
                                                          int q_start, int Tc_cap, int Tp, int n_qt_arg, int n_slots,
                                                          int n_rows, float scale, float *__restrict__ out)
{
    constexpr int G = IDENT ? 1 : kGroup;
    extern __shared__ __attribute__((aligned(1024))) char lds_raw[];
    char *const k_lds = lds_raw;                                   // [kKBufs][kKTile][128] bf16, swizzled rows
    char *const v_lds = lds_raw + kKBufs * kKBufBytes;             // [kVBufs][G][kHeadDim][kKTile] fp16, swizzled rows

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r = lane & 31, hl = lane >> 5;

    // A work item is a PAIR of query tiles, the p-th largest and the p-th smallest of a group: under the causal
    // mask tile q walks q+1 key tiles' worth of work, so every pair costs the same and the workgroups of a launch
    // finish together instead of leaving a tail of long ones.
    // (n_qt < 0: a small launch; every tile is then an item of its own, see the numbering above.  On launches of
    // many rounds single tiles measured 3-8 % SLOWER than pairs: the tiles of a group no longer run side by side and
    // stop sharing its keys and values in L2.)
    const bool paired = n_qt_arg > 0;
    const int n_qt = paired ? n_qt_arg : -n_qt_arg;
    const int n_pairs = paired ? (n_qt + 1) / 2 : n_qt;
    int pi, gi, b;
    if (paired) {
        const unsigned n = blockIdx.x, N = gridDim.x;
        const unsigned x = n & 7u, per = N >> 3, rem = N & 7u;
        const unsigned item = x * per + min(x, rem) + (n >> 3);
        pi = (int)(item % (unsigned)n_pairs);
        const unsigned rest = item / (unsigned)n_pairs;
        gi = (int)(rest % (unsigned)n_slots);
        b = (int)(rest / (unsigned)n_slots);
    } else {
        // single tiles, the largest first: XCD x owns `per_xcd` consecutive (batch row, group) slots, and its
        // workgroups come in the order tile n_qt-1 of every slot, then tile n_qt-2 of every slot, ...; the hardware
        // hands the next workgroup to the first CU that is free, which is longest-job-first list scheduling
        const unsigned n = blockIdx.x, x = n & 7u, local = n >> 3;
        const unsigned per_xcd = gridDim.x / (8u * (unsigned)n_qt);
        const unsigned slot = x * per_xcd + local % per_xcd;
        if (slot >= (unsigned)(n_slots * n_rows)) return;
        pi = (int)(local / per_xcd);
        gi = (int)(slot % (unsigned)n_slots);
        b = (int)(slot / (unsigned)n_slots);
    }

    int cluster, n_mem, heads[G];
    if (IDENT) {
        cluster = gi; n_mem = 1;
        heads[0] = gi;
    } else {
        if (gi >= n_groups[b]) return;
        const int32_t *gr = groups + ((size_t)b * n_slots + gi) * kRec;
        cluster = min(max(gr[0], 0), k - 1);
        n_mem = min(max(gr[1], 1), kGroup);
#pragma unroll
        for (int g = 0; g < G; ++g) heads[g] = min(max(gr[2 + min(g, n_mem - 1)], 0), H - 1);
    }
    const int rhead = IDENT ? cluster : min(max(rep[(size_t)b * k + cluster], 0), H - 1);

    const float scale2 = scale * kLog2e;
    const int n_pass = (paired && (n_qt - 1 - pi) > pi) ? 2 : 1;     // the middle tile of an odd count is alone
    for (int pass = 0; pass < n_pass; ++pass) {
    const int qt = pass == 0 ? n_qt - 1 - pi : pi;
    const int i0 = qt * kQTile + w * kQWave;                 // first query row of this wave (relative)
    const int my_i = i0 + r;                                 // this lane's query row
    const int q_abs = q_start + min(my_i, Tq - 1);           // its sequence position (clamped for padding rows)
    const int wave_first = q_start + min(i0, Tq - 1);
    const int wave_last = q_start + min(i0 + kQWave - 1, Tq - 1);     // last position any lane of the wave sees
    const int wg_last = q_start + min(qt * kQTile + kQTile - 1, Tq - 1);
    const int n_tiles = wg_last / kKTile + 1;                // key tiles 0 .. n_tiles-1 cover positions <= wg_last
    const int n_hb = i0 < Tq ? wave_last / 32 + 1 : 0;       // 32-key blocks this wave works on (0: padding wave)
    const int n_keys = q_start + Tq;                         // keys that exist (rows past them are never read)

    // query fragments (B operand of S^T = K Q^T): Q[my_i][16*ks + 8*hl .. +7]
    Frag16 qf[kHeadDim / 16];
    {
        const char *qrow = q + (((size_t)b * H + rhead) * Tq + min(my_i, Tq - 1)) * (kHeadDim * 2) + hl * 16;
#pragma unroll
        for (int ks = 0; ks < kHeadDim / 16; ++ks) qf[ks].raw = *reinterpret_cast<const u32x4 *>(qrow + ks * 32);
    }

    // Staging with direct loads to LDS: one instruction moves 64 pieces of 16 bytes into 1 KB of consecutive LDS
    // (lane l's piece lands at base + 16 l), no registers and no LDS write instructions.  The BUFFER form of the
    // instruction is used: with the global form in a loop the compiler gives up counting LDS reads and waits for
    // all of them (lgkmcnt(0)) before every MFMA; with the buffer form it waits for exactly the fragment it needs
    // (measured 4-5 % faster, and the register allocation no longer spills).  Rows are unpadded, and bank
    // conflicts of the fragment reads are avoided by a swizzle instead: piece c of K row R sits in slot
    // c ^ (R & 15) of the row, piece c of V^T row R in slot c ^ ((R >> 1) & 7); 16 consecutive rows read at one
    // piece index then touch 16 different 16-byte slots of the 256-byte bank window.  A lane fetches whichever
    // piece belongs in the slot it fills.  Wave w fills K rows 4w..4w+3 and 32+4w.. (two instructions per tile)
    // and V^T rows 8w..8w+7 and 64+8w.. of every member (two instructions per member and tile).
    // Requesting the tiles one iteration earlier still (rings of six K half-tiles and three V^T tiles, the wait
    // before the barrier leaving the newest requests in flight) was measured too: no gain (565 against 553 us),
    // the loop does not wait for these loads.
    const char *ksrc = kc + ((size_t)b * k + cluster) * (size_t)Tc_cap * (kHeadDim * 2);
    const char *vsrc[G];
#pragma unroll
    for (int g = 0; g < G; ++g)
        vsrc[g] = reinterpret_cast<const char *>(vt + ((size_t)b * H + heads[g]) * (size_t)kHeadDim * Tp);
    const int k_row = 4 * w + (lane >> 4), k_piece = (lane & 15) ^ (k_row & 15);
    const int v_row = 8 * w + (lane >> 3), v_piece = (lane & 7) ^ ((v_row >> 1) & 7);
    // V^T in memory: blocks of 32 keys, [block][row][32 keys]; piece c of a 64-key row = block c/4, 16 B piece c%4
    const unsigned int v_off = (unsigned int)(((v_piece >> 2) * kHeadDim + v_row) * 64 + (v_piece & 3) * 16);
    // (the instruction exists only in the device pass of the compiler; the host pass sees an empty body)
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __amdgpu_buffer_rsrc_t Rsrc;
    auto make_rsrc = [](const char *base) {
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(base), 0, 0x7fffffff, 0x00020000);
    };
    auto load_to_lds = [](Rsrc rs, unsigned int off, char *dst) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void *)dst, 16, (int)off, 0, 0, 0);
    };
#else
    typedef const char *Rsrc;
    auto make_rsrc = [](const char *base) { return base; };
    auto load_to_lds = [](Rsrc, unsigned int, char *) {};
#endif
    const Rsrc k_rs = make_rsrc(ksrc);
    Rsrc v_rs[G];
#pragma unroll
    for (int g = 0; g < G; ++g) v_rs[g] = make_rsrc(vsrc[g]);
    auto dma_k = [&](int kt, int buf) {
        const int key0 = kt * kKTile;
#pragma unroll
        for (int i = 0; i < 2; ++i)
            load_to_lds(k_rs, (unsigned int)(min(key0 + k_row + 32 * i, n_keys - 1) * (kHeadDim * 2) + k_piece * 16),
                        k_lds + buf * kKBufBytes + (w + 8 * i) * 1024);
    };
    auto dma_v = [&](int kt, int g, int buf) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            load_to_lds(v_rs[g], (unsigned int)kt * (2 * kHeadDim * 64) + v_off + i * 64 * 64,
                        v_lds + (buf * G + g) * kVBufBytes + (w + 8 * i) * 1024);
    };
    // The barrier of the tile loop: every wave first waits for its own requests (the compiler does not track loads
    // that land in LDS), then a bare s_barrier -- __syncthreads() would add fences the loads-to-LDS do not need.
    auto tile_barrier = [&]() {
#if defined(__HIP_DEVICE_COMPILE__)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
#endif
    };
    // fragment read offsets: this lane's row r of a 32-row block, piece index p -> byte offset inside the block
    const int k_sw = r & 15, v_sw = (r >> 1) & 7;

    f32x16 acc[G][kHeadDim / 32];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int blk = 0; blk < kHeadDim / 32; ++blk)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[g][blk][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;          // running maximum (log2 units) and denominator of this query

    // S^T block: 32 keys (rows half*32 .. +31 of K buffer `buf`) x 32 queries
    auto score_block = [&](int buf, int half) {
        f32x16 st;
#pragma unroll
        for (int e = 0; e < 16; ++e) st[e] = 0.f;
        const char *kb = k_lds + buf * kKBufBytes + (half * 32 + r) * (kHeadDim * 2);
#pragma unroll
        for (int ks = 0; ks < kHeadDim / 16; ++ks) {
            Frag16 kf;
            kf.raw = *reinterpret_cast<const u32x4 *>(kb + (((2 * ks + hl) ^ k_sw) << 4));
            st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf.bf, qf[ks].bf, st, 0, 0, 0);
        }
        return st;
    };

    // One block (keys kbase .. kbase+31, scores st): online softmax and the product with the members' values from
    // V^T buffer vbuf.  HAS_NEXT: the scores of the wave's next block (K buffer nbuf, half nhalf) are issued in the
    // same stretch of code as the exponentials, one MFMA per handful of vector instructions, so that the matrix
    // pipe is busy while this wave exponentiates; they are returned.
    // Wave priority: raised while a wave is in the stretch that mixes vector work with score MFMAs, so that the
    // SIMD's arbiter favours it over the other wave's back-to-back value MFMAs, which lose nothing by waiting a
    // few cycles (measured: 1.5-4 % faster).
    auto wave_priority = [](bool high) {
#if defined(__HIP_DEVICE_COMPILE__)
        if (high) __builtin_amdgcn_s_setprio(2);
        else __builtin_amdgcn_s_setprio(0);
#else
        (void)high;
#endif
    };
    auto block = [&](f32x16 st, int kbase, int vbuf, int half, auto has_next, int nbuf, int nhalf) {
        constexpr bool HAS_NEXT = decltype(has_next)::value;
        // causal mask: only blocks that reach past the wave's first query need it (a real branch, uniform per
        // wave -- the empty asm keeps the compiler from turning it into 32 selects on every block)
        if (kbase + 31 > wave_first) {
            asm volatile("" ::: "memory");
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int key = kbase + (e >> 2) * 8 + hl * 4 + (e & 3);
                st[e] = key <= q_abs ? st[e] : -INFINITY;
            }
        }
        // maximum of the raw scores (scale > 0 is required); the scale, times log2 e, is folded into the
        // exponent: p = exp2(s * scale2 - m)
        float ext = st[0];
#pragma unroll
        for (int e = 1; e < 16; ++e) ext = fmaxf(ext, st[e]);
        float mx_lo, mx_hi;
        both_halves(ext * scale2, mx_lo, mx_hi);
        const float mx = fmaxf(mx_lo, mx_hi);
        // lazy reference: the running maximum only moves when a block exceeds it by more than kRescaleSlack, so
        // most blocks skip the rescaling of the accumulators (p < 2^slack)
        const bool need = mx > m_run + kRescaleSlack;
        const float m_new = need ? mx : m_run;
        const float alpha = need ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.0f;   // exp2(-inf) = 0 at the start
        if (__any(need)) {
            l_run *= alpha;
#pragma unroll
            for (int g = 0; g < G; ++g)
                if (g < n_mem)
#pragma unroll
                    for (int blk = 0; blk < kHeadDim / 32; ++blk)
#pragma unroll
                        for (int e = 0; e < 16; ++e) acc[g][blk][e] *= alpha;
        }
        m_run = m_new;

        wave_priority(true);
        f32x16 s_next = st;
        float rs = 0.f;
        Frag16 pf[2];
        if (HAS_NEXT) {
            // Exponentials of this block and scores of the next one, written out in the issue order wanted: per
            // step one MFMA of the next block's scores (its K fragment was requested two steps earlier) and the
            // vector work of two probabilities.  The scheduling barriers keep the compiler from regrouping it
            // into "all MFMAs, then all exponentials", which would leave the matrix pipe idle during the latter.
#pragma unroll
            for (int e = 0; e < 16; ++e) s_next[e] = 0.f;
            const char *kb = k_lds + nbuf * kKBufBytes + (nhalf * 32 + r) * (kHeadDim * 2);
            Frag16 kf[kHeadDim / 16];
            kf[0].raw = *reinterpret_cast<const u32x4 *>(kb + ((hl ^ k_sw) << 4));
            kf[1].raw = *reinterpret_cast<const u32x4 *>(kb + (((2 + hl) ^ k_sw) << 4));
#pragma unroll
            for (int i = 0; i < kHeadDim / 16; ++i) {
                if (i + 2 < kHeadDim / 16)
                    kf[i + 2].raw = *reinterpret_cast<const u32x4 *>(kb + (((2 * (i + 2) + hl) ^ k_sw) << 4));
                s_next = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i].bf, qf[i].bf, s_next, 0, 0, 0);
#pragma unroll
                for (int e = 2 * i; e < 2 * i + 2; ++e) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(st[e], scale2, -m_run));
                    rs += p;
                    pf[e >> 3].h[e & 7] = (_Float16)p;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = __builtin_amdgcn_exp2f(fmaf(st[e], scale2, -m_run));
                rs += p;
                pf[e >> 3].h[e & 7] = (_Float16)p;
            }
        }
        float rs_lo, rs_hi;
        both_halves(rs, rs_lo, rs_hi);
        l_run += rs_lo + rs_hi;
        wave_priority(false);
        // O^T[d][query] += V^T P^T for every member head: fragment j = (blk, s) of a member, requested
        // kVAhead MFMAs before its use so that the LDS latency hides behind the matrix pipe
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (g < n_mem) {
                const char *vb = v_lds + (vbuf * G + g) * kVBufBytes + r * (kKTile * 2);
                constexpr int kBlks = kHeadDim / 32, kFrags = 2 * kBlks, kVAhead = 3;
                // fragment j: value rows 32 * (j % kBlks) .., keys 16 * (j / kBlks) .. of the block (piece
                // 4 * half + 2 * (j / kBlks) + hl of the row); the two MFMAs that add into the same accumulator are
                // kBlks apart
                auto v_frag = [&](int j) {
                    return *reinterpret_cast<const u32x4 *>(vb + (j % kBlks) * 32 * (kKTile * 2) +
                                                            (((4 * half + 2 * (j / kBlks) + hl) ^ v_sw) << 4));
                };
                Frag16 vf[kFrags];
#pragma unroll
                for (int j = 0; j < kVAhead; ++j) vf[j].raw = v_frag(j);
#pragma unroll
                for (int j = 0; j < kFrags; ++j) {
                    if (j + kVAhead < kFrags) vf[j + kVAhead].raw = v_frag(j + kVAhead);
                    acc[g][j % kBlks] =
                        __builtin_amdgcn_mfma_f32_32x32x16_f16(vf[j].h, pf[j / kBlks].h, acc[g][j % kBlks], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        return s_next;
    };
    const std::true_type with_next;
    const std::false_type last_block;

    // prologue: K(0), K(1), V(0) requested together; the previous pass's last barrier has freed every buffer
    dma_k(0, 0);
#pragma unroll
    for (int g = 0; g < G; ++g)
        if (g < n_mem) dma_v(0, g, 0);
    if (n_tiles > 1) dma_k(1, 1);
    tile_barrier();
    // every wave, padding waves included: the first use of the query fragments is then outside the loop
    f32x16 s_cur = score_block(0, 0);

    // Iteration kt computes tile kt while K(kt+2) and V(kt+1) stream into the buffers that tile kt-1 has left
    // (its readers passed the barrier that ended iteration kt-1); they must have landed by the barrier that ends
    // this iteration.
    int kb3 = 0, vb2 = 0;                      // kt % 3, kt % 2
    for (int kt = 0; kt < n_tiles; ++kt) {
        const int kb3_1 = kb3 == 2 ? 0 : kb3 + 1, kb3_2 = kb3_1 == 2 ? 0 : kb3_1 + 1;
        if (kt + 2 < n_tiles) dma_k(kt + 2, kb3_2);
        if (kt + 1 < n_tiles) {
#pragma unroll
            for (int g = 0; g < G; ++g)
                if (g < n_mem) dma_v(kt + 1, g, vb2 ^ 1);
        }
        __builtin_amdgcn_sched_barrier(0);

        const int hb = 2 * kt;                             // blocks hb (first half of the tile) and hb + 1
        if (hb + 1 < n_hb) s_cur = block(s_cur, hb * 32, vb2, 0, with_next, kb3, 1);
        else if (hb < n_hb) s_cur = block(s_cur, hb * 32, vb2, 0, last_block, 0, 0);
        if (hb + 2 < n_hb) s_cur = block(s_cur, hb * 32 + 32, vb2, 1, with_next, kb3_1, 0);
        else if (hb + 1 < n_hb) s_cur = block(s_cur, hb * 32 + 32, vb2, 1, last_block, 0, 0);
        tile_barrier();                                    // tile kt is done with; tiles kt+1 / kt+2 are in LDS
        kb3 = kb3_1;
        vb2 ^= 1;
    }

    if (n_hb != 0 && my_i < Tq) {
        const float inv = 1.0f / l_run;
#pragma unroll
        for (int g = 0; g < G; ++g) {
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
    }   // the two query tiles of the pair
}

size_t round256(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace

int prefill_max_groups(int H, int k) { return (H + kGroup - 1) / kGroup + k; }

// work list + group counts + V^T
size_t prefill_workspace_bytes(int B, int H, int k, int n_keys)
{
    const size_t Tp = ((size_t)n_keys + kKTile - 1) / kKTile * kKTile;
    return round256((size_t)B * prefill_max_groups(H, k) * kRec * sizeof(int32_t)) +
           round256((size_t)B * sizeof(int32_t)) + round256((size_t)B * H * kHeadDim * Tp * sizeof(_Float16));
}

int launch_prefill(const void *q, const void *kc, const void *v, const int32_t *h2c, const int32_t *rep, int B, int H,
                   int k, int Tq, int q_start, int Tc_cap, int T_cap, float scale, float *out, void *workspace,
                   bool identity, const KernelEvents &ev, hipStream_t stream)
{
    const int n_keys = q_start + Tq;
    const int Tp = (n_keys + kKTile - 1) / kKTile * kKTile;
    const int max_groups = identity ? H : prefill_max_groups(H, k);
    char *ws = static_cast<char *>(workspace);
    int32_t *groups = reinterpret_cast<int32_t *>(ws);
    ws += round256((size_t)B * prefill_max_groups(H, k) * kRec * sizeof(int32_t));
    int32_t *n_groups = reinterpret_cast<int32_t *>(ws);
    ws += round256((size_t)B * sizeof(int32_t));
    _Float16 *vt = reinterpret_cast<_Float16 *>(ws);
    const int n_qt = (Tq + kQTile - 1) / kQTile;

    hipError_t e = launch_kernel(vt_kernel, dim3(Tp / kKTile, H, B), dim3(256), 0, stream, KernelEvents(),
                                 static_cast<const char *>(v), H, T_cap, n_keys, Tp, vt);
    if (e != hipSuccess) return (int)e;
    static DeviceFlags lds_ident, lds_clustered;
    e = identity ? allow_dynamic_lds(reinterpret_cast<const void *>(&prefill_kernel<true>), prefill_lds_bytes(true), lds_ident)
                 : allow_dynamic_lds(reinterpret_cast<const void *>(&prefill_kernel<false>), prefill_lds_bytes(false),
                                     lds_clustered);
    if (e != hipSuccess) return (int)e;
    // A workgroup takes a large and a small query tile (equal work for all), unless the launch is small: below
    // kPairedRounds rounds of the chip a partly filled last round of equal workgroups costs more than pairing
    // gains, and the tiles go out singly, the largest first.
    const bool paired = (long long)((n_qt + 1) / 2) * max_groups * B >= (long long)kPairedRounds * 256;
    const int n_qt_arg = paired ? n_qt : -n_qt;
    const long long slots = (long long)max_groups * B;
    const long long n_wg_ll = paired ? (long long)((n_qt + 1) / 2) * slots : 8LL * n_qt * ((slots + 7) / 8);
    if (n_wg_ll > 0x7fffffffLL) return (int)hipErrorInvalidConfiguration;
    const unsigned int n_wg = (unsigned int)n_wg_ll;
    if (identity) {
        return (int)launch_kernel(prefill_kernel<true>, dim3(n_wg), dim3(kPBlock), prefill_lds_bytes(true), stream, ev,
                                  static_cast<const char *>(q), static_cast<const char *>(kc), vt, nullptr, nullptr,
                                  nullptr, H, k, Tq, q_start, Tc_cap, Tp, n_qt_arg, max_groups, B, scale, out);
    }
    e = launch_kernel(prefill_plan_kernel, dim3(B), dim3(256), (size_t)(H + 2 * k) * sizeof(int32_t), stream,
                      KernelEvents(), h2c, rep, H, k, kGroup, max_groups, groups, n_groups);
    if (e != hipSuccess) return (int)e;
    return (int)launch_kernel(prefill_kernel<false>, dim3(n_wg), dim3(kPBlock), prefill_lds_bytes(false), stream, ev,
                              static_cast<const char *>(q), static_cast<const char *>(kc), vt, rep, groups, n_groups, H, k,
                              Tq, q_start, Tc_cap, Tp, n_qt_arg, max_groups, B, scale, out);
}

}  // namespace chai
