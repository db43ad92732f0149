// K-cache pruning and cache growth (Section 3.5: after membership is fixed only the representatives' keys are
// kept; all values are kept).  Pure 16-byte copies: bit-exact by construction, bound by HBM bandwidth.
#include "chai_internal.h"

#include <hip/hip_ext.h>

namespace chai {

namespace {

// Copy shape measured on MI355X (64 MiB and 512 MiB of keys, read + write): non-temporal loads, plain stores and
// eight 16-byte pieces per thread reach 73-76 % of the 8 TB/s peak; plain loads with four pieces 57-62 %,
// non-temporal stores as well 78 % on the small and 67-73 % on the large copy.
constexpr int kCopyUnroll = 8;
typedef unsigned int copy_u32x4 __attribute__((ext_vector_type(4)));

// grid (ceil(vec_per_stream / (256*8)), k, B): copies the first T rows of the representative's key stream.
__global__ __launch_bounds__(kBlock) void compact_kernel(const uint4 *__restrict__ k_full,
                                                         const int32_t *__restrict__ rep,
                                                         uint4 *__restrict__ k_compact, int H, int k,
                                                         long long vec_per_stream, long long src_stride,
                                                         long long dst_stride)
{
    const int j = blockIdx.y, b = blockIdx.z;
    int r = rep[(size_t)b * k + j];
    if (r < 0) return;
    r = min(r, H - 1);
    const uint4 *src = k_full + ((size_t)b * H + r) * src_stride;
    uint4 *dst = k_compact + ((size_t)b * k + j) * dst_stride;
    const long long base = ((long long)blockIdx.x * kCopyUnroll) * kBlock + threadIdx.x;
    uint4 tmp[kCopyUnroll];
#pragma unroll
    for (int u = 0; u < kCopyUnroll; ++u) {
        const long long i = base + (long long)u * kBlock;
        if (i < vec_per_stream) {
            const copy_u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const copy_u32x4 *>(src + i));
            tmp[u] = make_uint4(t.x, t.y, t.z, t.w);
        }
    }
#pragma unroll
    for (int u = 0; u < kCopyUnroll; ++u) {
        const long long i = base + (long long)u * kBlock;
        if (i < vec_per_stream) dst[i] = tmp[u];
    }
}

// grid (k + H, B), one wave: rows 0..k-1 are key rows of the representatives, rows k..k+H-1 are value rows.
__global__ __launch_bounds__(64) void append_kernel(const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new,
                                                    const int32_t *__restrict__ rep, uint4 *__restrict__ k_compact,
                                                    uint4 *__restrict__ v_cache, int H, int k, int pos,
                                                    long long kc_stride, long long v_stride, int vec_per_row)
{
    const int row = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    if (lane >= vec_per_row) return;
    if (row < k) {
        int r = rep[(size_t)b * k + row];
        if (r < 0) return;
        r = min(r, H - 1);
        k_compact[((size_t)b * k + row) * kc_stride + (size_t)pos * vec_per_row + lane] =
            k_new[((size_t)b * H + r) * vec_per_row + lane];
    } else {
        const int h = row - k;
        v_cache[((size_t)b * H + h) * v_stride + (size_t)pos * vec_per_row + lane] =
            v_new[((size_t)b * H + h) * vec_per_row + lane];
    }
}

// ---------------------------------------------------------------------------------------------------------
// Quantised caches (the paper names K,V-cache quantisation as orthogonal to clustering heads): rows of 128
// elements become 8-bit floating point codes (E4M3 of the OCP 8-bit floating point specification: bias 7,
// subnormals, largest finite value 448) with one fp32 scale per row: scale = amax / 448, code = nearest E4M3
// value (ties to even) of x * (448 / amax), all in fp32; an all-zero row gets scale 0 and codes 0.
// ---------------------------------------------------------------------------------------------------------

// E4M3 code of a finite y with |y| <= 448, by integer arithmetic on the fp32 bits (round to nearest, ties to even).
__device__ __forceinline__ unsigned int e4m3_code(float y)
{
    const unsigned int u = __float_as_uint(y);
    const unsigned int sign = (u >> 24) & 0x80u;
    const unsigned int a = u & 0x7fffffffu;
    const float af = __uint_as_float(a);
    unsigned int code;
    if (af < 0.015625f) {
        // below the smallest normal (2^-6) the codes are evenly spaced by 2^-9: count the steps (8 = 2^-6 itself)
        code = (unsigned int)__builtin_rintf(af * 512.0f);
    } else {
        // keep three mantissa bits: add half of the dropped part (minus one when the kept part is even), then
        // re-bias the exponent from 127 to 7; a carry out of the mantissa moves into the exponent by itself
        const unsigned int t = (a + 0x7ffffu + ((a >> 20) & 1u)) >> 20;
        code = t - ((127u - 7u) << 3);
    }
    return sign | code;
}

// Sixteen lanes quantise one row, eight elements each: returns the eight codes of this lane (two words) and the
// row's scale.  All sixteen lanes of the group must call it together.
template <bool BF16>
__device__ __forceinline__ uint2 quantize_piece(const char *row, int piece, float &scale)
{
    float x[8];
    if (BF16) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(row + piece * 16);
        const unsigned int w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __uint_as_float(w[i] << 16);
            x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    } else {
        const float4 lo = *reinterpret_cast<const float4 *>(row + piece * 32);
        const float4 hi = *reinterpret_cast<const float4 *>(row + piece * 32 + 16);
        x[0] = lo.x; x[1] = lo.y; x[2] = lo.z; x[3] = lo.w;
        x[4] = hi.x; x[5] = hi.y; x[6] = hi.z; x[7] = hi.w;
    }
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(x[i]));
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
    if (amax == 0.f) {
        scale = 0.f;
        return make_uint2(0u, 0u);
    }
    scale = amax / 448.0f;
    const float inv = 448.0f / amax;
    unsigned int c[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) c[i] = e4m3_code(fminf(fmaxf(x[i] * inv, -448.0f), 448.0f));
    return make_uint2(c[0] | (c[1] << 8) | (c[2] << 16) | (c[3] << 24), c[4] | (c[5] << 8) | (c[6] << 16) | (c[7] << 24));
}

// grid ceil(n_rows / 16), 256 threads: sixteen rows per workgroup, sixteen lanes per row
template <bool BF16>
__global__ __launch_bounds__(kBlock) void quantize_rows_kernel(const char *__restrict__ x, long long n_rows,
                                                               uint2 *__restrict__ codes, float *__restrict__ scales)
{
    const long long gid = (long long)blockIdx.x * kBlock + threadIdx.x;
    const long long row = gid >> 4;
    const int piece = (int)(gid & 15);
    const long long src = row < n_rows ? row : n_rows - 1;          // lanes past the end keep the shuffles whole
    float scale;
    const uint2 c = quantize_piece<BF16>(x + (size_t)src * (kHeadDim * (BF16 ? 2 : 4)), piece, scale);
    if (row < n_rows) {
        codes[row * 16 + piece] = c;
        if (piece == 0) scales[row] = scale;
    }
}

// grid (k + H, B), 64 threads (the first sixteen work): the new token's key rows of the representatives and value
// rows of all heads, quantised on their way into the caches
template <bool BF16>
__global__ __launch_bounds__(64) void append_q8_kernel(const char *__restrict__ k_new, const char *__restrict__ v_new,
                                                       const int32_t *__restrict__ rep, uint2 *__restrict__ k8,
                                                       float *__restrict__ kscale, uint2 *__restrict__ v8,
                                                       float *__restrict__ vscale, int H, int k, int pos, int Tc_cap,
                                                       int T_cap)
{
    const int row = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    if (lane >= 16) return;
    constexpr int kRowBytes = kHeadDim * (BF16 ? 2 : 4);
    float scale;
    if (row < k) {
        int r = rep[(size_t)b * k + row];
        if (r < 0) return;
        r = min(r, H - 1);
        const uint2 c = quantize_piece<BF16>(k_new + ((size_t)b * H + r) * kRowBytes, lane, scale);
        const size_t dst = ((size_t)b * k + row) * Tc_cap + pos;
        k8[dst * 16 + lane] = c;
        if (lane == 0) kscale[dst] = scale;
    } else {
        const int h = row - k;
        const uint2 c = quantize_piece<BF16>(v_new + ((size_t)b * H + h) * kRowBytes, lane, scale);
        const size_t dst = ((size_t)b * H + h) * T_cap + pos;
        v8[dst * 16 + lane] = c;
        if (lane == 0) vscale[dst] = scale;
    }
}

// grid (2k, B), one wave: rows 0..k-1 key rows, rows k..2k-1 value rows, both of the representatives.
__global__ __launch_bounds__(64) void append_shared_kernel(const uint4 *__restrict__ k_new,
                                                           const uint4 *__restrict__ v_new,
                                                           const int32_t *__restrict__ rep,
                                                           uint4 *__restrict__ k_compact, uint4 *__restrict__ v_compact,
                                                           int H, int k, int pos, long long kc_stride,
                                                           long long vc_stride, int vec_per_row)
{
    const int row = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
    if (lane >= vec_per_row) return;
    const int j = row < k ? row : row - k;
    int r = rep[(size_t)b * k + j];
    if (r < 0) return;
    r = min(r, H - 1);
    const size_t src = ((size_t)b * H + r) * vec_per_row + lane;
    if (row < k) k_compact[((size_t)b * k + j) * kc_stride + (size_t)pos * vec_per_row + lane] = k_new[src];
    else v_compact[((size_t)b * k + j) * vc_stride + (size_t)pos * vec_per_row + lane] = v_new[src];
}

// Bare streaming read (measurement aid): every workgroup reads `per_wg` consecutive bytes with the same 16-byte
// non-temporal loads, eight in flight per lane, as the decode kernels use, and adds the words up so that the loads
// cannot be dropped.  What this kernel reaches is the practical ceiling for the decode kernels on this part.
__global__ __launch_bounds__(kBlock) void stream_read_kernel(const char *__restrict__ buf, unsigned long long per_wg,
                                                             unsigned long long bytes, float *__restrict__ sink)
{
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const unsigned long long begin = (unsigned long long)blockIdx.x * per_wg;
    const unsigned long long nvec = (min(begin + per_wg, bytes) - begin) / 16;
    const char *base = buf + begin;
    float acc = 0.f;
    for (unsigned long long i = threadIdx.x; i < nvec; i += (unsigned long long)kBlock * 8) {
        u32x4 r[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const unsigned long long j = min(i + (unsigned long long)u * kBlock, nvec - 1);
            r[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(base + j * 16));
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            acc += __uint_as_float(r[u].x) + __uint_as_float(r[u].y) + __uint_as_float(r[u].z) + __uint_as_float(r[u].w);
    }
    if (acc == 123.456f) sink[0] = acc;          // practically never true: the sum only keeps the loads alive
}

}  // namespace

int launch_stream_read(const void *buf, size_t bytes, float *sink, const KernelEvents &ev, hipStream_t stream)
{
    // Best of a sweep on MI355X over workgroup size (256/512/1024 threads), loads in flight per lane (4/8/16),
    // bytes per workgroup (64 KiB .. 1 MiB) and plain against non-temporal loads: from 256 MiB up, ONE workgroup
    // per CU with 1/256 of the buffer each (88.6 % of the 8 TB/s peak at 256 MiB against 85 % for the next best
    // shape); below that, 128 KiB per workgroup (80.7 % at 144 MiB, 66-72 % at 45 MiB, where larger pieces leave
    // CUs without work).  Workgroups of 512 and 1024 threads and 4 or 16 loads per lane are within 1-2 % of
    // 256 threads x 8 loads; plain loads are ~10 % behind non-temporal ones.
    unsigned long long per_wg = 131072;
    if (bytes >= ((size_t)256 << 20)) per_wg = ((unsigned long long)bytes / 256 + 16383) / 16384 * 16384;
    const unsigned int n_wg = (unsigned int)((bytes + per_wg - 1) / per_wg);
    return (int)launch_kernel(stream_read_kernel, dim3(n_wg), dim3(kBlock), 0, stream, ev, static_cast<const char *>(buf),
                              per_wg, (unsigned long long)bytes, sink);
}

int launch_quantize_rows(const void *x, int dtype, long long n_rows, uint8_t *codes, float *scales, hipStream_t stream)
{
    const unsigned int n_wg = (unsigned int)((n_rows + 15) / 16);
    const char *xc = static_cast<const char *>(x);
    uint2 *out = reinterpret_cast<uint2 *>(codes);
    if (dtype == CHAI_BF16)
        return (int)launch_kernel(quantize_rows_kernel<true>, dim3(n_wg), dim3(kBlock), 0, stream, KernelEvents(), xc,
                                  n_rows, out, scales);
    return (int)launch_kernel(quantize_rows_kernel<false>, dim3(n_wg), dim3(kBlock), 0, stream, KernelEvents(), xc, n_rows,
                              out, scales);
}

int launch_append_kv_q8(const void *k_new, const void *v_new, const int32_t *rep, uint8_t *k8, float *kscale, uint8_t *v8,
                        float *vscale, int B, int H, int k, int pos, int Tc_cap, int T_cap, int dtype, hipStream_t stream)
{
    const char *kn = static_cast<const char *>(k_new), *vn = static_cast<const char *>(v_new);
    uint2 *k8v = reinterpret_cast<uint2 *>(k8), *v8v = reinterpret_cast<uint2 *>(v8);
    if (dtype == CHAI_BF16)
        return (int)launch_kernel(append_q8_kernel<true>, dim3(k + H, B), dim3(64), 0, stream, KernelEvents(), kn, vn, rep,
                                  k8v, kscale, v8v, vscale, H, k, pos, Tc_cap, T_cap);
    return (int)launch_kernel(append_q8_kernel<false>, dim3(k + H, B), dim3(64), 0, stream, KernelEvents(), kn, vn, rep,
                              k8v, kscale, v8v, vscale, H, k, pos, Tc_cap, T_cap);
}

int launch_append_kv_shared(const void *k_new, const void *v_new, const int32_t *rep, void *k_compact, void *v_compact,
                            int B, int H, int k, int pos, int Tc_cap, int Tv_cap, int dtype, hipStream_t stream)
{
    const int vec_per_row = kHeadDim * (dtype == CHAI_BF16 ? 2 : 4) / 16;
    return (int)launch_kernel(append_shared_kernel, dim3(2 * k, B), dim3(64), 0, stream, KernelEvents(),
                              static_cast<const uint4 *>(k_new), static_cast<const uint4 *>(v_new), rep,
                              static_cast<uint4 *>(k_compact), static_cast<uint4 *>(v_compact), H, k, pos,
                              (long long)Tc_cap * vec_per_row, (long long)Tv_cap * vec_per_row, vec_per_row);
}

int launch_compact_kcache(const void *k_full, const int32_t *rep, void *k_compact, int B, int H, int k, int T,
                          int T_cap, int Tc_cap, int dtype, hipStream_t stream)
{
    const long long vec_per_row = kHeadDim * (dtype == CHAI_BF16 ? 2 : 4) / 16;
    const long long vec_per_stream = (long long)T * vec_per_row;
    const long long per_block = (long long)kBlock * kCopyUnroll;
    const unsigned int gx = (unsigned int)((vec_per_stream + per_block - 1) / per_block);
    return (int)launch_kernel(compact_kernel, dim3(gx, k, B), dim3(kBlock), 0, stream, KernelEvents(),
                              static_cast<const uint4 *>(k_full), rep, static_cast<uint4 *>(k_compact), H, k,
                              vec_per_stream, (long long)T_cap * vec_per_row, (long long)Tc_cap * vec_per_row);
}

int launch_append_kv(const void *k_new, const void *v_new, const int32_t *rep, void *k_compact, void *v_cache, int B,
                     int H, int k, int pos, int Tc_cap, int T_cap, int dtype, hipStream_t stream)
{
    const int vec_per_row = kHeadDim * (dtype == CHAI_BF16 ? 2 : 4) / 16;
    return (int)launch_kernel(append_kernel, dim3(k + H, B), dim3(64), 0, stream, KernelEvents(),
                              static_cast<const uint4 *>(k_new), static_cast<const uint4 *>(v_new), rep,
                              static_cast<uint4 *>(k_compact), static_cast<uint4 *>(v_cache), H, k, pos,
                              (long long)Tc_cap * vec_per_row, (long long)T_cap * vec_per_row, vec_per_row);
}

}  // namespace chai
