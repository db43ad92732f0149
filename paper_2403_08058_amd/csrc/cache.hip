// K-cache pruning and cache growth (Section 3.5: after membership is fixed only the representatives' keys are
// kept; all values are kept).  Pure 16-byte copies: bit-exact by construction, bound by HBM bandwidth.
#include "chai_internal.h"

#include <hip/hip_ext.h>

namespace chai {

namespace {

constexpr int kCopyUnroll = 4;

// grid (ceil(vec_per_stream / (256*4)), k, B): copies the first T rows of the representative's key stream.
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
        if (i < vec_per_stream) tmp[u] = src[i];
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
    // about 2048 workgroups (8 per CU), between 64 KiB and 512 KiB each
    unsigned long long per_wg = ((unsigned long long)bytes / 2048 + 16383) / 16384 * 16384;
    per_wg = per_wg < 65536 ? 65536 : (per_wg > 524288 ? 524288 : per_wg);
    const unsigned int n_wg = (unsigned int)((bytes + per_wg - 1) / per_wg);
    return (int)launch_kernel(stream_read_kernel, dim3(n_wg), dim3(kBlock), 0, stream, ev, static_cast<const char *>(buf),
                              per_wg, (unsigned long long)bytes, sink);
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
