// Internal declarations shared by the translation units of libchai.so (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <stddef.h>
#include <stdint.h>

#include "chai.h"
#include "chai_probe.h"

namespace chai {

constexpr int kHeadDim = 128;       // the only head dimension the kernels are written for
constexpr int kBlock = 256;         // threads per workgroup of the streaming kernels (4 wave64)

// How one decode call is cut into workgroups.  Derived from the sizes alone, so the workspace query and the
// call itself always agree.
struct DecodePlan {
    int cs;          // tokens per workgroup of the score kernel
    int n_cs;        // score chunks per (b, cluster) = ceil(T / cs)
    int n_rec;       // softmax-statistics records per (b, cluster): one per wave of every score workgroup
    int cp;          // tokens per workgroup of the value kernel
    int n_cp;        // value chunks per (b, head) = ceil(T / cp)
    int ds;          // workgroups per (b, head, chunk) of the value kernel: 1, or 2 with half of the columns each
    size_t off_scores, off_stats, off_partial, off_rows, bytes;   // off_rows: [B,H,128] fp32 staging rows
};

// column_split = false: never cut rows into column parts (caches whose rows are a single cache line)
DecodePlan make_decode_plan(int B, int H, int k, int T, bool column_split = true);

// Kernels that use more than 64 KB of dynamic LDS must be told so once on every device they run on.  `done` is the
// caller's per-kernel table (zero-initialised, one flag per device ordinal); a repeated call costs one hipGetDevice.
// The flags are atomics: any thread may call; setting the attribute twice in a race is harmless.
constexpr int kMaxDevices = 64;
typedef std::atomic<bool> DeviceFlags[kMaxDevices];
inline hipError_t allow_dynamic_lds(const void *kernel, size_t bytes, DeviceFlags &done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < kMaxDevices && done[dev].load(std::memory_order_acquire)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess && dev >= 0 && dev < kMaxDevices) done[dev].store(true, std::memory_order_release);
    return e;
}

// Optional events the runtime stamps with the begin and the end of a kernel (NULL = not wanted).
struct KernelEvents {
    hipEvent_t start = nullptr;
    hipEvent_t stop = nullptr;
};

// Kernel launch that reports the status of THIS launch: the return value of the runtime's launch call, not the
// thread's sticky "last error" (which may hold, and would clear, an unrelated earlier error of the caller).
// Arguments are converted to the kernel's own parameter types; the events may be NULL.
template <typename T>
struct same_type {
    typedef T type;
};
template <typename... KArgs>
inline hipError_t launch_kernel(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream,
                                const KernelEvents &ev, typename same_type<KArgs>::type... args)
{
    void *argv[] = {const_cast<void *>(static_cast<const void *>(&args))...};
    return hipExtLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, argv, lds_bytes, stream, ev.start,
                              ev.stop, 0);
}

// Enqueue the two kernels of one decode call.  identity = true: every head is its own cluster and the maps
// are not read (dense attention).  k_new / v_new [B,H,d] (clustered calls only): position T-1 is the token being
// decoded, its rows are taken from there and written to the caches by the same kernels.  Each returns a
// hipError_t as int.
int launch_scores(const void *q, const void *kc, const int32_t *rep, int B, int H, int k, int T, int Tc_cap,
                  int dtype, float scale, void *workspace, const DecodePlan &plan, bool identity,
                  const KernelEvents &ev, hipStream_t stream, const void *k_new = nullptr);
// members: when set, the H streams of `v` are compact (one per cluster) and the finished row of stream j goes
// to out_members[b][h] of every head h (of n_heads) with head_to_cluster[b][h] == j; `out` is then staging.
struct MemberRows {
    const int32_t *head_to_cluster = nullptr;
    int n_heads = 0;
    float *out_members = nullptr;
};
int launch_values(const void *v, const int32_t *h2c, const int32_t *rep, int B, int H, int k, int T, int T_cap,
                  int dtype, float *out, float *probs_out, void *workspace, const DecodePlan &plan, bool identity,
                  const KernelEvents &ev, hipStream_t stream, const MemberRows *members = nullptr,
                  const void *v_new = nullptr);

// The same two kernels over caches of 8-bit E4M3 codes with one fp32 scale per row; q stays fp32 or bf16 (q_dtype).
// The plan must have been made with column_split = false.
int launch_scores_q8(const void *q, int q_dtype, const void *k8, const float *kscale, const int32_t *rep, int B, int H,
                     int k, int T, int Tc_cap, float scale, void *workspace, const DecodePlan &plan,
                     const KernelEvents &ev, hipStream_t stream);
int launch_values_q8(const void *v8, const float *vscale, const int32_t *h2c, const int32_t *rep, int B, int H, int k,
                     int T, int T_cap, float *out, float *probs_out, void *workspace, const DecodePlan &plan,
                     const KernelEvents &ev, hipStream_t stream);
// rows of 128 elements (fp32 / bf16) -> E4M3 codes + one fp32 scale per row
int launch_quantize_rows(const void *x, int dtype, long long n_rows, uint8_t *codes, float *scales, hipStream_t stream);
int launch_append_kv_q8(const void *k_new, const void *v_new, const int32_t *rep, uint8_t *k8, float *kscale, uint8_t *v8,
                        float *vscale, int B, int H, int k, int pos, int Tc_cap, int T_cap, int dtype,
                        hipStream_t stream);

int launch_score_features(const void *q5, const void *k5, int B, int H, int n_tok, int dtype, int64_t qs,
                          int64_t ks, float scale, float *feat, hipStream_t stream);

int launch_assign_clusters(const float *feat, int B, int H, int F, int k, const int32_t *init_heads, int max_iter,
                           int32_t *h2c, int32_t *rep, int32_t *ncl, int32_t *iters, hipStream_t stream);
size_t assign_clusters_lds_bytes(int H, int F, int k);

// sse and rep_out (nearest-to-mean member of every cluster) are optional outputs of the same kernel
int launch_cluster_error(const float *feat, const int32_t *h2c, int B, int H, int F, int k, double *sse,
                         int32_t *rep_out, hipStream_t stream);
size_t cluster_error_lds_bytes(int H, int F, int k);

// Clustered attention over a block of prompt positions (bf16 only).  identity = dense attention.  The events
// cover the main kernel, not the V^T pre-pass or the work list.
int launch_prefill(const void *q, const void *kc, const void *v, const int32_t *h2c, const int32_t *rep, int B,
                   int H, int k, int Tq, int q_start, int Tc_cap, int T_cap, float scale, float *out,
                   void *workspace, bool identity, const KernelEvents &ev, hipStream_t stream);
size_t prefill_workspace_bytes(int B, int H, int k, int n_keys);

// Query and key projections of the representatives (bf16, d = 128, D a multiple of 64); the events cover the kernel.
int launch_project_qk(const void *x, const void *w_q, const void *w_k, const int32_t *rep, int B, int H, int k, int Tn,
                      int D, void *q_out, void *k_compact, int pos0, int Tc_cap, const KernelEvents &ev,
                      hipStream_t stream);

// the matrix pipe alone: `rounds` rounds of 8 MFMAs per wave on operands taken from buf; flops of one launch
int launch_mfma_probe(const void *buf, size_t bytes, int rounds, float *sink, const KernelEvents &ev, hipStream_t stream);
double mfma_probe_flops(int rounds);

// bare streaming read of `bytes` (a multiple of 16) bytes; the events cover the kernel
int launch_stream_read(const void *buf, size_t bytes, float *sink, const KernelEvents &ev, hipStream_t stream);

int launch_compact_kcache(const void *k_full, const int32_t *rep, void *k_compact, int B, int H, int k, int T,
                          int T_cap, int Tc_cap, int dtype, hipStream_t stream);

// Both caches compact (the variant that prunes values too): rows of the representatives only.
int launch_append_kv_shared(const void *k_new, const void *v_new, const int32_t *rep, void *k_compact, void *v_compact,
                            int B, int H, int k, int pos, int Tc_cap, int Tv_cap, int dtype, hipStream_t stream);

int launch_append_kv(const void *k_new, const void *v_new, const int32_t *rep, void *k_compact, void *v_cache, int B,
                     int H, int k, int pos, int Tc_cap, int T_cap, int dtype, hipStream_t stream);

}  // namespace chai
