// extern "C" entry points of libchai.so: host-side argument checks, then kernel launches.  Nothing here
// allocates, synchronises or reads device memory.
#include "chai_internal.h"

#include <mutex>

using namespace chai;

// Scratch of chai_decode_attention_static: a fixed array inside the library's code object, so the entry point
// needs no workspace from the caller and no allocation.  Every GPU the library runs on holds its own copy (at
// its own address) until the process ends.  In host code the NAME below is only a handle for
// hipGetSymbolAddress; kernels get the looked-up device address.
static __device__ __align__(256) unsigned char scratch[CHAI_STATIC_SCRATCH_BYTES];

namespace {

std::mutex g_scratch_lock;
void *g_scratch_ptr[kMaxDevices];      // device address of `scratch` on each device, looked up once

// Address of the current device's copy of `scratch` (first call on a device looks it up; no allocation).
hipError_t static_scratch(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (g_scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

constexpr int kVersion = 100;
constexpr int kMaxGridYZ = 65535;

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool bad_dtype(int dtype) { return dtype != CHAI_F32 && dtype != CHAI_BF16; }
inline int hip_status(int e) { return e == (int)hipSuccess ? CHAI_OK : CHAI_ERR_HIP; }

// size checks common to every decode entry point; fills the launch plan
int check_sizes(int B, int H, int k, int T, int Tc_cap, int T_cap, int d, int dtype, const void *workspace,
                size_t workspace_bytes, DecodePlan *plan)
{
    if (bad_dtype(dtype)) return CHAI_ERR_DTYPE;
    if (B < 0 || H < 1 || k < 1 || k > H || T < 1 || T > T_cap || T > Tc_cap || d < 1) return CHAI_ERR_SHAPE;
    if (d != kHeadDim || B > kMaxGridYZ || H > kMaxGridYZ) return CHAI_ERR_UNSUPPORTED;
    *plan = make_decode_plan(B, H, k, T);
    if (B > 0 && (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || workspace_bytes < plan->bytes))
        return CHAI_ERR_WORKSPACE;
    return CHAI_OK;
}

int check_scores(const void *q, const void *kc, int B, int H, int k, int T, int Tc_cap, int d, int dtype,
                 const void *workspace, size_t workspace_bytes, DecodePlan *plan)
{
    if (!q || !kc) return CHAI_ERR_NULL;
    const int st = check_sizes(B, H, k, T, Tc_cap, T, d, dtype, workspace, workspace_bytes, plan);
    if (st != CHAI_OK && st != CHAI_ERR_WORKSPACE) return st;
    if (!aligned16(q) || !aligned16(kc)) return CHAI_ERR_ALIGN;
    return st;
}

int check_values(const void *v, const float *out, int B, int H, int k, int T, int T_cap, int d, int dtype,
                 const void *workspace, size_t workspace_bytes, DecodePlan *plan)
{
    if (!v || !out) return CHAI_ERR_NULL;
    const int st = check_sizes(B, H, k, T, T, T_cap, d, dtype, workspace, workspace_bytes, plan);
    if (st != CHAI_OK && st != CHAI_ERR_WORKSPACE) return st;
    if (!aligned16(v) || !aligned16(out)) return CHAI_ERR_ALIGN;
    return st;
}

}  // namespace

extern "C" {

int chai_version(void) { return kVersion; }

const char *chai_status_string(int status)
{
    switch (status) {
    case CHAI_OK: return "ok";
    case CHAI_ERR_NULL: return "a required pointer is NULL";
    case CHAI_ERR_SHAPE: return "a size is out of range or inconsistent";
    case CHAI_ERR_DTYPE: return "unknown dtype";
    case CHAI_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case CHAI_ERR_UNSUPPORTED: return "sizes not supported by this build";
    case CHAI_ERR_HIP: return "HIP runtime error at kernel launch";
    case CHAI_ERR_ALIGN: return "tensor pointer not 16-byte aligned";
    case CHAI_ERR_STATIC_LIMIT: return "sizes need more scratch than the library's static buffer holds";
    default: return "unknown status";
    }
}

int chai_score_features(const void *q5, const void *k5, int B, int H, int n_tok, int d, int dtype,
                        int64_t q_head_stride, int64_t k_head_stride, float scale, float *feat, void *stream)
{
    if (!q5 || !k5 || !feat) return CHAI_ERR_NULL;
    if (bad_dtype(dtype)) return CHAI_ERR_DTYPE;
    if (B < 0 || H < 1 || n_tok < 1 || d < 1) return CHAI_ERR_SHAPE;
    if (q_head_stride < (int64_t)n_tok * d || k_head_stride < (int64_t)n_tok * d) return CHAI_ERR_SHAPE;
    if ((q_head_stride & 7) || (k_head_stride & 7)) return CHAI_ERR_SHAPE;
    if (d != kHeadDim || n_tok > 8 || B > kMaxGridYZ) return CHAI_ERR_UNSUPPORTED;
    if (!aligned16(q5) || !aligned16(k5)) return CHAI_ERR_ALIGN;
    if (B == 0) return CHAI_OK;
    return hip_status(launch_score_features(q5, k5, B, H, n_tok, dtype, q_head_stride, k_head_stride, scale, feat,
                                            static_cast<hipStream_t>(stream)));
}

int chai_assign_clusters(const float *feat, int B, int H, int F, int k, const int32_t *init_heads, int max_iter,
                         int32_t *head_to_cluster, int32_t *rep_heads, int32_t *n_clusters, int32_t *iters,
                         void *stream)
{
    if (!feat || !init_heads || !head_to_cluster || !rep_heads || !n_clusters) return CHAI_ERR_NULL;
    if (B < 0 || H < 1 || F < 1 || k < 1 || k > H || max_iter < 1) return CHAI_ERR_SHAPE;
    if (H > 256 || F > 64 || (long long)k * F > 7168) return CHAI_ERR_UNSUPPORTED;
    if (assign_clusters_lds_bytes(H, F, k) > 64 * 1024 - 64) return CHAI_ERR_UNSUPPORTED;
    if (B == 0) return CHAI_OK;
    return hip_status(launch_assign_clusters(feat, B, H, F, k, init_heads, max_iter, head_to_cluster, rep_heads,
                                             n_clusters, iters, static_cast<hipStream_t>(stream)));
}

int chai_cluster_error(const float *feat, const int32_t *head_to_cluster, int B, int H, int F, int k, double *sse,
                       void *stream)
{
    if (!feat || !head_to_cluster || !sse) return CHAI_ERR_NULL;
    if (B < 0 || H < 1 || F < 1 || k < 1 || k > H) return CHAI_ERR_SHAPE;
    if (H > 256 || F > 64 || (long long)k * F > 7168) return CHAI_ERR_UNSUPPORTED;
    if (cluster_error_lds_bytes(H, F, k) > 64 * 1024 - 64) return CHAI_ERR_UNSUPPORTED;
    if (B == 0) return CHAI_OK;
    return hip_status(launch_cluster_error(feat, head_to_cluster, B, H, F, k, sse, nullptr,
                                           static_cast<hipStream_t>(stream)));
}

int chai_closest_representatives(const float *feat, const int32_t *head_to_cluster, int B, int H, int F, int k,
                                 int32_t *rep_heads, void *stream)
{
    if (!feat || !head_to_cluster || !rep_heads) return CHAI_ERR_NULL;
    if (B < 0 || H < 1 || F < 1 || k < 1 || k > H) return CHAI_ERR_SHAPE;
    if (H > 256 || F > 64 || (long long)k * F > 7168) return CHAI_ERR_UNSUPPORTED;
    if (cluster_error_lds_bytes(H, F, k) > 64 * 1024 - 64) return CHAI_ERR_UNSUPPORTED;
    if (B == 0) return CHAI_OK;
    return hip_status(launch_cluster_error(feat, head_to_cluster, B, H, F, k, nullptr, rep_heads,
                                           static_cast<hipStream_t>(stream)));
}

int chai_pick_cluster_count(const double *mean_error, const int32_t *ks, int n, double tol, int32_t *k_out)
{
    if (!mean_error || !ks || !k_out) return CHAI_ERR_NULL;
    if (n < 1 || !(tol >= 0.0)) return CHAI_ERR_SHAPE;
    for (int i = 1; i < n; ++i)
        if (ks[i] <= ks[i - 1]) return CHAI_ERR_SHAPE;
    const double floor_err = mean_error[n - 1];
    const double slack = tol * (mean_error[0] - floor_err);
    int pick = ks[n - 1];
    for (int i = 0; i < n; ++i) {
        if (mean_error[i] - floor_err <= slack) { pick = ks[i]; break; }
    }
    *k_out = pick;
    return CHAI_OK;
}

int chai_compact_kcache(const void *k_full, const int32_t *rep_heads, void *k_compact, int B, int H, int k, int T,
                        int T_cap, int Tc_cap, int d, int dtype, void *stream)
{
    if (!k_full || !rep_heads || !k_compact) return CHAI_ERR_NULL;
    if (bad_dtype(dtype)) return CHAI_ERR_DTYPE;
    if (B < 0 || H < 1 || k < 1 || k > H || T < 0 || T > T_cap || T > Tc_cap || d < 1) return CHAI_ERR_SHAPE;
    if (d != kHeadDim || B > kMaxGridYZ || k > kMaxGridYZ) return CHAI_ERR_UNSUPPORTED;
    if (!aligned16(k_full) || !aligned16(k_compact)) return CHAI_ERR_ALIGN;
    if (B == 0 || T == 0) return CHAI_OK;
    return hip_status(launch_compact_kcache(k_full, rep_heads, k_compact, B, H, k, T, T_cap, Tc_cap, dtype,
                                            static_cast<hipStream_t>(stream)));
}

int chai_append_kv(const void *k_new, const void *v_new, const int32_t *rep_heads, void *k_compact, void *v_cache,
                   int B, int H, int k, int pos, int Tc_cap, int T_cap, int d, int dtype, void *stream)
{
    if (!k_new || !v_new || !rep_heads || !k_compact || !v_cache) return CHAI_ERR_NULL;
    if (bad_dtype(dtype)) return CHAI_ERR_DTYPE;
    if (B < 0 || H < 1 || k < 1 || k > H || pos < 0 || pos >= T_cap || pos >= Tc_cap || d < 1) return CHAI_ERR_SHAPE;
    if (d != kHeadDim || B > kMaxGridYZ) return CHAI_ERR_UNSUPPORTED;
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_compact) || !aligned16(v_cache)) return CHAI_ERR_ALIGN;
    if (B == 0) return CHAI_OK;
    return hip_status(launch_append_kv(k_new, v_new, rep_heads, k_compact, v_cache, B, H, k, pos, Tc_cap, T_cap,
                                       dtype, static_cast<hipStream_t>(stream)));
}

int chai_mfma_rate_probe(const void *buf, size_t bytes, int rounds, float *sink, double *flops, void *stream,
                         void *start_event, void *stop_event)
{
    if (!buf || !sink) return CHAI_ERR_NULL;
    if (bytes < 16 || rounds < 1) return CHAI_ERR_SHAPE;
    if (!aligned16(buf)) return CHAI_ERR_ALIGN;
    if (flops) *flops = mfma_probe_flops(rounds);
    KernelEvents ev;
    ev.start = static_cast<hipEvent_t>(start_event);
    ev.stop = static_cast<hipEvent_t>(stop_event);
    return hip_status(launch_mfma_probe(buf, bytes, rounds, sink, ev, static_cast<hipStream_t>(stream)));
}

int chai_stream_read_probe(const void *buf, size_t bytes, float *sink, void *stream, void *start_event,
                           void *stop_event)
{
    if (!buf || !sink) return CHAI_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0) return CHAI_ERR_SHAPE;
    if (bytes > ((size_t)1 << 40)) return CHAI_ERR_UNSUPPORTED;
    if (!aligned16(buf)) return CHAI_ERR_ALIGN;
    KernelEvents ev;
    ev.start = static_cast<hipEvent_t>(start_event);
    ev.stop = static_cast<hipEvent_t>(stop_event);
    return hip_status(launch_stream_read(buf, bytes, sink, ev, static_cast<hipStream_t>(stream)));
}

size_t chai_decode_workspace_bytes(int B, int H, int k, int T, int d, int dtype)
{
    if (B < 0 || H < 1 || k < 1 || k > H || T < 1 || d != kHeadDim || bad_dtype(dtype)) return 0;
    if (B == 0) return 256;
    return make_decode_plan(B, H, k, T).bytes;
}

int chai_decode_scores_timed(const void *q, const void *k_compact, const int32_t *rep_heads, int B, int H, int k,
                             int T, int Tc_cap, int d, int dtype, float scale, void *workspace,
                             size_t workspace_bytes, void *stream, void *start_event, void *stop_event)
{
    if (!rep_heads) return CHAI_ERR_NULL;
    DecodePlan plan;
    const int st = check_scores(q, k_compact, B, H, k, T, Tc_cap, d, dtype, workspace, workspace_bytes, &plan);
    if (st != CHAI_OK) return st;
    if (B == 0) return CHAI_OK;
    KernelEvents ev;
    ev.start = static_cast<hipEvent_t>(start_event);
    ev.stop = static_cast<hipEvent_t>(stop_event);
    return hip_status(launch_scores(q, k_compact, rep_heads, B, H, k, T, Tc_cap, dtype, scale, workspace, plan, false,
                                    ev, static_cast<hipStream_t>(stream)));
}

int chai_decode_values_timed(const void *v_cache, const int32_t *head_to_cluster, const int32_t *rep_heads, int B,
                             int H, int k, int T, int T_cap, int d, int dtype, float *out, float *probs_out,
                             void *workspace, size_t workspace_bytes, void *stream, void *start_event,
                             void *stop_event)
{
    if (!head_to_cluster || !rep_heads) return CHAI_ERR_NULL;
    DecodePlan plan;
    const int st = check_values(v_cache, out, B, H, k, T, T_cap, d, dtype, workspace, workspace_bytes, &plan);
    if (st != CHAI_OK) return st;
    if (B == 0) return CHAI_OK;
    KernelEvents ev;
    ev.start = static_cast<hipEvent_t>(start_event);
    ev.stop = static_cast<hipEvent_t>(stop_event);
    return hip_status(launch_values(v_cache, head_to_cluster, rep_heads, B, H, k, T, T_cap, dtype, out, probs_out,
                                    workspace, plan, false, ev, static_cast<hipStream_t>(stream)));
}

int chai_decode_scores(const void *q, const void *k_compact, const int32_t *rep_heads, int B, int H, int k, int T,
                       int Tc_cap, int d, int dtype, float scale, void *workspace, size_t workspace_bytes,
                       void *stream)
{
    return chai_decode_scores_timed(q, k_compact, rep_heads, B, H, k, T, Tc_cap, d, dtype, scale, workspace,
                                    workspace_bytes, stream, nullptr, nullptr);
}

int chai_decode_values(const void *v_cache, const int32_t *head_to_cluster, const int32_t *rep_heads, int B, int H,
                       int k, int T, int T_cap, int d, int dtype, float *out, float *probs_out, void *workspace,
                       size_t workspace_bytes, void *stream)
{
    return chai_decode_values_timed(v_cache, head_to_cluster, rep_heads, B, H, k, T, T_cap, d, dtype, out, probs_out,
                                    workspace, workspace_bytes, stream, nullptr, nullptr);
}

int chai_decode_attention(const void *q, const void *k_compact, const void *v_cache, const int32_t *head_to_cluster,
                          const int32_t *rep_heads, int B, int H, int k, int T, int Tc_cap, int T_cap, int d,
                          int dtype, float scale, float *out, float *probs_out, void *workspace,
                          size_t workspace_bytes, void *stream)
{
    if (!head_to_cluster || !rep_heads) return CHAI_ERR_NULL;
    DecodePlan plan;
    int st = check_scores(q, k_compact, B, H, k, T, Tc_cap, d, dtype, workspace, workspace_bytes, &plan);
    if (st == CHAI_OK) st = check_values(v_cache, out, B, H, k, T, T_cap, d, dtype, workspace, workspace_bytes, &plan);
    if (st != CHAI_OK) return st;
    if (B == 0) return CHAI_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = hip_status(launch_scores(q, k_compact, rep_heads, B, H, k, T, Tc_cap, dtype, scale, workspace, plan, false,
                                  KernelEvents(), s));
    if (st != CHAI_OK) return st;
    return hip_status(launch_values(v_cache, head_to_cluster, rep_heads, B, H, k, T, T_cap, dtype, out, probs_out,
                                    workspace, plan, false, KernelEvents(), s));
}

int chai_decode_attention_static(const void *q, const void *k_compact, const void *v_cache,
                                 const int32_t *head_to_cluster, const int32_t *rep_heads, int B, int H, int k, int T,
                                 int Tc_cap, int T_cap, int d, int dtype, float scale, float *out, float *probs_out,
                                 void *stream)
{
    if (!head_to_cluster || !rep_heads) return CHAI_ERR_NULL;
    // sizes first, with a stand-in workspace of the full static size: a plan that needs more is refused here
    DecodePlan plan;
    int st = check_scores(q, k_compact, B, H, k, T, Tc_cap, d, dtype, nullptr, 0, &plan);
    if (st == CHAI_OK || st == CHAI_ERR_WORKSPACE)
        st = check_values(v_cache, out, B, H, k, T, T_cap, d, dtype, nullptr, 0, &plan);
    if (st != CHAI_OK && st != CHAI_ERR_WORKSPACE) return st;
    if (B == 0) return CHAI_OK;
    if (plan.bytes > (size_t)CHAI_STATIC_SCRATCH_BYTES) return CHAI_ERR_STATIC_LIMIT;
    void *ws = nullptr;
    if (static_scratch(&ws) != hipSuccess) return CHAI_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = hip_status(launch_scores(q, k_compact, rep_heads, B, H, k, T, Tc_cap, dtype, scale, ws, plan, false,
                                  KernelEvents(), s));
    if (st != CHAI_OK) return st;
    return hip_status(launch_values(v_cache, head_to_cluster, rep_heads, B, H, k, T, T_cap, dtype, out, probs_out, ws,
                                    plan, false, KernelEvents(), s));
}

int chai_decode_step(const void *q, const void *k_new, const void *v_new, void *k_compact, void *v_cache,
                     const int32_t *head_to_cluster, const int32_t *rep_heads, int B, int H, int k, int T, int Tc_cap,
                     int T_cap, int d, int dtype, float scale, float *out, void *workspace, size_t workspace_bytes,
                     void *stream)
{
    if (!k_new || !v_new || !head_to_cluster || !rep_heads) return CHAI_ERR_NULL;
    DecodePlan plan;
    int st = check_scores(q, k_compact, B, H, k, T, Tc_cap, d, dtype, workspace, workspace_bytes, &plan);
    if (st == CHAI_OK) st = check_values(v_cache, out, B, H, k, T, T_cap, d, dtype, workspace, workspace_bytes, &plan);
    if (st != CHAI_OK) return st;
    if (!aligned16(k_new) || !aligned16(v_new)) return CHAI_ERR_ALIGN;
    if (B == 0) return CHAI_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = hip_status(launch_scores(q, k_compact, rep_heads, B, H, k, T, Tc_cap, dtype, scale, workspace, plan, false,
                                  KernelEvents(), s, k_new));
    if (st != CHAI_OK) return st;
    return hip_status(launch_values(v_cache, head_to_cluster, rep_heads, B, H, k, T, T_cap, dtype, out, nullptr,
                                    workspace, plan, false, KernelEvents(), s, nullptr, v_new));
}

int chai_quantize_rows(const void *x, int dtype, long long n_rows, int d, uint8_t *codes, float *scales, void *stream)
{
    if (!x || !codes || !scales) return CHAI_ERR_NULL;
    if (bad_dtype(dtype)) return CHAI_ERR_DTYPE;
    if (n_rows < 0 || d < 1) return CHAI_ERR_SHAPE;
    if (d != kHeadDim || n_rows > (1LL << 34)) return CHAI_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(codes)) return CHAI_ERR_ALIGN;
    if (n_rows == 0) return CHAI_OK;
    return hip_status(launch_quantize_rows(x, dtype, n_rows, codes, scales, static_cast<hipStream_t>(stream)));
}

int chai_append_kv_q8(const void *k_new, const void *v_new, const int32_t *rep_heads, uint8_t *k8, float *kscale,
                      uint8_t *v8, float *vscale, int B, int H, int k, int pos, int Tc_cap, int T_cap, int d, int dtype,
                      void *stream)
{
    if (!k_new || !v_new || !rep_heads || !k8 || !kscale || !v8 || !vscale) return CHAI_ERR_NULL;
    if (bad_dtype(dtype)) return CHAI_ERR_DTYPE;
    if (B < 0 || H < 1 || k < 1 || k > H || pos < 0 || pos >= T_cap || pos >= Tc_cap || d < 1) return CHAI_ERR_SHAPE;
    if (d != kHeadDim || B > kMaxGridYZ) return CHAI_ERR_UNSUPPORTED;
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k8) || !aligned16(v8)) return CHAI_ERR_ALIGN;
    if (B == 0) return CHAI_OK;
    return hip_status(launch_append_kv_q8(k_new, v_new, rep_heads, k8, kscale, v8, vscale, B, H, k, pos, Tc_cap, T_cap,
                                          dtype, static_cast<hipStream_t>(stream)));
}

size_t chai_decode_q8_workspace_bytes(int B, int H, int k, int T, int d)
{
    if (B < 0 || H < 1 || k < 1 || k > H || T < 1 || d != kHeadDim) return 0;
    if (B == 0) return 256;
    return make_decode_plan(B, H, k, T, false).bytes;
}

int chai_decode_attention_q8_timed(const void *q, const uint8_t *k8, const float *kscale, const uint8_t *v8,
                                   const float *vscale, const int32_t *head_to_cluster, const int32_t *rep_heads, int B,
                                   int H, int k, int T, int Tc_cap, int T_cap, int d, int q_dtype, float scale,
                                   float *out, float *probs_out, void *workspace, size_t workspace_bytes, void *stream,
                                   void *score_start, void *score_stop, void *value_start, void *value_stop)
{
    if (!q || !k8 || !kscale || !v8 || !vscale || !head_to_cluster || !rep_heads || !out) return CHAI_ERR_NULL;
    if (bad_dtype(q_dtype)) return CHAI_ERR_DTYPE;
    if (B < 0 || H < 1 || k < 1 || k > H || T < 1 || T > T_cap || T > Tc_cap || d < 1) return CHAI_ERR_SHAPE;
    if (d != kHeadDim || B > kMaxGridYZ || H > kMaxGridYZ) return CHAI_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k8) || !aligned16(v8) || !aligned16(out)) return CHAI_ERR_ALIGN;
    const DecodePlan plan = make_decode_plan(B, H, k, T, false);
    if (B > 0 && (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || workspace_bytes < plan.bytes))
        return CHAI_ERR_WORKSPACE;
    if (B == 0) return CHAI_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    KernelEvents es, evv;
    es.start = static_cast<hipEvent_t>(score_start);
    es.stop = static_cast<hipEvent_t>(score_stop);
    evv.start = static_cast<hipEvent_t>(value_start);
    evv.stop = static_cast<hipEvent_t>(value_stop);
    const int st = hip_status(launch_scores_q8(q, q_dtype, k8, kscale, rep_heads, B, H, k, T, Tc_cap, scale, workspace,
                                               plan, es, s));
    if (st != CHAI_OK) return st;
    return hip_status(launch_values_q8(v8, vscale, head_to_cluster, rep_heads, B, H, k, T, T_cap, out, probs_out, workspace,
                                       plan, evv, s));
}

int chai_decode_attention_q8(const void *q, const uint8_t *k8, const float *kscale, const uint8_t *v8,
                             const float *vscale, const int32_t *head_to_cluster, const int32_t *rep_heads, int B, int H,
                             int k, int T, int Tc_cap, int T_cap, int d, int q_dtype, float scale, float *out,
                             float *probs_out, void *workspace, size_t workspace_bytes, void *stream)
{
    return chai_decode_attention_q8_timed(q, k8, kscale, v8, vscale, head_to_cluster, rep_heads, B, H, k, T, Tc_cap, T_cap,
                                          d, q_dtype, scale, out, probs_out, workspace, workspace_bytes, stream, nullptr,
                                          nullptr, nullptr, nullptr);
}

int chai_append_kv_shared_v(const void *k_new, const void *v_new, const int32_t *rep_heads, void *k_compact,
                            void *v_compact, int B, int H, int k, int pos, int Tc_cap, int Tv_cap, int d, int dtype,
                            void *stream)
{
    if (!k_new || !v_new || !rep_heads || !k_compact || !v_compact) return CHAI_ERR_NULL;
    if (bad_dtype(dtype)) return CHAI_ERR_DTYPE;
    if (B < 0 || H < 1 || k < 1 || k > H || pos < 0 || pos >= Tv_cap || pos >= Tc_cap || d < 1) return CHAI_ERR_SHAPE;
    if (d != kHeadDim || B > kMaxGridYZ) return CHAI_ERR_UNSUPPORTED;
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_compact) || !aligned16(v_compact)) return CHAI_ERR_ALIGN;
    if (B == 0) return CHAI_OK;
    return hip_status(launch_append_kv_shared(k_new, v_new, rep_heads, k_compact, v_compact, B, H, k, pos, Tc_cap,
                                              Tv_cap, dtype, static_cast<hipStream_t>(stream)));
}

int chai_decode_attention_shared_v(const void *q, const void *k_compact, const void *v_compact,
                                   const int32_t *head_to_cluster, const int32_t *rep_heads, int B, int H, int k,
                                   int T, int Tc_cap, int Tv_cap, int d, int dtype, float scale, float *out,
                                   void *workspace, size_t workspace_bytes, void *stream)
{
    if (!q || !k_compact || !v_compact || !head_to_cluster || !rep_heads || !out) return CHAI_ERR_NULL;
    if (bad_dtype(dtype)) return CHAI_ERR_DTYPE;
    if (B < 0 || H < 1 || k < 1 || k > H || T < 1 || T > Tc_cap || T > Tv_cap || d < 1) return CHAI_ERR_SHAPE;
    if (d != kHeadDim || B > kMaxGridYZ || H > kMaxGridYZ) return CHAI_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k_compact) || !aligned16(v_compact) || !aligned16(out)) return CHAI_ERR_ALIGN;
    // both caches hold k streams per batch row: the launch plan of k heads in k clusters
    const DecodePlan plan = make_decode_plan(B, k, k, T);
    if (B > 0 && (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || workspace_bytes < plan.bytes))
        return CHAI_ERR_WORKSPACE;
    if (B == 0) return CHAI_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int e = launch_scores(q, k_compact, rep_heads, B, H, k, T, Tc_cap, dtype, scale, workspace, plan, false,
                          KernelEvents{}, s);
    if (e != (int)hipSuccess) return CHAI_ERR_HIP;
    float *rows = reinterpret_cast<float *>(static_cast<char *>(workspace) + plan.off_rows);
    MemberRows members;
    members.head_to_cluster = head_to_cluster;
    members.n_heads = H;
    members.out_members = out;
    return hip_status(launch_values(v_compact, nullptr, nullptr, B, k, k, T, Tv_cap, dtype, rows, nullptr, workspace,
                                    plan, true, KernelEvents{}, s, &members));
}

int chai_dense_decode_attention(const void *q, const void *k_cache, const void *v_cache, int B, int H, int T,
                                int T_cap, int d, int dtype, float scale, float *out, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    DecodePlan plan;
    int st = check_scores(q, k_cache, B, H, H, T, T_cap, d, dtype, workspace, workspace_bytes, &plan);
    if (st == CHAI_OK) st = check_values(v_cache, out, B, H, H, T, T_cap, d, dtype, workspace, workspace_bytes, &plan);
    if (st != CHAI_OK) return st;
    if (B == 0) return CHAI_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    st = hip_status(launch_scores(q, k_cache, nullptr, B, H, H, T, T_cap, dtype, scale, workspace, plan, true,
                                  KernelEvents(), s));
    if (st != CHAI_OK) return st;
    return hip_status(launch_values(v_cache, nullptr, nullptr, B, H, H, T, T_cap, dtype, out, nullptr, workspace, plan,
                                    true, KernelEvents(), s));
}

int chai_project_qk_timed(const void *x, const void *w_q, const void *w_k, const int32_t *rep_heads, int B, int H, int k,
                          int Tn, int D, int d, int dtype, void *q_out, void *k_compact, int pos0, int Tc_cap,
                          void *stream, void *start_event, void *stop_event)
{
    if (!x || !w_q || !w_k || !rep_heads || !q_out || !k_compact) return CHAI_ERR_NULL;
    if (bad_dtype(dtype)) return CHAI_ERR_DTYPE;
    if (B < 0 || H < 1 || k < 1 || k > H || Tn < 1 || D < 1 || d < 1 || pos0 < 0) return CHAI_ERR_SHAPE;
    if ((long long)pos0 + Tn > Tc_cap) return CHAI_ERR_SHAPE;
    if (d != kHeadDim || dtype != CHAI_BF16 || D % 64 != 0 || (long long)Tn * D * 2 >= (1LL << 32) ||
        (long long)kHeadDim * D * 2 >= (1LL << 32))
        return CHAI_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(w_q) || !aligned16(w_k) || !aligned16(q_out) || !aligned16(k_compact))
        return CHAI_ERR_ALIGN;
    if (B == 0) return CHAI_OK;
    KernelEvents ev;
    ev.start = static_cast<hipEvent_t>(start_event);
    ev.stop = static_cast<hipEvent_t>(stop_event);
    return hip_status(launch_project_qk(x, w_q, w_k, rep_heads, B, H, k, Tn, D, q_out, k_compact, pos0, Tc_cap, ev,
                                        static_cast<hipStream_t>(stream)));
}

int chai_project_qk(const void *x, const void *w_q, const void *w_k, const int32_t *rep_heads, int B, int H, int k,
                    int Tn, int D, int d, int dtype, void *q_out, void *k_compact, int pos0, int Tc_cap, void *stream)
{
    return chai_project_qk_timed(x, w_q, w_k, rep_heads, B, H, k, Tn, D, d, dtype, q_out, k_compact, pos0, Tc_cap, stream,
                                 nullptr, nullptr);
}

size_t chai_prefill_workspace_bytes(int B, int H, int k, int n_keys)
{
    if (B < 0 || H < 1 || k < 1 || k > H || n_keys < 1) return 0;
    return prefill_workspace_bytes(B > 0 ? B : 1, H, k, n_keys);
}

static int check_prefill(const void *q, const void *kc, const void *v, const float *out, int B, int H, int k, int Tq,
                         int q_start, int Tc_cap, int T_cap, int d, int dtype, float scale, const void *workspace,
                         size_t workspace_bytes)
{
    if (!q || !kc || !v || !out) return CHAI_ERR_NULL;
    if (bad_dtype(dtype)) return CHAI_ERR_DTYPE;
    if (B < 0 || H < 1 || k < 1 || k > H || Tq < 1 || q_start < 0 || d < 1) return CHAI_ERR_SHAPE;
    if ((long long)q_start + Tq > T_cap || (long long)q_start + Tq > Tc_cap) return CHAI_ERR_SHAPE;
    if (d != kHeadDim || dtype != CHAI_BF16 || B > kMaxGridYZ || H > 4096 || !(scale > 0.f)) return CHAI_ERR_UNSUPPORTED;
    // the kernel addresses one head's keys and transposed values with 32-bit byte offsets below 2 GiB
    if ((long long)q_start + Tq > (1LL << 23) - 64) return CHAI_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(kc) || !aligned16(v) || !aligned16(out)) return CHAI_ERR_ALIGN;
    if (B > 0 && (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 ||
                  workspace_bytes < prefill_workspace_bytes(B, H, k, q_start + Tq)))
        return CHAI_ERR_WORKSPACE;
    return CHAI_OK;
}

int chai_prefill_attention_timed(const void *q, const void *k_compact, const void *v_cache,
                                 const int32_t *head_to_cluster, const int32_t *rep_heads, int B, int H, int k, int Tq,
                                 int q_start, int Tc_cap, int T_cap, int d, int dtype, float scale, float *out,
                                 void *workspace, size_t workspace_bytes, void *stream, void *start_event,
                                 void *stop_event)
{
    if (!head_to_cluster || !rep_heads) return CHAI_ERR_NULL;
    const int st = check_prefill(q, k_compact, v_cache, out, B, H, k, Tq, q_start, Tc_cap, T_cap, d, dtype, scale, workspace,
                                 workspace_bytes);
    if (st != CHAI_OK) return st;
    if (B == 0) return CHAI_OK;
    KernelEvents ev;
    ev.start = static_cast<hipEvent_t>(start_event);
    ev.stop = static_cast<hipEvent_t>(stop_event);
    return hip_status(launch_prefill(q, k_compact, v_cache, head_to_cluster, rep_heads, B, H, k, Tq, q_start, Tc_cap,
                                     T_cap, scale, out, workspace, false, ev, static_cast<hipStream_t>(stream)));
}

int chai_prefill_attention(const void *q, const void *k_compact, const void *v_cache, const int32_t *head_to_cluster,
                           const int32_t *rep_heads, int B, int H, int k, int Tq, int q_start, int Tc_cap, int T_cap,
                           int d, int dtype, float scale, float *out, void *workspace, size_t workspace_bytes,
                           void *stream)
{
    return chai_prefill_attention_timed(q, k_compact, v_cache, head_to_cluster, rep_heads, B, H, k, Tq, q_start, Tc_cap,
                                        T_cap, d, dtype, scale, out, workspace, workspace_bytes, stream, nullptr,
                                        nullptr);
}

int chai_dense_prefill_attention(const void *q, const void *k_cache, const void *v_cache, int B, int H, int Tq,
                                 int q_start, int T_cap, int d, int dtype, float scale, float *out, void *workspace,
                                 size_t workspace_bytes, void *stream)
{
    const int st = check_prefill(q, k_cache, v_cache, out, B, H, H, Tq, q_start, T_cap, T_cap, d, dtype, scale, workspace,
                                 workspace_bytes);
    if (st != CHAI_OK) return st;
    if (B == 0) return CHAI_OK;
    return hip_status(launch_prefill(q, k_cache, v_cache, nullptr, nullptr, B, H, H, Tq, q_start, T_cap, T_cap, scale,
                                     out, workspace, true, KernelEvents{}, static_cast<hipStream_t>(stream)));
}

}  // extern "C"
