"""Thin ctypes binding of libchai.so: argument marshalling only.

Every function has the name and the argument order of its C entry point (see include/chai.h) and takes torch
tensors that already live on the GPU; torch provides device memory and the current stream, nothing else.  All
computation happens inside the HIP library.  There is no CPU fallback: if the library is missing, importing
this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libchai.so")

CHAI_OK = 0
CHAI_F32, CHAI_BF16 = 0, 1
STATUS_NAMES = {0: "CHAI_OK", 1: "CHAI_ERR_NULL", 2: "CHAI_ERR_SHAPE", 3: "CHAI_ERR_DTYPE", 4: "CHAI_ERR_WORKSPACE",
                5: "CHAI_ERR_UNSUPPORTED", 6: "CHAI_ERR_HIP", 7: "CHAI_ERR_ALIGN", 8: "CHAI_ERR_STATIC_LIMIT"}
CHAI_STATIC_SCRATCH_BYTES = 32 << 20

EXPORTS = ["chai_version", "chai_status_string", "chai_score_features", "chai_assign_clusters",
           "chai_cluster_error", "chai_pick_cluster_count", "chai_closest_representatives",
           "chai_decode_attention_shared_v", "chai_append_kv_shared_v",
           "chai_compact_kcache", "chai_append_kv", "chai_decode_workspace_bytes", "chai_decode_attention", "chai_decode_step",
           "chai_decode_attention_static", "chai_quantize_rows", "chai_append_kv_q8", "chai_decode_q8_workspace_bytes",
           "chai_decode_attention_q8", "chai_decode_attention_q8_timed",
           "chai_decode_scores", "chai_decode_values", "chai_decode_scores_timed", "chai_decode_values_timed",
           "chai_dense_decode_attention", "chai_prefill_workspace_bytes", "chai_prefill_attention",
           "chai_prefill_attention_timed", "chai_dense_prefill_attention", "chai_project_qk", "chai_project_qk_timed", "chai_stream_read_probe", "chai_mfma_rate_probe"]


class ChaiError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        msg = _lib.chai_status_string(status).decode() if _lib is not None else "?"
        super().__init__(f"{fn}: {STATUS_NAMES.get(status, status)} ({msg})")


def _load(path: str = LIB_PATH) -> ctypes.CDLL:
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is not built; run `python -m paper_2403_08058_amd.build` (there is no fallback path)")
    L = ctypes.CDLL(path)
    vp, ci, cf, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_int64, ctypes.c_size_t
    L.chai_version.restype = ci
    L.chai_status_string.restype = ctypes.c_char_p
    L.chai_status_string.argtypes = [ci]
    L.chai_score_features.argtypes = [vp, vp, ci, ci, ci, ci, ci, i64, i64, cf, vp, vp]
    L.chai_assign_clusters.argtypes = [vp, ci, ci, ci, ci, vp, ci, vp, vp, vp, vp, vp]
    L.chai_cluster_error.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp]
    L.chai_pick_cluster_count.argtypes = [vp, vp, ci, ctypes.c_double, vp]
    L.chai_compact_kcache.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, vp]
    L.chai_append_kv.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, vp]
    L.chai_decode_workspace_bytes.restype = sz
    L.chai_decode_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci]
    L.chai_decode_attention.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, cf, vp, vp, vp, sz, vp]
    L.chai_decode_attention_static.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, cf, vp, vp, vp]
    L.chai_quantize_rows.argtypes = [vp, ci, ctypes.c_longlong, ci, vp, vp, vp]
    L.chai_append_kv_q8.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, vp]
    L.chai_decode_q8_workspace_bytes.restype = sz
    L.chai_decode_q8_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
    L.chai_decode_attention_q8.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, cf, vp, vp, vp, sz, vp]
    L.chai_decode_attention_q8_timed.argtypes = L.chai_decode_attention_q8.argtypes + [vp, vp, vp, vp]
    L.chai_decode_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, cf, vp, vp, sz, vp]
    L.chai_dense_decode_attention.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, cf, vp, vp, sz, vp]
    L.chai_decode_scores.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, cf, vp, sz, vp]
    L.chai_decode_values.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp, vp, vp, sz, vp]
    L.chai_decode_scores_timed.argtypes = L.chai_decode_scores.argtypes + [vp, vp]
    L.chai_decode_values_timed.argtypes = L.chai_decode_values.argtypes + [vp, vp]
    L.chai_closest_representatives.argtypes = [vp, vp, ci, ci, ci, ci, vp, vp]
    L.chai_decode_attention_shared_v.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, cf, vp, vp, sz, vp]
    L.chai_append_kv_shared_v.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, vp]
    L.chai_project_qk.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp, vp, ci, ci, vp]
    L.chai_project_qk_timed.argtypes = L.chai_project_qk.argtypes + [vp, vp]
    L.chai_stream_read_probe.argtypes = [vp, sz, vp, vp, vp, vp]
    L.chai_mfma_rate_probe.argtypes = [vp, sz, ci, vp, ctypes.POINTER(ctypes.c_double), vp, vp, vp]
    L.chai_prefill_workspace_bytes.restype = sz
    L.chai_prefill_workspace_bytes.argtypes = [ci, ci, ci, ci]
    L.chai_prefill_attention.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, ci, cf, vp, vp, sz, vp]
    L.chai_prefill_attention_timed.argtypes = L.chai_prefill_attention.argtypes + [vp, vp]
    L.chai_dense_prefill_attention.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, cf, vp, vp, sz, vp]
    for fn in EXPORTS:
        if fn not in ("chai_status_string", "chai_decode_workspace_bytes", "chai_prefill_workspace_bytes",
                      "chai_decode_q8_workspace_bytes"):
            getattr(L, fn).restype = ci
    return L


_lib: Optional[ctypes.CDLL] = None
_lib = _load()


def lib() -> ctypes.CDLL:
    return _lib


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return CHAI_F32
    if t.dtype == torch.bfloat16:
        return CHAI_BF16
    raise TypeError(f"q/K/V must be float32 or bfloat16, got {t.dtype}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("libchai takes device tensors")
    if not t.is_contiguous():
        raise ValueError("libchai takes contiguous tensors")
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _check(fn: str, status: int) -> None:
    if status != CHAI_OK:
        raise ChaiError(fn, status)


def chai_version() -> int:
    return int(_lib.chai_version())


def chai_status_string(status: int) -> str:
    return _lib.chai_status_string(int(status)).decode()


def chai_score_features(q5, k5, n_tok: int, scale: float, feat=None, stream=None):
    """q5 [B,H,nq,d], k5 [B,H,Tk,d] (nq, Tk >= n_tok; read in place) -> feat [B,H,n_tok*n_tok] fp32."""
    B, H, nq, d = q5.shape
    Tk = k5.shape[2]
    if feat is None:
        feat = torch.empty((B, H, n_tok * n_tok), dtype=torch.float32, device=q5.device)
    _check("chai_score_features",
           _lib.chai_score_features(_ptr(q5), _ptr(k5), B, H, n_tok, d, dtype_code(q5), nq * d, Tk * d, scale,
                                    _ptr(feat), _stream(stream)))
    return feat


def chai_assign_clusters(feat, init_heads, max_iter: int = 50, head_to_cluster=None, rep_heads=None, n_clusters=None,
                         iters=None, stream=None):
    """feat [B,H,F] fp32, init_heads [B,k] int32 -> (head_to_cluster [B,H], rep_heads [B,k], n_clusters [B], iters [B])."""
    B, H, F = feat.shape
    k = init_heads.shape[1]
    dev = feat.device
    head_to_cluster = torch.empty((B, H), dtype=torch.int32, device=dev) if head_to_cluster is None else head_to_cluster
    rep_heads = torch.empty((B, k), dtype=torch.int32, device=dev) if rep_heads is None else rep_heads
    n_clusters = torch.empty((B,), dtype=torch.int32, device=dev) if n_clusters is None else n_clusters
    iters = torch.empty((B,), dtype=torch.int32, device=dev) if iters is None else iters
    _check("chai_assign_clusters",
           _lib.chai_assign_clusters(_ptr(feat), B, H, F, k, _ptr(init_heads), max_iter, _ptr(head_to_cluster),
                                     _ptr(rep_heads), _ptr(n_clusters), _ptr(iters), _stream(stream)))
    return head_to_cluster, rep_heads, n_clusters, iters


def chai_cluster_error(feat, head_to_cluster, k: int, sse=None, stream=None):
    """feat [B,H,F] fp32, head_to_cluster [B,H] int32 -> sse [B] fp64 (device)."""
    B, H, F = feat.shape
    if sse is None:
        sse = torch.empty((B,), dtype=torch.float64, device=feat.device)
    _check("chai_cluster_error",
           _lib.chai_cluster_error(_ptr(feat), _ptr(head_to_cluster), B, H, F, k, _ptr(sse), _stream(stream)))
    return sse


def chai_closest_representatives(feat, head_to_cluster, k: int, rep_heads=None, stream=None):
    """feat [B,H,F] fp32, head_to_cluster [B,H] int32 -> rep_heads [B,k] int32: nearest-to-mean member per cluster."""
    B, H, F = feat.shape
    if rep_heads is None:
        rep_heads = torch.empty((B, k), dtype=torch.int32, device=feat.device)
    _check("chai_closest_representatives",
           _lib.chai_closest_representatives(_ptr(feat), _ptr(head_to_cluster), B, H, F, k, _ptr(rep_heads),
                                             _stream(stream)))
    return rep_heads


def chai_pick_cluster_count(mean_error, ks, tol: float) -> int:
    """Host-side plateau rule on an error curve (sequences of floats / ints)."""
    n = len(ks)
    err = (ctypes.c_double * n)(*[float(e) for e in mean_error])
    kk = (ctypes.c_int32 * n)(*[int(k) for k in ks])
    out = ctypes.c_int32(0)
    _check("chai_pick_cluster_count", _lib.chai_pick_cluster_count(err, kk, n, float(tol), ctypes.byref(out)))
    return int(out.value)


def chai_compact_kcache(k_full, rep_heads, k_compact, T: int, stream=None):
    """k_full [B,H,T_cap,d], rep_heads [B,k] -> first T rows of k_compact [B,k,Tc_cap,d]."""
    B, H, T_cap, d = k_full.shape
    k, Tc_cap = k_compact.shape[1], k_compact.shape[2]
    _check("chai_compact_kcache",
           _lib.chai_compact_kcache(_ptr(k_full), _ptr(rep_heads), _ptr(k_compact), B, H, k, T, T_cap, Tc_cap, d,
                                    dtype_code(k_full), _stream(stream)))
    return k_compact


def chai_append_kv(k_new, v_new, rep_heads, k_compact, v_cache, pos: int, stream=None):
    B, H, d = k_new.shape
    k, Tc_cap = k_compact.shape[1], k_compact.shape[2]
    T_cap = v_cache.shape[2]
    _check("chai_append_kv",
           _lib.chai_append_kv(_ptr(k_new), _ptr(v_new), _ptr(rep_heads), _ptr(k_compact), _ptr(v_cache), B, H, k, pos,
                               Tc_cap, T_cap, d, dtype_code(k_new), _stream(stream)))


def chai_append_kv_shared_v(k_new, v_new, rep_heads, k_compact, v_compact, pos: int, stream=None):
    B, H, d = k_new.shape
    k, Tc_cap = k_compact.shape[1], k_compact.shape[2]
    Tv_cap = v_compact.shape[2]
    _check("chai_append_kv_shared_v",
           _lib.chai_append_kv_shared_v(_ptr(k_new), _ptr(v_new), _ptr(rep_heads), _ptr(k_compact), _ptr(v_compact), B,
                                        H, k, pos, Tc_cap, Tv_cap, d, dtype_code(k_new), _stream(stream)))


def chai_decode_attention_shared_v(q, k_compact, v_compact, head_to_cluster, rep_heads, T: int, scale: float, out,
                                   workspace, stream=None):
    """The variant that prunes values too: q [B,H,d], k_compact / v_compact [B,k,cap,d] -> out [B,H,d] fp32."""
    B, H, d = q.shape
    k, Tc_cap = k_compact.shape[1], k_compact.shape[2]
    Tv_cap = v_compact.shape[2]
    _check("chai_decode_attention_shared_v",
           _lib.chai_decode_attention_shared_v(_ptr(q), _ptr(k_compact), _ptr(v_compact), _ptr(head_to_cluster),
                                               _ptr(rep_heads), B, H, k, T, Tc_cap, Tv_cap, d, dtype_code(q), scale,
                                               _ptr(out), _ptr(workspace),
                                               workspace.numel() * workspace.element_size(), _stream(stream)))
    return out


def chai_project_qk_timed(x, w_q, w_k, rep_heads, q_out, k_compact, pos0: int, stream=None, start_event=None,
                          stop_event=None):
    """x [B,Tn,D], w_q / w_k [H*d, D], rep_heads [B,k] -> rows of representatives of q_out [B,H,Tn,d] and rows
    pos0.. of k_compact [B,k,Tc_cap,d] (all bf16).  Events: raw hipEvent_t handles or None."""
    B, Tn, D = x.shape
    H, d = q_out.shape[1], q_out.shape[3]
    k, Tc_cap = k_compact.shape[1], k_compact.shape[2]
    _check("chai_project_qk_timed",
           _lib.chai_project_qk_timed(_ptr(x), _ptr(w_q), _ptr(w_k), _ptr(rep_heads), B, H, k, Tn, D, d, dtype_code(x),
                                      _ptr(q_out), _ptr(k_compact), pos0, Tc_cap, _stream(stream), start_event,
                                      stop_event))


def chai_project_qk(x, w_q, w_k, rep_heads, q_out, k_compact, pos0: int, stream=None):
    B, Tn, D = x.shape
    H, d = q_out.shape[1], q_out.shape[3]
    k, Tc_cap = k_compact.shape[1], k_compact.shape[2]
    _check("chai_project_qk",
           _lib.chai_project_qk(_ptr(x), _ptr(w_q), _ptr(w_k), _ptr(rep_heads), B, H, k, Tn, D, d, dtype_code(x),
                                _ptr(q_out), _ptr(k_compact), pos0, Tc_cap, _stream(stream)))


def chai_mfma_rate_probe(buf, rounds: int, sink, stream=None, start_event=None, stop_event=None) -> float:
    """The matrix pipe alone on operands taken from `buf` (measurement aid); returns the flops of the launch."""
    flops = ctypes.c_double(0.0)
    _check("chai_mfma_rate_probe",
           _lib.chai_mfma_rate_probe(_ptr(buf), buf.numel() * buf.element_size(), rounds, _ptr(sink), ctypes.byref(flops),
                                     _stream(stream), start_event, stop_event))
    return float(flops.value)


def chai_stream_read_probe(buf, sink, nbytes: Optional[int] = None, stream=None, start_event=None, stop_event=None):
    """Bare streaming read of a device tensor (measurement aid); sink: one fp32 on the device."""
    n = buf.numel() * buf.element_size() if nbytes is None else nbytes
    _check("chai_stream_read_probe",
           _lib.chai_stream_read_probe(_ptr(buf), n, _ptr(sink), _stream(stream), start_event, stop_event))


def chai_decode_workspace_bytes(B: int, H: int, k: int, T: int, d: int, dtype: int) -> int:
    return int(_lib.chai_decode_workspace_bytes(B, H, k, T, d, dtype))


def chai_decode_attention(q, k_compact, v_cache, head_to_cluster, rep_heads, T: int, scale: float, out, workspace,
                          probs_out=None, stream=None):
    """One clustered decode step of one layer; `out` [B,H,d] fp32 and `workspace` (uint8) are caller-provided."""
    B, H, d = q.shape
    k, Tc_cap = k_compact.shape[1], k_compact.shape[2]
    T_cap = v_cache.shape[2]
    _check("chai_decode_attention",
           _lib.chai_decode_attention(_ptr(q), _ptr(k_compact), _ptr(v_cache), _ptr(head_to_cluster), _ptr(rep_heads),
                                      B, H, k, T, Tc_cap, T_cap, d, dtype_code(q), scale, _ptr(out), _ptr(probs_out),
                                      _ptr(workspace), workspace.numel() * workspace.element_size(),
                                      _stream(stream)))
    return out


def chai_decode_attention_static(q, k_compact, v_cache, head_to_cluster, rep_heads, T: int, scale: float, out,
                                 probs_out=None, stream=None):
    """chai_decode_attention without a workspace: scratch is a fixed array inside the library (no allocation)."""
    B, H, d = q.shape
    k, Tc_cap = k_compact.shape[1], k_compact.shape[2]
    T_cap = v_cache.shape[2]
    _check("chai_decode_attention_static",
           _lib.chai_decode_attention_static(_ptr(q), _ptr(k_compact), _ptr(v_cache), _ptr(head_to_cluster),
                                             _ptr(rep_heads), B, H, k, T, Tc_cap, T_cap, d, dtype_code(q), scale,
                                             _ptr(out), _ptr(probs_out), _stream(stream)))
    return out


def chai_quantize_rows(x, codes=None, scales=None, stream=None):
    """x [..., 128] fp32 or bf16 -> (codes uint8 [..., 128], scales fp32 [...]): E4M3 codes, one scale per row."""
    d = x.shape[-1]
    n_rows = x.numel() // d
    if codes is None:
        codes = torch.empty(x.shape, dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty(x.shape[:-1], dtype=torch.float32, device=x.device)
    _check("chai_quantize_rows",
           _lib.chai_quantize_rows(_ptr(x), dtype_code(x), n_rows, d, _ptr(codes), _ptr(scales), _stream(stream)))
    return codes, scales


def chai_append_kv_q8(k_new, v_new, rep_heads, k8, kscale, v8, vscale, pos: int, stream=None):
    """Quantise the new token's rows into the 8-bit caches: k8 [B,k,Tc_cap,d] + kscale [B,k,Tc_cap], v8 [B,H,T_cap,d] +
    vscale [B,H,T_cap]."""
    B, H, d = k_new.shape
    k, Tc_cap = k8.shape[1], k8.shape[2]
    T_cap = v8.shape[2]
    _check("chai_append_kv_q8",
           _lib.chai_append_kv_q8(_ptr(k_new), _ptr(v_new), _ptr(rep_heads), _ptr(k8), _ptr(kscale), _ptr(v8), _ptr(vscale),
                                  B, H, k, pos, Tc_cap, T_cap, d, dtype_code(k_new), _stream(stream)))


def chai_decode_q8_workspace_bytes(B: int, H: int, k: int, T: int, d: int = 128) -> int:
    return int(_lib.chai_decode_q8_workspace_bytes(B, H, k, T, d))


def chai_decode_attention_q8_timed(q, k8, kscale, v8, vscale, head_to_cluster, rep_heads, T: int, scale: float, out,
                                   workspace, probs_out=None, stream=None, score_events=(None, None),
                                   value_events=(None, None)):
    """chai_decode_attention over caches of E4M3 codes with per-row scales; events: raw hipEvent_t handles or None."""
    B, H, d = q.shape
    k, Tc_cap = k8.shape[1], k8.shape[2]
    T_cap = v8.shape[2]
    _check("chai_decode_attention_q8",
           _lib.chai_decode_attention_q8_timed(_ptr(q), _ptr(k8), _ptr(kscale), _ptr(v8), _ptr(vscale),
                                               _ptr(head_to_cluster), _ptr(rep_heads), B, H, k, T, Tc_cap, T_cap, d,
                                               dtype_code(q), scale, _ptr(out), _ptr(probs_out), _ptr(workspace),
                                               workspace.numel() * workspace.element_size(), _stream(stream),
                                               score_events[0], score_events[1], value_events[0], value_events[1]))
    return out


def chai_decode_attention_q8(q, k8, kscale, v8, vscale, head_to_cluster, rep_heads, T: int, scale: float, out, workspace,
                             probs_out=None, stream=None):
    B, H, d = q.shape
    k, Tc_cap = k8.shape[1], k8.shape[2]
    T_cap = v8.shape[2]
    _check("chai_decode_attention_q8",
           _lib.chai_decode_attention_q8(_ptr(q), _ptr(k8), _ptr(kscale), _ptr(v8), _ptr(vscale), _ptr(head_to_cluster),
                                         _ptr(rep_heads), B, H, k, T, Tc_cap, T_cap, d, dtype_code(q), scale, _ptr(out),
                                         _ptr(probs_out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                         _stream(stream)))
    return out


def chai_decode_step(q, k_new, v_new, k_compact, v_cache, head_to_cluster, rep_heads, T: int, scale: float, out,
                     workspace, stream=None):
    """Cache growth + clustered decode in one call: row T-1 of both caches is taken from k_new / v_new [B,H,d]."""
    B, H, d = q.shape
    k, Tc_cap = k_compact.shape[1], k_compact.shape[2]
    T_cap = v_cache.shape[2]
    _check("chai_decode_step",
           _lib.chai_decode_step(_ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_compact), _ptr(v_cache),
                                 _ptr(head_to_cluster), _ptr(rep_heads), B, H, k, T, Tc_cap, T_cap, d, dtype_code(q),
                                 scale, _ptr(out), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                 _stream(stream)))
    return out


def chai_decode_scores_timed(q, k_compact, rep_heads, T: int, scale: float, workspace, stream=None, start_event=None,
                             stop_event=None):
    """First phase of chai_decode_attention: scores and chunk statistics of every cluster into the workspace.
    start_event / stop_event: raw hipEvent_t handles (ints) stamped with the kernel's begin and end, or None."""
    B, H, d = q.shape
    k, Tc_cap = k_compact.shape[1], k_compact.shape[2]
    _check("chai_decode_scores_timed",
           _lib.chai_decode_scores_timed(_ptr(q), _ptr(k_compact), _ptr(rep_heads), B, H, k, T, Tc_cap, d,
                                         dtype_code(q), scale, _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream), start_event,
                                         stop_event))


def chai_decode_values_timed(v_cache, head_to_cluster, rep_heads, T: int, out, workspace, probs_out=None, stream=None,
                             start_event=None, stop_event=None):
    """Second phase of chai_decode_attention: probabilities from the workspace applied to every head's values."""
    B, H, T_cap, d = v_cache.shape
    k = rep_heads.shape[1]
    _check("chai_decode_values_timed",
           _lib.chai_decode_values_timed(_ptr(v_cache), _ptr(head_to_cluster), _ptr(rep_heads), B, H, k, T, T_cap, d,
                                         dtype_code(v_cache), _ptr(out), _ptr(probs_out), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream), start_event,
                                         stop_event))
    return out


def chai_decode_scores(q, k_compact, rep_heads, T: int, scale: float, workspace, stream=None):
    B, H, d = q.shape
    k, Tc_cap = k_compact.shape[1], k_compact.shape[2]
    _check("chai_decode_scores",
           _lib.chai_decode_scores(_ptr(q), _ptr(k_compact), _ptr(rep_heads), B, H, k, T, Tc_cap, d, dtype_code(q),
                                   scale, _ptr(workspace), workspace.numel() * workspace.element_size(),
                                   _stream(stream)))


def chai_decode_values(v_cache, head_to_cluster, rep_heads, T: int, out, workspace, probs_out=None, stream=None):
    B, H, T_cap, d = v_cache.shape
    k = rep_heads.shape[1]
    _check("chai_decode_values",
           _lib.chai_decode_values(_ptr(v_cache), _ptr(head_to_cluster), _ptr(rep_heads), B, H, k, T, T_cap, d,
                                   dtype_code(v_cache), _ptr(out), _ptr(probs_out), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream(stream)))
    return out


def chai_dense_decode_attention(q, k_cache, v_cache, T: int, scale: float, out, workspace, stream=None):
    B, H, d = q.shape
    T_cap = k_cache.shape[2]
    _check("chai_dense_decode_attention",
           _lib.chai_dense_decode_attention(_ptr(q), _ptr(k_cache), _ptr(v_cache), B, H, T, T_cap, d, dtype_code(q),
                                            scale, _ptr(out), _ptr(workspace),
                                            workspace.numel() * workspace.element_size(), _stream(stream)))
    return out


def chai_prefill_workspace_bytes(B: int, H: int, k: int, n_keys: int) -> int:
    """n_keys = q_start + Tq, the number of cached positions the block sees."""
    return int(_lib.chai_prefill_workspace_bytes(B, H, k, n_keys))


def chai_prefill_attention_timed(q, k_compact, v_cache, head_to_cluster, rep_heads, q_start: int, scale: float, out,
                                 workspace, stream=None, start_event=None, stop_event=None):
    """q [B,H,Tq,d] (rows at positions q_start..), k_compact [B,k,Tc_cap,d], v_cache [B,H,T_cap,d] -> out [B,H,Tq,d] fp32.
    start_event / stop_event: raw hipEvent_t handles (ints) stamped with the main kernel's begin and end, or None."""
    B, H, Tq, d = q.shape
    k, Tc_cap = k_compact.shape[1], k_compact.shape[2]
    T_cap = v_cache.shape[2]
    _check("chai_prefill_attention_timed",
           _lib.chai_prefill_attention_timed(_ptr(q), _ptr(k_compact), _ptr(v_cache), _ptr(head_to_cluster),
                                             _ptr(rep_heads), B, H, k, Tq, q_start, Tc_cap, T_cap, d, dtype_code(q),
                                             scale, _ptr(out), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream(stream),
                                             start_event, stop_event))
    return out


def chai_prefill_attention(q, k_compact, v_cache, head_to_cluster, rep_heads, q_start: int, scale: float, out,
                           workspace, stream=None):
    B, H, Tq, d = q.shape
    k, Tc_cap = k_compact.shape[1], k_compact.shape[2]
    T_cap = v_cache.shape[2]
    _check("chai_prefill_attention",
           _lib.chai_prefill_attention(_ptr(q), _ptr(k_compact), _ptr(v_cache), _ptr(head_to_cluster), _ptr(rep_heads),
                                       B, H, k, Tq, q_start, Tc_cap, T_cap, d, dtype_code(q), scale, _ptr(out),
                                       _ptr(workspace), workspace.numel() * workspace.element_size(),
                                       _stream(stream)))
    return out


def chai_dense_prefill_attention(q, k_cache, v_cache, q_start: int, scale: float, out, workspace, stream=None):
    B, H, Tq, d = q.shape
    T_cap = k_cache.shape[2]
    _check("chai_dense_prefill_attention",
           _lib.chai_dense_prefill_attention(_ptr(q), _ptr(k_cache), _ptr(v_cache), B, H, Tq, q_start, T_cap, d,
                                             dtype_code(q), scale, _ptr(out), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream(stream)))
    return out


def alloc_workspace(B: int, H: int, k: int, T: int, d: int, dtype: int, device="cuda") -> torch.Tensor:
    """Device scratch of the size the decode calls ask for (torch allocations are 512-byte aligned)."""
    n = max(chai_decode_workspace_bytes(B, H, k, T, d, dtype), 256)
    return torch.empty((n,), dtype=torch.uint8, device=device)
