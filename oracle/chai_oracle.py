"""ctypes front end of the plain CPU oracle (``chai_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by
the benchmark's ``cpu_baseline`` leg.  Nothing in the product package imports
it, and it imports nothing from the product package.

Arrays are numpy arrays in host memory.  bf16 tensors are ``uint16`` arrays of
raw bit patterns; fp32 tensors are ``float32`` arrays.
"""
from __future__ import annotations

import contextlib
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "chai_oracle.c")
_LIB = os.path.join(_HERE, "libchai_oracle.so")

F32, BF16 = 0, 1
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp contraction off, OpenMP on)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-Wall", "-Wextra", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _configure(L: ctypes.CDLL) -> ctypes.CDLL:
    vp, i32p, i64 = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64
    ci, cd = ctypes.c_int, ctypes.c_double
    L.chai_oracle_num_threads.restype = ci
    L.chai_oracle_clustered_decode.argtypes = [vp, vp, vp, i32p, i32p, ci, ci, ci, ci, ci, ci, ci, cd, vp, vp]
    L.chai_oracle_clustered_prefill.argtypes = [vp, vp, vp, i32p, i32p, ci, ci, ci, ci, ci, ci, ci, ci, cd, vp]
    L.chai_oracle_shared_v_decode.argtypes = [vp, vp, vp, i32p, i32p, ci, ci, ci, ci, ci, ci, ci, cd, vp]
    L.chai_oracle_closest_representatives.argtypes = [vp, i32p, ci, ci, ci, ci, i32p]
    L.chai_oracle_dense_decode.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, cd, vp, vp]
    L.chai_oracle_score_features.argtypes = [vp, vp, ci, ci, ci, ci, ci, i64, i64, cd, vp]
    L.chai_oracle_kmeans.argtypes = [vp, ci, ci, ci, ci, i32p, ci, i32p, i32p, i32p, i32p, vp]
    L.chai_oracle_cluster_error.argtypes = [vp, i32p, ci, ci, ci, ci, vp]
    L.chai_oracle_pick_cluster_count.argtypes = [vp, i32p, ci, cd, vp]
    L.chai_oracle_project_qk.argtypes = [vp, vp, vp, i32p, ci, ci, ci, ci, ci, ci, ci, vp, vp]
    L.chai_oracle_compact_kcache.argtypes = [vp, i32p, vp, ci, ci, ci, ci, ci, ci, ci, ci, vp]
    L.chai_oracle_append_kv.argtypes = [vp, vp, i32p, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci]
    L.chai_oracle_e4m3_decode.argtypes = [ci]
    L.chai_oracle_e4m3_decode.restype = cd
    L.chai_oracle_e4m3_encode.argtypes = [ctypes.c_float]
    L.chai_oracle_e4m3_encode.restype = ci
    L.chai_oracle_quantize_rows.argtypes = [vp, i64, ci, ci, vp, vp]
    L.chai_oracle_dequantize_rows.argtypes = [vp, vp, i64, ci, vp]
    L.chai_oracle_clustered_decode_q8.argtypes = [vp, vp, vp, vp, vp, i32p, i32p, ci, ci, ci, ci, ci, ci, ci, cd, vp, vp]
    return L


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        _lib = _configure(ctypes.CDLL(_LIB))
    return _lib


@contextlib.contextmanager
def use_library(path: str):
    """Route the functions below through another build of the oracle (the tests use this to check that
    deliberately broken copies of the C file are caught by the pins)."""
    global _lib
    saved = _lib
    _lib = _configure(ctypes.CDLL(path))
    try:
        yield
    finally:
        _lib = saved


def num_threads() -> int:
    return int(lib().chai_oracle_num_threads())


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"expected float32 or uint16 (bf16 bits), got {a.dtype}")


def _c(a: np.ndarray, dtype=None) -> np.ndarray:
    a = np.ascontiguousarray(a) if dtype is None else np.ascontiguousarray(a, dtype=dtype)
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(scale) -> float:
    """The attention scale is an fp32 quantity (the device ABI takes a float): both sides use the same value."""
    return float(np.float32(scale))


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"{what}: oracle rejected the arguments (code {rc})")


def clustered_decode(q, k_full, v, head_to_cluster, rep_heads, T, scale, want_probs=False):
    """q [B,H,d]; k_full, v [B,H,T_cap,d]; maps int32.  Returns out [B,H,d] f64 (and probs [B,k,T])."""
    q, k_full, v = _c(q), _c(k_full), _c(v)
    dt = _dtype_code(q)
    assert _dtype_code(k_full) == dt and _dtype_code(v) == dt
    B, H, d = q.shape
    T_cap = k_full.shape[2]
    assert k_full.shape == (B, H, T_cap, d) and v.shape == (B, H, T_cap, d)
    h2c = _c(head_to_cluster, np.int32)
    rep = _c(rep_heads, np.int32)
    k = rep.shape[1]
    assert h2c.shape == (B, H) and rep.shape == (B, k)
    out = np.empty((B, H, d), np.float64)
    probs = np.empty((B, k, T), np.float64) if want_probs else None
    rc = lib().chai_oracle_clustered_decode(_p(q), _p(k_full), _p(v), _p(h2c), _p(rep), B, H, k, T, T_cap, d, dt,
                                            _f32(scale), _p(out), _p(probs))
    _check(rc, "clustered_decode")
    return (out, probs) if want_probs else out


def shared_v_decode(q, k_full, v, head_to_cluster, rep_heads, T, scale):
    """As clustered_decode, but every head also takes the representative's values.  Returns out [B,H,d] f64."""
    q, k_full, v = _c(q), _c(k_full), _c(v)
    dt = _dtype_code(q)
    assert _dtype_code(k_full) == dt and _dtype_code(v) == dt
    B, H, d = q.shape
    T_cap = k_full.shape[2]
    assert k_full.shape == (B, H, T_cap, d) and v.shape == (B, H, T_cap, d)
    h2c = _c(head_to_cluster, np.int32)
    rep = _c(rep_heads, np.int32)
    k = rep.shape[1]
    assert h2c.shape == (B, H) and rep.shape == (B, k)
    out = np.empty((B, H, d), np.float64)
    rc = lib().chai_oracle_shared_v_decode(_p(q), _p(k_full), _p(v), _p(h2c), _p(rep), B, H, k, T, T_cap, d, dt,
                                           _f32(scale), _p(out))
    _check(rc, "shared_v_decode")
    return out


def clustered_prefill(q, k_full, v, head_to_cluster, rep_heads, q_start, scale):
    """q [B,H,Tq,d] (rows at positions q_start..q_start+Tq-1); k_full, v [B,H,T_cap,d].  out [B,H,Tq,d] f64."""
    q, k_full, v = _c(q), _c(k_full), _c(v)
    dt = _dtype_code(q)
    assert _dtype_code(k_full) == dt and _dtype_code(v) == dt
    B, H, Tq, d = q.shape
    T_cap = k_full.shape[2]
    h2c = _c(head_to_cluster, np.int32)
    rep = _c(rep_heads, np.int32)
    k = rep.shape[1]
    out = np.empty((B, H, Tq, d), np.float64)
    rc = lib().chai_oracle_clustered_prefill(_p(q), _p(k_full), _p(v), _p(h2c), _p(rep), B, H, k, Tq, int(q_start),
                                             T_cap, d, dt, _f32(scale), _p(out))
    _check(rc, "clustered_prefill")
    return out


def dense_decode(q, k_cache, v, T, scale, want_probs=False):
    q, k_cache, v = _c(q), _c(k_cache), _c(v)
    dt = _dtype_code(q)
    assert _dtype_code(k_cache) == dt and _dtype_code(v) == dt
    B, H, d = q.shape
    T_cap = k_cache.shape[2]
    assert k_cache.shape == (B, H, T_cap, d) and v.shape == (B, H, T_cap, d)
    out = np.empty((B, H, d), np.float64)
    probs = np.empty((B, H, T), np.float64) if want_probs else None
    rc = lib().chai_oracle_dense_decode(_p(q), _p(k_cache), _p(v), B, H, T, T_cap, d, dt, _f32(scale), _p(out),
                                        _p(probs))
    _check(rc, "dense_decode")
    return (out, probs) if want_probs else out


def score_features(q5, k5, scale, n_tok=None):
    """q5 [B,H,n_tok,d]; k5 [B,H,Tk,d] with Tk >= n_tok (first n_tok rows are used).  feat [B,H,n_tok^2] f32."""
    q5, k5 = _c(q5), _c(k5)
    dt = _dtype_code(q5)
    assert _dtype_code(k5) == dt
    B, H, nq, d = q5.shape
    n_tok = nq if n_tok is None else n_tok
    assert k5.shape[:2] == (B, H) and k5.shape[3] == d and k5.shape[2] >= n_tok and nq >= n_tok
    feat = np.empty((B, H, n_tok * n_tok), np.float32)
    rc = lib().chai_oracle_score_features(_p(q5), _p(k5), B, H, n_tok, d, dt, nq * d, k5.shape[2] * d,
                                          _f32(scale), _p(feat))
    _check(rc, "score_features")
    return feat


def kmeans(feat, init_heads, max_iter=50, want_sse=False):
    """feat [B,H,F] f32; init_heads [B,k].  Returns head_to_cluster, rep_heads, n_clusters, iters (, sse)."""
    feat = _c(feat, np.float32)
    init = _c(init_heads, np.int32)
    B, H, F = feat.shape
    k = init.shape[1]
    assert init.shape == (B, k)
    h2c = np.empty((B, H), np.int32)
    rep = np.empty((B, k), np.int32)
    ncl = np.empty((B,), np.int32)
    its = np.empty((B,), np.int32)
    sse = np.empty((B,), np.float64) if want_sse else None
    rc = lib().chai_oracle_kmeans(_p(feat), B, H, F, k, _p(init), int(max_iter), _p(h2c), _p(rep), _p(ncl), _p(its),
                                  _p(sse))
    _check(rc, "kmeans")
    return (h2c, rep, ncl, its, sse) if want_sse else (h2c, rep, ncl, its)


def cluster_error(feat, head_to_cluster, k):
    """Sum of squared distances of every head's features to the mean of its cluster; [B] f64."""
    feat = _c(feat, np.float32)
    h2c = _c(head_to_cluster, np.int32)
    B, H, F = feat.shape
    sse = np.empty((B,), np.float64)
    _check(lib().chai_oracle_cluster_error(_p(feat), _p(h2c), B, H, F, int(k), _p(sse)), "cluster_error")
    return sse


def closest_representatives(feat, head_to_cluster, k):
    """Per cluster the member closest to the mean of the members (ties -> lowest head), -1 for empty slots; [B,k]."""
    feat = _c(feat, np.float32)
    h2c = _c(head_to_cluster, np.int32)
    B, H, F = feat.shape
    rep = np.empty((B, int(k)), np.int32)
    _check(lib().chai_oracle_closest_representatives(_p(feat), _p(h2c), B, H, F, int(k), _p(rep)),
           "closest_representatives")
    return rep


def pick_cluster_count(err, ks, tol):
    err = _c(err, np.float64)
    ks = _c(ks, np.int32)
    out = np.zeros((1,), np.int32)
    _check(lib().chai_oracle_pick_cluster_count(_p(err), _p(ks), len(ks), float(tol), _p(out)), "pick_cluster_count")
    return int(out[0])


def project_qk(x, w_q, w_k, rep_heads, d):
    """x [B,Tn,D]; w_q, w_k [H*d, D]; rep_heads [B,k].  Returns (q_rep, k_rep), each [B,k,Tn,d] f64, unrounded."""
    x, w_q, w_k = _c(x), _c(w_q), _c(w_k)
    dt = _dtype_code(x)
    assert _dtype_code(w_q) == dt and _dtype_code(w_k) == dt
    B, Tn, D = x.shape
    H = w_q.shape[0] // d
    assert w_q.shape == (H * d, D) and w_k.shape == (H * d, D)
    rep = _c(rep_heads, np.int32)
    k = rep.shape[1]
    assert rep.shape == (B, k)
    q_rep = np.empty((B, k, Tn, d), np.float64)
    k_rep = np.empty((B, k, Tn, d), np.float64)
    _check(lib().chai_oracle_project_qk(_p(x), _p(w_q), _p(w_k), _p(rep), B, H, k, Tn, D, d, dt, _p(q_rep), _p(k_rep)),
           "project_qk")
    return q_rep, k_rep


def compact_kcache(k_full, rep_heads, T, Tc_cap=None, k_compact=None, want_src_rows=False):
    k_full = _c(k_full)
    dt = _dtype_code(k_full)
    rep = _c(rep_heads, np.int32)
    B, H, T_cap, d = k_full.shape
    k = rep.shape[1]
    if k_compact is None:
        Tc_cap = T_cap if Tc_cap is None else Tc_cap
        k_compact = np.zeros((B, k, Tc_cap, d), k_full.dtype)
    Tc_cap = k_compact.shape[2]
    assert k_compact.flags.c_contiguous and k_compact.dtype == k_full.dtype
    src = np.empty((B, k, T), np.int64) if want_src_rows else None
    rc = lib().chai_oracle_compact_kcache(_p(k_full), _p(rep), _p(k_compact), B, H, k, T, T_cap, Tc_cap, d, dt,
                                          _p(src))
    _check(rc, "compact_kcache")
    return (k_compact, src) if want_src_rows else k_compact


def append_kv(k_new, v_new, rep_heads, k_compact, v_cache, pos):
    """In-place append into k_compact [B,k,Tc_cap,d] and v_cache [B,H,T_cap,d] at row `pos`."""
    k_new, v_new = _c(k_new), _c(v_new)
    dt = _dtype_code(k_new)
    rep = _c(rep_heads, np.int32)
    B, H, d = k_new.shape
    k = rep.shape[1]
    assert k_compact.flags.c_contiguous and v_cache.flags.c_contiguous
    assert k_compact.shape[:2] == (B, k) and v_cache.shape[:2] == (B, H)
    rc = lib().chai_oracle_append_kv(_p(k_new), _p(v_new), _p(rep), _p(k_compact), _p(v_cache), B, H, k, int(pos),
                                     k_compact.shape[2], v_cache.shape[2], d, dt)
    _check(rc, "append_kv")


def e4m3_decode(code: int) -> float:
    """Value of one 8-bit E4M3 code (NaN for 0x7f / 0xff)."""
    return float(lib().chai_oracle_e4m3_decode(int(code)))


def e4m3_encode(y: float) -> int:
    """Nearest E4M3 code of the fp32 value y (ties to even, saturating at 448)."""
    return int(lib().chai_oracle_e4m3_encode(float(np.float32(y))))


def quantize_rows(x):
    """x [..., d] fp32 or bf16 bits -> (codes uint8 [..., d], scales fp32 [...]): one scale per row."""
    x = _c(x)
    d = x.shape[-1]
    n = int(np.prod(x.shape[:-1]))
    codes = np.empty(x.shape, np.uint8)
    scales = np.empty(x.shape[:-1], np.float32)
    _check(lib().chai_oracle_quantize_rows(_p(x), n, d, _dtype_code(x), _p(codes), _p(scales)), "quantize_rows")
    return codes, scales


def dequantize_rows(codes, scales):
    """codes uint8 [..., d], scales fp32 [...] -> f64 [..., d]."""
    codes, scales = _c(codes, np.uint8), _c(scales, np.float32)
    d = codes.shape[-1]
    n = int(np.prod(codes.shape[:-1]))
    assert scales.shape == codes.shape[:-1]
    out = np.empty(codes.shape, np.float64)
    _check(lib().chai_oracle_dequantize_rows(_p(codes), _p(scales), n, d, _p(out)), "dequantize_rows")
    return out


def clustered_decode_q8(q, k8, kscale, v8, vscale, head_to_cluster, rep_heads, T, scale, want_probs=False):
    """Clustered decode over quantised FULL caches: q [B,H,d] (fp32 / bf16 bits); k8, v8 uint8 [B,H,T_cap,d];
    kscale, vscale fp32 [B,H,T_cap].  Returns out [B,H,d] f64 (and probs [B,k,T])."""
    q, k8, v8 = _c(q), _c(k8, np.uint8), _c(v8, np.uint8)
    kscale, vscale = _c(kscale, np.float32), _c(vscale, np.float32)
    B, H, d = q.shape
    T_cap = k8.shape[2]
    assert k8.shape == (B, H, T_cap, d) and v8.shape == (B, H, T_cap, d)
    assert kscale.shape == (B, H, T_cap) and vscale.shape == (B, H, T_cap)
    h2c = _c(head_to_cluster, np.int32)
    rep = _c(rep_heads, np.int32)
    k = rep.shape[1]
    out = np.empty((B, H, d), np.float64)
    probs = np.empty((B, k, T), np.float64) if want_probs else None
    rc = lib().chai_oracle_clustered_decode_q8(_p(q), _p(k8), _p(kscale), _p(v8), _p(vscale), _p(h2c), _p(rep), B, H, k,
                                               T, T_cap, d, _dtype_code(q), _f32(scale), _p(out), _p(probs))
    _check(rc, "clustered_decode_q8")
    return (out, probs) if want_probs else out
