"""Helpers of the GPU parity tests: run one layer through libchai (via the Python binding, i.e. the C ABI) and
through the CPU oracle on the same bytes, and compare."""
from __future__ import annotations

import numpy as np
import torch

import paper_2403_08058_amd as C
import workloads as W
from oracle import chai_oracle as O

# Tolerances (normwise per output row: max_i |gpu_i - oracle_i| <= rtol * max_i |oracle_i|).
# The contract is 1e-5 for fp32 inputs and 2e-3 for bf16 inputs with fp32 accumulation.  bf16 products are exact
# in fp32 and both paths see the same bits, so the bf16 path is held to a bar far tighter than 2e-3: a single
# dropped token at T = 2048 already moves an output by ~5e-4, which the looser bar would hide.
RTOL = {W.F32: 1e-5, W.BF16: 2e-5}
RTOL_CONTRACT = {W.F32: 1e-5, W.BF16: 2e-3}
PROB_ATOL = 2e-6        # probabilities are <= 1; fp32 softmax of fp32 scores


def dev(a: np.ndarray) -> torch.Tensor:
    return W.host_to_torch(a, "cuda")


ELEMENT_FLOOR = 0.25    # share of a row's largest magnitude that every element's own bar is raised by


def rows_close(gpu: np.ndarray, ref: np.ndarray, rtol: float):
    """Normwise comparison per output row; returns (ok, worst ratio err/allowed).  At the tight bars of the decode
    path (rtol <= 2e-5) every element is also held to rtol * (|its own value| + ELEMENT_FLOOR * the row's largest
    magnitude): the small elements of a row may not hide behind its largest one."""
    gpu = np.asarray(gpu, np.float64).reshape(-1, ref.shape[-1])
    ref = np.asarray(ref, np.float64).reshape(-1, ref.shape[-1])
    diff = np.abs(gpu - ref)
    err = diff.max(axis=1)
    rowmax = np.abs(ref).max(axis=1)
    allowed = rtol * rowmax
    worst = float((err / np.maximum(allowed, 1e-300)).max()) if len(err) else 0.0
    ok = bool(np.all(err <= allowed)) and bool(np.all(np.isfinite(gpu)))
    if rtol <= 2e-5:
        ok = ok and bool(np.all(diff <= rtol * (np.abs(ref) + ELEMENT_FLOOR * rowmax[:, None])))
    return ok, worst


def guarded(shape, dtype, fill):
    """Tensor with guard rows before and after, to catch out-of-bounds writes.  Returns (whole, view)."""
    n = int(np.prod(shape))
    pad = 1024
    whole = torch.full((n + 2 * pad,), fill, dtype=dtype, device="cuda")
    return whole, whole[pad:pad + n].view(*shape)


def guards_intact(whole, shape, fill) -> bool:
    n = int(np.prod(shape))
    pad = 1024
    lo, hi = whole[:pad], whole[pad + n:]
    if isinstance(fill, float) and np.isnan(fill):
        return bool(torch.isnan(lo).all() and torch.isnan(hi).all())
    return bool((lo == fill).all() and (hi == fill).all())


def poisoned_workspace(B, H, k, T, d, dtype):
    ws = C.alloc_workspace(B, H, k, T, d, dtype)
    ws.fill_(0xFF)          # NaN patterns as floats, huge values as counters: nothing may rely on old contents
    return ws


def gpu_membership(x: W.LayerInputs, cfg: W.Config, k_dev: torch.Tensor):
    """Feature + k-means kernels on the device; returns device maps and the host copies."""
    q5 = dev(x.q5)
    feat = C.chai_score_features(q5, k_dev, W.N_TOK, cfg.scale)
    h2c, rep, ncl, iters = C.chai_assign_clusters(feat, dev(x.init_heads))
    return feat, h2c, rep, ncl, iters


def run_clustered_layer(cfg: W.Config, x: W.LayerInputs, check_probs=True):
    """Membership (as the config prescribes), compaction and one decode step on the GPU, against the oracle.
    Returns a dict of diagnostics; raises AssertionError on any mismatch."""
    B, H, d, T, T_cap = cfg.B, cfg.H, cfg.d, cfg.T, cfg.T_cap
    k = x.k_layer
    k_dev, v_dev, q_dev = dev(x.k), dev(x.v), dev(x.q)

    if x.init_heads is not None:
        feat, h2c_d, rep_d, ncl_d, it_d = gpu_membership(x, cfg, k_dev)
        torch.cuda.synchronize()
        feat_h = feat.cpu().numpy()
        # the same feature bits through the oracle's k-means: integer outputs must be identical
        h2c_o, rep_o, ncl_o, it_o = O.kmeans(feat_h, x.init_heads)
        assert np.array_equal(h2c_d.cpu().numpy(), h2c_o), "head_to_cluster differs from the oracle"
        assert np.array_equal(rep_d.cpu().numpy(), rep_o), "rep_heads differs from the oracle"
        assert np.array_equal(ncl_d.cpu().numpy(), ncl_o) and np.array_equal(it_d.cpu().numpy(), it_o)
        # features against the oracle's own (fp64 on both sides, rounded once to fp32)
        feat_o = O.score_features(x.q5, x.k, cfg.scale, n_tok=W.N_TOK)
        assert np.abs(feat_h - feat_o).max() <= 1e-6, "features differ from the oracle"
        # end to end (oracle features -> oracle k-means) gives the same membership on these seeded inputs
        h2c_e, rep_e, _, _ = O.kmeans(feat_o, x.init_heads)
        assert np.array_equal(h2c_e, h2c_o) and np.array_equal(rep_e, rep_o), "membership not robust to feature rounding"
        h2c_h, rep_h = h2c_o, rep_o
    else:
        h2c_h, rep_h = x.h2c, x.rep
        h2c_d, rep_d = dev(h2c_h), dev(rep_h)

    # compaction: bytes equal to the index gather
    Tc_cap = T_cap
    kc_whole, kc = guarded((B, k, Tc_cap, d), k_dev.dtype, 0.0)
    kc.fill_(3.0)
    C.chai_compact_kcache(k_dev, rep_d, kc, T)
    torch.cuda.synchronize()
    kc_sent = np.full((B, k, Tc_cap, d), W.store(np.array([3.0]), cfg.dtype)[0], x.k.dtype)
    kc_o = O.compact_kcache(x.k, rep_h, T, k_compact=kc_sent)
    assert np.array_equal(W.torch_to_host_bits(kc), kc_o), "compact K cache differs from the gather"
    assert guards_intact(kc_whole, (B, k, Tc_cap, d), 0.0)

    # one decode step
    out_whole, out = guarded((B, H, d), torch.float32, float("nan"))
    probs = torch.full((B, k, T), float("nan"), dtype=torch.float32, device="cuda")
    ws = poisoned_workspace(B, H, k, T, d, cfg.dtype)
    C.chai_decode_attention(q_dev, kc, v_dev, h2c_d, rep_d, T, cfg.scale, out, ws, probs_out=probs)
    torch.cuda.synchronize()
    out_o, probs_o = O.clustered_decode(x.q, x.k, x.v, h2c_h, rep_h, T, cfg.scale, want_probs=True)
    ok, worst = rows_close(out.cpu().numpy(), out_o, RTOL[cfg.dtype])
    assert ok, f"clustered decode output off: worst err/allowed = {worst:.3g}"
    assert guards_intact(out_whole, (B, H, d), float("nan"))
    if check_probs:
        p = probs.cpu().numpy().astype(np.float64)
        used = rep_h >= 0
        assert np.abs(p[used] - probs_o[used]).max() <= PROB_ATOL
        assert np.abs(p[used].sum(-1) - 1.0).max() <= 1e-5 and np.all(p[used] >= 0)
        assert np.all(np.isnan(p[~used]))
    return {"worst": worst, "h2c": h2c_h, "rep": rep_h, "out": out, "kc": kc, "v": v_dev, "k": k_dev, "q": q_dev}
