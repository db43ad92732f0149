"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element, on seeded inputs
of the five configurations at sizes the oracle finishes in seconds (several chunks plus a ragged tail), and on
the edge cases of the method."""
import dataclasses
import math

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

if not torch.cuda.is_available():       # collected everywhere, run only where a GPU exists
    pytest.skip("needs a GPU", allow_module_level=True)

import paper_2403_08058_amd as C
import workloads as W
from oracle import chai_oracle as O

import gpu_util as G
from gpu_util import dev


# ----------------------------------------------------------------------------------------------
# the five configurations, reduced
# ----------------------------------------------------------------------------------------------
REDUCED = {
    "cfg1": W.CONFIGS["cfg1"],                                              # already small: run in full
    "cfg2": W.CONFIGS["cfg2"].reduced(L=3, B=3, T=1300, T_cap=1333),        # one unclustered layer, two k=8
    "cfg3": W.CONFIGS["cfg3"].reduced(L=4, B=2, T=777, T_cap=800),
    "cfg5": W.CONFIGS["cfg5"].reduced(L=2, B=2, T=4500, T_cap=4608),
}


@pytest.mark.parametrize("name", sorted(REDUCED))
def test_config_layers_match_oracle(name):
    cfg = REDUCED[name]
    for layer in range(cfg.L):
        print(f"[parity] {cfg.name} layer {layer} k={cfg.ks[layer]} B={cfg.B} H={cfg.H} T={cfg.T}", flush=True)
        x = W.layer_inputs(cfg, layer)
        res = G.run_clustered_layer(cfg, x)
        if cfg.membership == "planted":
            # k-means recovers the planted groups (canonical numbering = order of first appearance)
            for b in range(cfg.B):
                seen = {}
                canon = [seen.setdefault(int(a), len(seen)) for a in x.groups[b]]
                assert res["h2c"][b].tolist() == canon


def test_cfg4_end_to_end_reduced():
    """Prompt -> features -> k-means -> compaction -> decode steps with cache growth, against the oracle doing the
    same on the host (OPT-66B head structure, shortened prompt and step count)."""
    cfg = dataclasses.replace(W.CONFIGS["cfg4"], name="cfg4-reduced", L=2, B=2, T=0, T_cap=96, prompt=70,
                              decode_steps=9, ks=(16, 16))
    B, H, d, k = cfg.B, cfg.H, cfg.d, 16
    for layer in range(cfg.L):
        print(f"[parity] {cfg.name} layer {layer}", flush=True)
        x = W.layer_inputs(cfg, layer)
        # cache rows at and beyond the prompt are not part of the prompt: poison them on both sides
        nan_bits = np.uint16(0x7FC0)
        x.k[:, :, cfg.prompt:] = nan_bits
        x.v[:, :, cfg.prompt:] = nan_bits
        k_dev, v_dev = dev(x.k), dev(x.v)
        feat, h2c_d, rep_d, ncl_d, it_d = G.gpu_membership(x, cfg, k_dev)
        h2c_o, rep_o, ncl_o, it_o = O.kmeans(feat.cpu().numpy(), x.init_heads)
        assert np.array_equal(h2c_d.cpu().numpy(), h2c_o) and np.array_equal(rep_d.cpu().numpy(), rep_o)
        Tc_cap = cfg.T_cap - 8                     # the compact cache may have its own capacity
        kc = torch.zeros((B, k, Tc_cap, d), dtype=torch.bfloat16, device="cuda")
        C.chai_compact_kcache(k_dev, rep_d, kc, cfg.prompt)
        kc_o = O.compact_kcache(x.k, rep_o, cfg.prompt, Tc_cap=Tc_cap)
        k_full_o, v_o = x.k.copy(), x.v.copy()      # the oracle keeps the full K cache
        out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
        for step in range(cfg.decode_steps):
            pos = cfg.prompt + step
            T = pos + 1
            q, kn, vn = W.step_inputs(cfg, layer, step)
            C.chai_append_kv(dev(kn), dev(vn), rep_d, kc, v_dev, pos)
            ws = G.poisoned_workspace(B, H, k, T, d, cfg.dtype)
            C.chai_decode_attention(dev(q), kc, v_dev, h2c_d, rep_d, T, cfg.scale, out, ws)
            torch.cuda.synchronize()
            O.append_kv(kn, vn, rep_o, kc_o, v_o, pos)
            k_full_o[:, :, pos] = kn
            ref = O.clustered_decode(q, k_full_o, v_o, h2c_o, rep_o, T, cfg.scale)
            ok, worst = G.rows_close(out.cpu().numpy(), ref, G.RTOL[cfg.dtype])
            assert ok, (layer, step, worst)
        assert np.array_equal(W.torch_to_host_bits(kc)[:, :, :T], kc_o[:, :, :T])
        assert np.array_equal(W.torch_to_host_bits(v_dev)[:, :, :T], v_o[:, :, :T])


# ----------------------------------------------------------------------------------------------
# dense baseline and reductions the paper fixes
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,B,H,T,T_cap", [(W.F32, 2, 5, 300, 320), (W.BF16, 3, 32, 1000, 1024),
                                               (W.BF16, 1, 52, 2049, 2049), (W.F32, 1, 3, 1, 4)])
def test_dense_decode_matches_oracle(dtype, B, H, T, T_cap):
    g = np.random.default_rng(B * 1000 + H)
    q, k, v = W.normal(g, (B, H, 128), dtype), W.normal(g, (B, H, T_cap, 128), dtype), W.normal(g, (B, H, T_cap, 128), dtype)
    scale = float(np.float32(1 / math.sqrt(128)))
    out = torch.empty((B, H, 128), dtype=torch.float32, device="cuda")
    ws = G.poisoned_workspace(B, H, H, T, 128, dtype)
    C.chai_dense_decode_attention(dev(q), dev(k), dev(v), T, scale, out, ws)
    torch.cuda.synchronize()
    ok, worst = G.rows_close(out.cpu().numpy(), O.dense_decode(q, k, v, T, scale), G.RTOL[dtype])
    assert ok, worst


def test_one_head_per_cluster_equals_dense_kernel():
    """k = H with identity maps through the clustered entry point gives the dense entry point's result bit for
    bit (same kernels, same order), and both match the oracle's dense attention."""
    B, H, T, dtype = 2, 32, 600, W.BF16
    g = np.random.default_rng(5)
    q, k, v = W.normal(g, (B, H, 128), dtype), W.normal(g, (B, H, T, 128), dtype), W.normal(g, (B, H, T, 128), dtype)
    ident = torch.arange(H, dtype=torch.int32, device="cuda").repeat(B, 1).contiguous()
    o1 = torch.empty((B, H, 128), dtype=torch.float32, device="cuda")
    o2 = torch.empty_like(o1)
    qd, kd, vd = dev(q), dev(k), dev(v)
    C.chai_decode_attention(qd, kd, vd, ident, ident, T, 0.088, o1, G.poisoned_workspace(B, H, H, T, 128, dtype))
    C.chai_dense_decode_attention(qd, kd, vd, T, 0.088, o2, G.poisoned_workspace(B, H, H, T, 128, dtype))
    torch.cuda.synchronize()
    assert torch.equal(o1, o2)
    ok, worst = G.rows_close(o1.cpu().numpy(), O.dense_decode(q, k, v, T, 0.088), G.RTOL[dtype])
    assert ok, worst


def test_members_with_identical_qk_equal_dense():
    """Heads of a cluster share Q and K exactly: clustered attention equals dense attention for every head."""
    B, H, T, kk, dtype = 2, 32, 900, 6, W.BF16
    g = np.random.default_rng(6)
    h2c, rep = W.random_membership(g, B, H, kk)
    qc, kc_ = W.normal(g, (B, kk, 128), dtype), W.normal(g, (B, kk, T, 128), dtype)
    q = np.stack([qc[b, h2c[b]] for b in range(B)])
    k = np.stack([kc_[b, h2c[b]] for b in range(B)])
    v = W.normal(g, (B, H, T, 128), dtype)
    kd = dev(k)
    kcomp = torch.empty((B, kk, T, 128), dtype=torch.bfloat16, device="cuda")
    C.chai_compact_kcache(kd, dev(rep), kcomp, T)
    out = torch.empty((B, H, 128), dtype=torch.float32, device="cuda")
    C.chai_decode_attention(dev(q), kcomp, dev(v), dev(h2c), dev(rep), T, 0.088, out,
                            G.poisoned_workspace(B, H, kk, T, 128, dtype))
    dense = torch.empty_like(out)
    C.chai_dense_decode_attention(dev(q), kd, dev(v), T, 0.088, dense, G.poisoned_workspace(B, H, H, T, 128, dtype))
    torch.cuda.synchronize()
    # the two calls cut the token axis differently, so they agree to rounding, not bit for bit
    ok, worst = G.rows_close(out.cpu().numpy(), dense.cpu().numpy().astype(np.float64), 1e-5)
    assert ok, worst
    ok, worst = G.rows_close(out.cpu().numpy(), O.dense_decode(q, k, v, T, 0.088), G.RTOL[dtype])
    assert ok, worst


# ----------------------------------------------------------------------------------------------
# edge cases of the decode path
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
@pytest.mark.parametrize("B,H,kk,T,T_cap", [
    (1, 32, 8, 1, 16),          # a single cached token
    (1, 32, 1, 257, 300),       # one cluster for all heads, one token past a chunk
    (2, 72, 16, 127, 127),      # cache exactly full, odd length
    (1, 52, 52, 64, 64),        # every head alone
    (5, 32, 4, 1025, 1100),     # chunk boundary + 1
    (1, 1, 1, 33, 40),          # one head
    (2, 32, 8, 16, 16),         # exactly one load group (bf16) / two (fp32)
    (4, 72, 16, 1300, 1333),    # 288 heads: two workgroups per head, half of the columns each
    (6, 32, 8, 77, 80),         # 192 heads, short context
])
def test_decode_edge_shapes(dtype, B, H, kk, T, T_cap):
    cfg = W.Config("edge", L=1, H=H, d=128, B=B, T=T, T_cap=T_cap, dtype=dtype, ks=(kk,), membership="random",
                   seed=B * 7 + H * 13 + kk * 17 + T)
    G.run_clustered_layer(cfg, W.layer_inputs(cfg, 0))


def test_unused_cluster_slots_and_arbitrary_labels():
    """Slots with rep = -1 are skipped (their probs_out rows stay untouched); cluster ids need not be canonical."""
    B, H, kk, T, dtype = 2, 32, 8, 300, W.BF16
    cfg = W.Config("slots", L=1, H=H, d=128, B=B, T=T, T_cap=T, dtype=dtype, ks=(kk,), membership="random", seed=77)
    x = W.layer_inputs(cfg, 0)
    # move every head of slots 2 and 5 into slot 0 and mark them unused
    for b in range(B):
        x.h2c[b][(x.h2c[b] == 2) | (x.h2c[b] == 5)] = 0
    x.rep = W.representatives(x.h2c, kk)
    assert np.all(x.rep[:, [2, 5]] == -1)
    G.run_clustered_layer(cfg, x)


@pytest.mark.parametrize("scale", [80.0, -80.0, 0.0])
def test_softmax_stable_for_extreme_scores(scale):
    B, H, kk, T, dtype = 1, 32, 8, 700, W.F32
    cfg = W.Config("extreme", L=1, H=H, d=128, B=B, T=T, T_cap=T, dtype=dtype, ks=(kk,), membership="random", seed=88)
    x = W.layer_inputs(cfg, 0)
    kd, vd, qd = dev(x.k), dev(x.v), dev(x.q)
    kc = torch.empty((B, kk, T, 128), dtype=torch.float32, device="cuda")
    C.chai_compact_kcache(kd, dev(x.rep), kc, T)
    out = torch.empty((B, H, 128), dtype=torch.float32, device="cuda")
    probs = torch.empty((B, kk, T), dtype=torch.float32, device="cuda")
    C.chai_decode_attention(qd, kc, vd, dev(x.h2c), dev(x.rep), T, scale, out, G.poisoned_workspace(B, H, kk, T, 128, dtype),
                            probs_out=probs)
    torch.cuda.synchronize()
    ref, pref = O.clustered_decode(x.q, x.k, x.v, x.h2c, x.rep, T, scale, want_probs=True)
    p = probs.cpu().numpy()
    assert np.all(np.isfinite(p)) and np.abs(p.sum(-1) - 1).max() < 1e-5
    # scores of magnitude ~1000 carry fp32 rounding of ~1e-4 absolute, which the softmax turns into relative
    # error of the same size: compare the winners and the outputs at a bar that reflects it
    assert np.array_equal(p.argmax(-1), pref.argmax(-1))
    ok, worst = G.rows_close(out.cpu().numpy(), ref, 2e-3 if scale != 0.0 else 1e-5)
    assert ok, worst


def test_workspace_reuse_across_calls_and_shapes():
    """One workspace serves consecutive calls of different sizes (stale contents of the previous call)."""
    dtype = W.BF16
    ws = C.alloc_workspace(4, 32, 8, 3000, 128, dtype)
    ws.fill_(0xFF)
    for seed, (B, T) in enumerate([(4, 3000), (2, 700), (4, 2999), (1, 5)]):
        cfg = W.Config("reuse", L=1, H=32, d=128, B=B, T=T, T_cap=T, dtype=dtype, ks=(8,), membership="random", seed=seed)
        x = W.layer_inputs(cfg, 0)
        kc = torch.empty((B, 8, T, 128), dtype=torch.bfloat16, device="cuda")
        C.chai_compact_kcache(dev(x.k), dev(x.rep), kc, T)
        out = torch.empty((B, 32, 128), dtype=torch.float32, device="cuda")
        C.chai_decode_attention(dev(x.q), kc, dev(x.v), dev(x.h2c), dev(x.rep), T, cfg.scale, out, ws)
        torch.cuda.synchronize()
        ok, worst = G.rows_close(out.cpu().numpy(), O.clustered_decode(x.q, x.k, x.v, x.h2c, x.rep, T, cfg.scale),
                                 G.RTOL[dtype])
        assert ok, (B, T, worst)


def test_runs_on_a_side_stream():
    B, H, kk, T, dtype = 2, 32, 8, 1500, W.BF16
    cfg = W.Config("stream", L=1, H=H, d=128, B=B, T=T, T_cap=T, dtype=dtype, ks=(kk,), membership="random", seed=99)
    x = W.layer_inputs(cfg, 0)
    s = torch.cuda.Stream()
    qd, kd, vd, hd, rd = dev(x.q), dev(x.k), dev(x.v), dev(x.h2c), dev(x.rep)
    kc = torch.empty((B, kk, T, 128), dtype=torch.bfloat16, device="cuda")
    out = torch.empty((B, H, 128), dtype=torch.float32, device="cuda")
    ws = G.poisoned_workspace(B, H, kk, T, 128, dtype)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        C.chai_compact_kcache(kd, rd, kc, T)
        C.chai_decode_attention(qd, kc, vd, hd, rd, T, cfg.scale, out, ws)
    s.synchronize()
    ok, worst = G.rows_close(out.cpu().numpy(), O.clustered_decode(x.q, x.k, x.v, x.h2c, x.rep, T, cfg.scale), G.RTOL[dtype])
    assert ok, worst


# ----------------------------------------------------------------------------------------------
# membership kernels
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
@pytest.mark.parametrize("n_tok", [1, 5, 8])
def test_score_features_match_oracle(dtype, n_tok):
    B, H = 3, 52
    g = np.random.default_rng(n_tok + 10 * dtype)
    q5 = W.normal(g, (B, H, n_tok + 2, 128), dtype)       # more query rows than used: stride > n_tok*d
    kc = W.normal(g, (B, H, 40, 128), dtype)              # keys read in place from a cache
    feat = C.chai_score_features(dev(q5), dev(kc), n_tok, 0.0884)
    torch.cuda.synchronize()
    ref = O.score_features(q5, kc, 0.0884, n_tok=n_tok)
    f = feat.cpu().numpy()
    assert np.abs(f - ref).max() <= 1e-6
    # structure that must hold exactly: causal zeros, first row (1, 0, ...)
    fm = f.reshape(B, H, n_tok, n_tok)
    assert np.all(fm[..., 0, 0] == 1.0)
    assert np.all(fm[np.broadcast_to(np.triu(np.ones((n_tok, n_tok), bool), 1), fm.shape)] == 0.0)
    # almost every value is the same fp32 number (fp64 on both sides, one rounding)
    assert np.mean(f == ref) > 0.999


@pytest.mark.parametrize("H,F,k", [(32, 25, 8), (32, 25, 32), (52, 25, 4), (52, 25, 16), (72, 25, 16), (72, 25, 1),
                                   (32, 5, 8), (256, 25, 64), (7, 64, 3), (1, 1, 1)])
def test_assign_clusters_bit_exact(H, F, k):
    g = np.random.default_rng(H * 100 + F * 10 + k)
    B = 6
    feat = g.random((B, H, F)).astype(np.float32)
    feat[1] = np.round(feat[1] * 4) / 4                    # many exact ties
    if H > 3:
        feat[2, 1] = feat[2, 0]                            # duplicate points
        feat[2, H - 1] = feat[2, 0]
    feat[3] = feat[3, 0]                                   # all points equal
    init = W.distinct_heads(g, B, H, k)
    if k >= 2:
        init[2, 0], init[2, 1] = 0, 1 if H > 3 else init[2, 1]    # two starting centres on duplicate points
    for max_iter in (50, 1, 2):
        h2c, rep, ncl, it = C.chai_assign_clusters(dev(feat), dev(init), max_iter=max_iter)
        torch.cuda.synchronize()
        h2c_o, rep_o, ncl_o, it_o = O.kmeans(feat, init, max_iter=max_iter)
        assert np.array_equal(h2c.cpu().numpy(), h2c_o), max_iter
        assert np.array_equal(rep.cpu().numpy(), rep_o), max_iter
        assert np.array_equal(ncl.cpu().numpy(), ncl_o) and np.array_equal(it.cpu().numpy(), it_o), max_iter


def test_assign_clusters_on_feature_like_data():
    """k-means on real feature vectors (5x5 causal softmax blocks) of many random heads: bit-exact, 200 problems."""
    g = np.random.default_rng(2024)
    for H, k in [(32, 8), (52, 16), (72, 16)]:
        B = 70
        q5, k5 = W.normal(g, (B, H, 5, 128), W.BF16), W.normal(g, (B, H, 5, 128), W.BF16)
        feat = C.chai_score_features(dev(q5), dev(k5), 5, 0.0884)
        init = W.distinct_heads(g, B, H, k)
        h2c, rep, ncl, it = C.chai_assign_clusters(feat, dev(init))
        torch.cuda.synchronize()
        h2c_o, rep_o, ncl_o, it_o = O.kmeans(feat.cpu().numpy(), init)
        assert np.array_equal(h2c.cpu().numpy(), h2c_o) and np.array_equal(rep.cpu().numpy(), rep_o)
        assert np.array_equal(ncl.cpu().numpy(), ncl_o) and np.array_equal(it.cpu().numpy(), it_o)


def test_cluster_error_bit_exact_and_sweep():
    """Clustering error of a partition: same fp64 bits as the oracle; and the offline sweep over candidate
    cluster counts (k-means + error per sample, plateau rule on the mean curve) finds the planted count."""
    g = np.random.default_rng(4242)
    for H, F, k in [(32, 25, 8), (72, 25, 16), (52, 5, 52), (256, 25, 3), (1, 1, 1)]:
        B = 9
        feat = g.random((B, H, F)).astype(np.float32)
        lab = g.integers(0, k, size=(B, H)).astype(np.int32)       # arbitrary labels, some may be unused
        sse = C.chai_cluster_error(dev(feat), dev(lab), k)
        torch.cuda.synchronize()
        assert np.array_equal(sse.cpu().numpy(), O.cluster_error(feat, lab, k)), (H, F, k)
    # sweep on features of planted heads (cfg3 recipe): N samples = batch rows
    cfg = W.CONFIGS["cfg3"].reduced(L=1, B=12, T=8)
    planted = cfg.ks[0]
    x = W.layer_inputs(cfg, 0)
    feat = C.chai_score_features(dev(x.q5), dev(x.k), W.N_TOK, cfg.scale)
    ks = [1, 2, 4, 8, 16, 32, 52]
    curve, curve_o = [], []
    feat_h = feat.cpu().numpy()
    for k in ks:
        init = W.distinct_heads(np.random.default_rng(k), cfg.B, cfg.H, k)
        h2c, _, _, _ = C.chai_assign_clusters(feat, dev(init))
        sse = C.chai_cluster_error(feat, h2c, k)
        torch.cuda.synchronize()
        h2c_o, _, _, _ = O.kmeans(feat_h, init)
        assert np.array_equal(h2c.cpu().numpy(), h2c_o)
        assert np.array_equal(sse.cpu().numpy(), O.cluster_error(feat_h, h2c_o, k))
        curve.append(float(sse.mean()))
        curve_o.append(float(O.cluster_error(feat_h, h2c_o, k).mean()))
    picked = C.chai_pick_cluster_count(curve, ks, 0.05)
    assert picked == O.pick_cluster_count(curve_o, ks, 0.05)
    assert picked in (planted, 2 * planted) or picked == min(kk for kk in ks if kk >= planted)


# ----------------------------------------------------------------------------------------------
# cache kernels
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
@pytest.mark.parametrize("B,H,kk,T,T_cap,Tc_cap", [(2, 32, 8, 1000, 1024, 1001), (1, 72, 16, 1, 8, 8),
                                                   (3, 52, 52, 129, 129, 200), (1, 32, 4, 0, 16, 16)])
def test_compact_kcache_bit_exact(dtype, B, H, kk, T, T_cap, Tc_cap):
    g = np.random.default_rng(T + kk)
    kf = W.normal(g, (B, H, T_cap, 128), dtype)
    _, rep = W.random_membership(g, B, H, kk)
    if kk > 2:
        rep[0, 1] = -1
    tdt = torch.float32 if dtype == W.F32 else torch.bfloat16
    whole, kc = G.guarded((B, kk, Tc_cap, 128), tdt, 0.0)
    kc.fill_(3.0)
    C.chai_compact_kcache(dev(kf), dev(rep), kc, T)
    torch.cuda.synchronize()
    sent = np.full((B, kk, Tc_cap, 128), W.store(np.array([3.0]), dtype)[0], kf.dtype)
    ref, src = O.compact_kcache(kf, rep, T, k_compact=sent, want_src_rows=True)
    assert np.array_equal(W.torch_to_host_bits(kc), ref)
    assert G.guards_intact(whole, (B, kk, Tc_cap, 128), 0.0)
    # the compaction indices: every copied row comes from the representative's row of the same token
    flat = kf.reshape(B * H * T_cap, 128)
    got = W.torch_to_host_bits(kc)
    for b in range(B):
        for j in range(kk):
            if rep[b, j] >= 0 and T > 0:
                assert np.array_equal(got[b, j, :T], flat[src[b, j]])


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_append_kv_bit_exact(dtype):
    B, H, kk, T_cap, Tc_cap = 3, 52, 8, 40, 33
    g = np.random.default_rng(31 + dtype)
    _, rep = W.random_membership(g, B, H, kk)
    rep[1, 3] = -1
    kc0, v0 = W.normal(g, (B, kk, Tc_cap, 128), dtype), W.normal(g, (B, H, T_cap, 128), dtype)
    kcd, vd = dev(kc0), dev(v0)
    kc_o, v_o = kc0.copy(), v0.copy()
    for pos in (0, 17, 32):
        kn, vn = W.normal(g, (B, H, 128), dtype), W.normal(g, (B, H, 128), dtype)
        C.chai_append_kv(dev(kn), dev(vn), dev(rep), kcd, vd, pos)
        O.append_kv(kn, vn, rep, kc_o, v_o, pos)
    torch.cuda.synchronize()
    assert np.array_equal(W.torch_to_host_bits(kcd), kc_o)
    assert np.array_equal(W.torch_to_host_bits(vd), v_o)


# ----------------------------------------------------------------------------------------------
# argument errors are caught on the host, nothing is launched, outputs stay untouched
# ----------------------------------------------------------------------------------------------
def test_argument_errors():
    B, H, kk, T = 1, 32, 8, 64
    q = torch.zeros((B, H, 128), dtype=torch.bfloat16, device="cuda")
    kc = torch.zeros((B, kk, T, 128), dtype=torch.bfloat16, device="cuda")
    v = torch.zeros((B, H, T, 128), dtype=torch.bfloat16, device="cuda")
    h2c = torch.zeros((B, H), dtype=torch.int32, device="cuda")
    rep = torch.zeros((B, kk), dtype=torch.int32, device="cuda")
    out = torch.full((B, H, 128), 7.0, dtype=torch.float32, device="cuda")
    ws = C.alloc_workspace(B, H, kk, T, 128, C.CHAI_BF16)

    def status(fn, *a, **kw):
        with pytest.raises(C.ChaiError) as e:
            fn(*a, **kw)
        return e.value.status

    assert status(C.chai_decode_attention, q, kc, v, h2c, rep, T + 1, 0.1, out, ws) == 2          # T > capacity
    assert status(C.chai_decode_attention, q, kc, v, h2c, rep, 0, 0.1, out, ws) == 2              # T = 0
    assert status(C.chai_decode_attention, q, kc, v, h2c, rep, T, 0.1, out, ws[:128]) == 4        # workspace too small
    assert status(C.chai_decode_attention, q, kc, v, h2c, rep, T, 0.1, out, ws[8:]) == 4          # workspace misaligned
    q64 = torch.zeros((B, H, 64), dtype=torch.bfloat16, device="cuda")
    assert status(C.chai_decode_attention, q64, kc, v, h2c, rep, T, 0.1, out, ws) == 5            # d != 128
    qoff = torch.zeros((B * H * 128 + 8,), dtype=torch.bfloat16, device="cuda")[1:1 + B * H * 128].view(B, H, 128)
    assert status(C.chai_decode_attention, qoff, kc, v, h2c, rep, T, 0.1, out, ws) == 7           # misaligned q
    L = C.lib()
    assert L.chai_decode_attention(None, kc.data_ptr(), v.data_ptr(), h2c.data_ptr(), rep.data_ptr(), B, H, kk, T, T, T,
                                   128, 1, 0.1, out.data_ptr(), None, ws.data_ptr(), ws.numel(), None) == 1
    assert L.chai_decode_attention(q.data_ptr(), kc.data_ptr(), v.data_ptr(), h2c.data_ptr(), rep.data_ptr(), B, H, kk,
                                   T, T, T, 128, 9, 0.1, out.data_ptr(), None, ws.data_ptr(), ws.numel(), None) == 3
    assert L.chai_decode_attention(q.data_ptr(), kc.data_ptr(), v.data_ptr(), h2c.data_ptr(), rep.data_ptr(), B, H,
                                   H + 1, T, T, T, 128, 1, 0.1, out.data_ptr(), None, ws.data_ptr(), ws.numel(), None) == 2
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
    # B = 0 is a no-op that succeeds
    assert L.chai_decode_attention(q.data_ptr(), kc.data_ptr(), v.data_ptr(), h2c.data_ptr(), rep.data_ptr(), 0, H, kk,
                                   T, T, T, 128, 1, 0.1, out.data_ptr(), None, None, 0, None) == 0
    feat = torch.zeros((1, 300, 4), dtype=torch.float32, device="cuda")
    init = torch.zeros((1, 2), dtype=torch.int32, device="cuda")
    assert status(C.chai_assign_clusters, feat, init) == 5                                        # H > 256


def _random_shapes(n, seed):
    """Seeded draw of decode shapes around the planner's thresholds (192 / 384 heads, 1536 tokens, chunk edges)."""
    g = np.random.default_rng(seed)
    out = []
    for i in range(n):
        H = int(g.choice([1, 3, 8, 32, 40, 52, 72]))
        B = int(g.choice([1, 2, 3, 5, 6, 8, 12]))
        kk = int(g.integers(1, H + 1)) if H < 8 else int(g.choice([1, 2, 4, 8]))
        T = int(g.choice([1, 2, 31, 33, 64, 127, 129, 255, 257, 640, 1000, 1535, 1537, 2049]))
        out.append((W.F32 if i % 3 == 0 else W.BF16, B, H, min(kk, H), T, T + int(g.integers(0, 9))))
    return out


@pytest.mark.parametrize("dtype,B,H,kk,T,T_cap", _random_shapes(24, 20240527))
def test_decode_random_shapes(dtype, B, H, kk, T, T_cap):
    cfg = W.Config("rand", L=1, H=H, d=128, B=B, T=T, T_cap=T_cap, dtype=dtype, ks=(kk,), membership="random",
                   seed=B * 3 + H * 5 + kk * 11 + T)
    G.run_clustered_layer(cfg, W.layer_inputs(cfg, 0))


def test_stream_read_probe_runs_and_checks_arguments():
    buf = torch.ones((1 << 20,), dtype=torch.float32, device="cuda")          # 4 MiB
    sink = torch.full((1,), 7.0, dtype=torch.float32, device="cuda")
    C.chai_stream_read_probe(buf, sink)
    C.chai_stream_read_probe(buf, sink, nbytes=16)
    torch.cuda.synchronize()
    assert float(sink[0]) == 7.0
    with pytest.raises(C.ChaiError) as e:
        C.chai_stream_read_probe(buf, sink, nbytes=24)                          # not a multiple of 16
    assert e.value.status == 2


def test_out_of_range_map_entries_stay_contained():
    """Device-side cluster maps cannot be checked on the host.  A corrupted entry (a cluster id or a representative
    outside its range) must neither make a kernel touch memory outside the caller's tensors nor disturb the rows of
    heads whose own entries are sound: the kernels clamp, and only the rows that depend on the bad entry change."""
    B, H, kk, T, T_cap = 2, 32, 8, 700, 768
    cfg = W.Config("corrupt", L=1, H=H, d=128, B=B, T=T, T_cap=T_cap, dtype=W.BF16, ks=(kk,), membership="random", seed=77)
    x = W.layer_inputs(cfg, 0)
    kd, vd, qd = dev(x.k), dev(x.v), dev(x.q)

    def run(h2c_h, rep_h):
        kc_whole, kc = G.guarded((B, kk, T_cap, 128), torch.bfloat16, 0.0)
        C.chai_compact_kcache(kd, dev(rep_h), kc, T)
        out_whole, out = G.guarded((B, H, 128), torch.float32, float("nan"))
        ws = G.poisoned_workspace(B, H, kk, T, 128, cfg.dtype)
        ws_guard = torch.full((ws.numel() + 2048,), 0x5A, dtype=torch.uint8, device="cuda")
        off = (-ws_guard.data_ptr()) % 256 + 256
        ws_in = ws_guard[off:off + ws.numel()]
        ws_in.fill_(0xFF)
        C.chai_decode_attention(qd, kc, vd, dev(h2c_h), dev(rep_h), T, cfg.scale, out, ws_in)
        torch.cuda.synchronize()
        assert G.guards_intact(kc_whole, (B, kk, T_cap, 128), 0.0)
        assert G.guards_intact(out_whole, (B, H, 128), float("nan"))
        assert bool((ws_guard[:off] == 0x5A).all()) and bool((ws_guard[off + ws.numel():] == 0x5A).all())
        return out.cpu().numpy()

    good = run(x.h2c, x.rep)
    assert np.all(np.isfinite(good))
    # 1. head (0, 3) names a cluster far outside [0, k); head (1, 5) a negative one
    h2c_bad = x.h2c.copy()
    h2c_bad[0, 3], h2c_bad[1, 5] = 9999, -7
    got = run(h2c_bad, x.rep)
    same = np.ones((B, H), bool)
    same[0, 3] = same[1, 5] = False
    assert np.array_equal(got[same], good[same])
    assert np.all(np.isfinite(got))                      # clamped into range: some valid cluster's probabilities
    # 2. the representative of cluster (0, 2) is a head id past H
    rep_bad = x.rep.copy()
    rep_bad[0, 2] = H + 100
    got = run(x.h2c, rep_bad)
    touched = np.zeros((B, H), bool)
    touched[0] = x.h2c[0] == 2                            # only the members of that cluster see other scores
    assert np.array_equal(got[~touched], good[~touched])
    assert np.all(np.isfinite(got))
