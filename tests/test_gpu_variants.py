"""GPU parity of the method's variants against the CPU oracle: the ablation that prunes values as well, the
nearest-to-mean representative, and membership that is the same for every request (static)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

if not torch.cuda.is_available():
    pytest.skip("needs a GPU", allow_module_level=True)

import paper_2403_08058_amd as C
import workloads as W
from oracle import chai_oracle as O

import gpu_util as G
from gpu_util import dev


@pytest.mark.parametrize("H,F,k", [(32, 25, 8), (72, 25, 16), (52, 5, 52), (256, 25, 3), (1, 1, 1), (32, 64, 32)])
def test_closest_representatives_bit_exact(H, F, k):
    g = np.random.default_rng(H * 1000 + F * 10 + k)
    B = 7
    feat = g.random((B, H, F)).astype(np.float32)
    lab = g.integers(0, k, size=(B, H)).astype(np.int32)           # arbitrary labels, some may be unused
    feat[0, : H // 2] = feat[0, 0]                                   # identical heads: ties go to the lowest
    rep = C.chai_closest_representatives(dev(feat), dev(lab), k)
    torch.cuda.synchronize()
    assert np.array_equal(rep.cpu().numpy(), O.closest_representatives(feat, lab, k))


def test_closest_representatives_drive_the_decode_path():
    """Features -> k-means -> nearest-to-mean representatives -> compaction -> decode, all on the device, against
    the oracle with the same maps: every entry point accepts a representative that is not the lowest member."""
    cfg = W.CONFIGS["cfg3"].reduced(L=1, B=3, T=600, T_cap=640)
    x = W.layer_inputs(cfg, 0)
    k = x.k_layer
    kd, vd, qd = dev(x.k), dev(x.v), dev(x.q)
    feat = C.chai_score_features(dev(x.q5), kd, W.N_TOK, cfg.scale)
    h2c, rep_low, _, _ = C.chai_assign_clusters(feat, dev(x.init_heads))
    rep = C.chai_closest_representatives(feat, h2c, k)
    torch.cuda.synchronize()
    feat_h, h2c_h, rep_h = feat.cpu().numpy(), h2c.cpu().numpy(), rep.cpu().numpy()
    assert np.array_equal(rep_h, O.closest_representatives(feat_h, h2c_h, k))
    assert np.any(rep_h != rep_low.cpu().numpy()), "the case should exercise a non-lowest representative"
    kc = torch.empty((cfg.B, k, cfg.T_cap, cfg.d), dtype=kd.dtype, device="cuda")
    C.chai_compact_kcache(kd, rep, kc, cfg.T)
    out = torch.full((cfg.B, cfg.H, cfg.d), float("nan"), dtype=torch.float32, device="cuda")
    ws = G.poisoned_workspace(cfg.B, cfg.H, k, cfg.T, cfg.d, cfg.dtype)
    C.chai_decode_attention(qd, kc, vd, h2c, rep, cfg.T, cfg.scale, out, ws)
    torch.cuda.synchronize()
    ref = O.clustered_decode(x.q, x.k, x.v, h2c_h, rep_h, cfg.T, cfg.scale)
    ok, worst = G.rows_close(out.cpu().numpy(), ref, G.RTOL[cfg.dtype])
    assert ok, worst


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
@pytest.mark.parametrize("B,H,kk,T,cap", [
    (2, 32, 8, 1300, 1333),      # split value chunks + combine
    (48, 32, 8, 300, 320),       # one workgroup per compact stream
    (1, 32, 1, 257, 300),        # one cluster holds every head
    (2, 52, 52, 64, 64),         # every head alone: dense attention
    (3, 72, 16, 1, 8),           # a single cached token
    (1, 1, 1, 33, 40),
])
def test_shared_v_decode_matches_oracle(dtype, B, H, kk, T, cap):
    cfg = W.Config("sharedv", L=1, H=H, d=128, B=B, T=T, T_cap=cap, dtype=dtype, ks=(kk,), membership="random",
                   seed=B * 3 + H * 5 + kk * 7 + T)
    x = W.layer_inputs(cfg, 0)
    h2c, rep = x.h2c.copy(), x.rep.copy()
    if kk >= 8:                                    # an unused slot: its heads move to slot 0
        for b in range(B):
            h2c[b][h2c[b] == 3] = 0
        rep = W.representatives(h2c, kk)
    kd, vd, qd, hd, rd = dev(x.k), dev(x.v), dev(x.q), dev(h2c), dev(rep)
    kc_whole, kc = G.guarded((B, kk, cap, 128), kd.dtype, 0.0)
    vc_whole, vc = G.guarded((B, kk, cap, 128), kd.dtype, 0.0)
    C.chai_compact_kcache(kd, rd, kc, T)
    C.chai_compact_kcache(vd, rd, vc, T)           # the same gather prunes the values
    out_whole, out = G.guarded((B, H, 128), torch.float32, float("nan"))
    ws = G.poisoned_workspace(B, H, kk, T, 128, dtype)
    C.chai_decode_attention_shared_v(qd, kc, vc, hd, rd, T, cfg.scale, out, ws)
    torch.cuda.synchronize()
    ref = O.shared_v_decode(x.q, x.k, x.v, h2c, rep, T, cfg.scale)
    ok, worst = G.rows_close(out.cpu().numpy(), ref, G.RTOL[dtype])
    assert ok, f"worst err/allowed = {worst:.3g}"
    assert G.guards_intact(out_whole, (B, H, 128), float("nan"))
    assert G.guards_intact(kc_whole, (B, kk, cap, 128), 0.0) and G.guards_intact(vc_whole, (B, kk, cap, 128), 0.0)
    # members of a cluster get the same row, bit for bit
    o = out.cpu().numpy()
    for b in range(B):
        for h in range(H):
            assert np.array_equal(o[b, h], o[b, rep[b, h2c[b, h]]])


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_shared_v_cache_growth(dtype):
    """Prompt in both compact caches, then tokens appended one by one, attention after each: against the oracle
    on full caches that grew the same way."""
    B, H, kk, T0, cap, steps = 2, 32, 8, 250, 260, 5
    g = np.random.default_rng(900 + dtype)
    h2c, rep = W.random_membership(g, B, H, kk)
    kf, vf = W.normal(g, (B, H, cap, 128), dtype), W.normal(g, (B, H, cap, 128), dtype)
    hd, rd = dev(h2c), dev(rep)
    kc = torch.zeros((B, kk, cap, 128), dtype=dev(kf[:1, :1, :1]).dtype, device="cuda")
    vc = torch.zeros_like(kc)
    C.chai_compact_kcache(dev(kf), rd, kc, T0)
    C.chai_compact_kcache(dev(vf), rd, vc, T0)
    vc_o = O.compact_kcache(vf, rep, T0, Tc_cap=cap, k_compact=np.zeros((B, kk, cap, 128), vf.dtype))
    ws = G.poisoned_workspace(B, H, kk, cap, 128, dtype)
    out = torch.empty((B, H, 128), dtype=torch.float32, device="cuda")
    scale = float(np.float32(128 ** -0.5))
    for s in range(steps):
        pos = T0 + s
        kn, vn, qn = W.normal(g, (B, H, 128), dtype), W.normal(g, (B, H, 128), dtype), W.normal(g, (B, H, 128), dtype)
        kf[:, :, pos], vf[:, :, pos] = kn, vn
        C.chai_append_kv_shared_v(dev(kn), dev(vn), rd, kc, vc, pos)
        # expected bytes of the compact value cache: the oracle's "row of the representative" append
        O.append_kv(vn, vn, rep, vc_o, vf.copy(), pos)
        C.chai_decode_attention_shared_v(dev(qn), kc, vc, hd, rd, pos + 1, scale, out, ws)
        torch.cuda.synchronize()
        ref = O.shared_v_decode(qn, kf, vf, h2c, rep, pos + 1, scale)
        ok, worst = G.rows_close(out.cpu().numpy(), ref, G.RTOL[dtype])
        assert ok, (s, worst)
    assert np.array_equal(W.torch_to_host_bits(vc), vc_o)


def test_static_membership_is_a_broadcast_of_the_maps():
    """Membership fixed offline and shared by every request (Section 3.3's static variant): the same maps in
    every batch row, through the unchanged decode path."""
    cfg = W.Config("static", L=1, H=32, d=128, B=4, T=700, T_cap=704, dtype=W.BF16, ks=(8,), membership="random",
                   seed=4321)
    x = W.layer_inputs(cfg, 0)
    x.h2c = np.tile(x.h2c[:1], (cfg.B, 1))
    x.rep = np.tile(x.rep[:1], (cfg.B, 1))
    G.run_clustered_layer(cfg, x)


def test_shared_v_argument_errors():
    q = torch.zeros((1, 32, 128), dtype=torch.bfloat16, device="cuda")
    kc = torch.zeros((1, 8, 64, 128), dtype=torch.bfloat16, device="cuda")
    maps = torch.zeros((1, 32), dtype=torch.int32, device="cuda")
    rep = torch.zeros((1, 8), dtype=torch.int32, device="cuda")
    out = torch.full((1, 32, 128), 7.0, dtype=torch.float32, device="cuda")
    ws = C.alloc_workspace(1, 32, 8, 64, 128, W.BF16)
    with pytest.raises(C.ChaiError) as e:
        C.chai_decode_attention_shared_v(q, kc, kc, maps, rep, 65, 0.1, out, ws)        # beyond the caches
    assert e.value.status == 2
    with pytest.raises(C.ChaiError) as e:
        C.chai_decode_attention_shared_v(q, kc, kc, maps, rep, 64, 0.1, out, ws[:256])  # workspace too small
    assert e.value.status == 4
    with pytest.raises(C.ChaiError) as e:
        C.chai_append_kv_shared_v(q, q, rep, kc, kc, 64)                                 # row past the capacity
    assert e.value.status == 2
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
@pytest.mark.parametrize("B,H,kk,T0,cap", [
    (2, 32, 8, 255, 300),        # the new token is the last of a score chunk, then the first of the next
    (3, 72, 16, 0, 16),          # the very first token: no cached row at all
    (48, 32, 8, 127, 140),       # one value workgroup per head; new token starts a 128-row value chunk
    (1, 32, 4, 1023, 1100),      # split value chunks + combine
])
def test_decode_step_folds_the_append(dtype, B, H, kk, T0, cap):
    """chai_decode_step at contexts T0+1, T0+2, ..: outputs against the oracle on full caches that grew the same
    way, and the caches themselves byte for byte against chai_append_kv's."""
    g = np.random.default_rng(B * 11 + H + T0 + dtype)
    h2c, rep = W.random_membership(g, B, H, kk)
    if kk >= 8:
        for b in range(B):
            h2c[b][h2c[b] == 3] = 0                      # an unused slot
        rep = W.representatives(h2c, kk)
    kf, vf = W.normal(g, (B, H, cap, 128), dtype), W.normal(g, (B, H, cap, 128), dtype)
    hd, rd = dev(h2c), dev(rep)
    tdt = torch.float32 if dtype == W.F32 else torch.bfloat16
    kc = torch.zeros((B, kk, cap, 128), dtype=tdt, device="cuda")
    kc_ref = torch.zeros_like(kc)
    vd, vd_ref = dev(vf), dev(vf)
    if T0 > 0:
        C.chai_compact_kcache(dev(kf), rd, kc, T0)
        C.chai_compact_kcache(dev(kf), rd, kc_ref, T0)
    ws = G.poisoned_workspace(B, H, kk, cap, 128, dtype)
    out_whole, out = G.guarded((B, H, 128), torch.float32, float("nan"))
    scale = float(np.float32(128 ** -0.5))
    for s in range(3):
        T = T0 + s + 1
        kn, vn, qn = W.normal(g, (B, H, 128), dtype), W.normal(g, (B, H, 128), dtype), W.normal(g, (B, H, 128), dtype)
        kf[:, :, T - 1], vf[:, :, T - 1] = kn, vn
        C.chai_decode_step(dev(qn), dev(kn), dev(vn), kc, vd, hd, rd, T, scale, out, ws)
        C.chai_append_kv(dev(kn), dev(vn), rd, kc_ref, vd_ref, T - 1)
        torch.cuda.synchronize()
        ref = O.clustered_decode(qn, kf, vf, h2c, rep, T, scale)
        ok, worst = G.rows_close(out.cpu().numpy(), ref, G.RTOL[dtype])
        assert ok, f"context {T}: worst err/allowed {worst:.3g}"
        assert torch.equal(kc.view(torch.uint8), kc_ref.view(torch.uint8)), f"compact K cache differs at context {T}"
        assert torch.equal(vd.view(torch.uint8), vd_ref.view(torch.uint8)), f"V cache differs at context {T}"
    assert G.guards_intact(out_whole, (B, H, 128), float("nan"))
