"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py times
(same B, H, k, T per layer, same workspace sizing).  The oracle cannot sweep whole layers at these sizes in a test,
so outputs are checked on sampled (batch row, head) pairs computed one by one by the oracle from the bytes
downloaded from the device, plus properties that hold at any size (probability rows sum to 1, compact rows are
the representatives' rows, cluster maps identical to the oracle's k-means on the device's feature bits)."""
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

N_SAMPLES = 20


def oracle_one_head(q_rep, k_rep, v_head, T, scale):
    """out of one head whose cluster is represented by (q_rep, k_rep): a two-head, one-cluster oracle call."""
    d = q_rep.shape[-1]
    T_cap = k_rep.shape[0]
    q = np.stack([q_rep, np.zeros_like(q_rep)])[None]                      # [1,2,d]
    k = np.stack([k_rep, np.zeros_like(k_rep)])[None]                      # [1,2,T_cap,d]
    v = np.stack([np.zeros_like(v_head), v_head])[None]
    h2c = np.zeros((1, 2), np.int32)
    rep = np.zeros((1, 1), np.int32)
    out, p = O.clustered_decode(q, k, v, h2c, rep, T, scale, want_probs=True)
    return out[0, 1], p[0, 0]


def check_layer(cfg, layer, T, q, kfull, v, h2c_d, rep_d, kc, seed):
    """Decode one full-size layer on the GPU and compare sampled heads with the oracle."""
    B, H, d = cfg.B, cfg.H, cfg.d
    k = rep_d.shape[1]
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    probs = torch.empty((B, k, T), dtype=torch.float32, device="cuda")
    ws = C.alloc_workspace(B, H, H, T, d, cfg.dtype)         # as bench.py sizes it
    ws.fill_(0xFF)
    C.chai_decode_attention(q, kc, v, h2c_d, rep_d, T, cfg.scale, out, ws, probs_out=probs)
    torch.cuda.synchronize()
    h2c, rep = h2c_d.cpu().numpy(), rep_d.cpu().numpy()
    assert bool(torch.isfinite(out).all())
    used = torch.as_tensor(rep >= 0, device="cuda")
    psum = probs.sum(-1)
    assert float((psum[used] - 1).abs().max()) < 2e-5 and bool((probs[used] >= 0).all())
    g = np.random.default_rng(seed)
    worst = 0.0
    for _ in range(N_SAMPLES):
        b, h = int(g.integers(B)), int(g.integers(H))
        c = int(h2c[b, h])
        r = int(rep[b, c])
        q_rep = W.torch_to_host_bits(q[b, r])
        k_rep = W.torch_to_host_bits(kfull[b, r]) if kfull is not None else W.torch_to_host_bits(kc[b, c])
        # compaction: the compact stream of the cluster is the representative's stream, byte for byte
        assert np.array_equal(W.torch_to_host_bits(kc[b, c, :T]), k_rep[:T])
        ref, p_ref = oracle_one_head(q_rep, k_rep, W.torch_to_host_bits(v[b, h]), T, cfg.scale)
        ok, ratio = G.rows_close(out[b, h].cpu().numpy()[None], ref[None], G.RTOL[cfg.dtype])
        assert ok, f"{cfg.name} layer {layer} (b={b}, h={h}): err/allowed {ratio:.3g}"
        assert np.abs(probs[b, c].cpu().numpy() - p_ref).max() <= G.PROB_ATOL
        worst = max(worst, ratio)
    return worst


def device_membership(cfg, layer, k, kfull, q5, init):
    feat = C.chai_score_features(q5, kfull, W.N_TOK, cfg.scale)
    h2c, rep, ncl, it = C.chai_assign_clusters(feat, W.host_to_torch(init))
    torch.cuda.synchronize()
    h2c_o, rep_o, ncl_o, it_o = O.kmeans(feat.cpu().numpy(), init)
    assert np.array_equal(h2c.cpu().numpy(), h2c_o) and np.array_equal(rep.cpu().numpy(), rep_o)
    assert np.array_equal(ncl.cpu().numpy(), ncl_o) and np.array_equal(it.cpu().numpy(), it_o)
    return h2c, rep


@pytest.mark.parametrize("name,layers", [("cfg2", [0, 5]), ("cfg3", [0, 1, 2]), ("cfg5", [0])])
def test_full_size_layers(name, layers):
    cfg = W.CONFIGS[name]
    B, H, d, T = cfg.B, cfg.H, cfg.d, cfg.T
    for layer in layers:
        k = cfg.ks[layer]
        print(f"[full-size] {name} layer {layer}: B={B} H={H} k={k} T={T}", flush=True)
        seed = cfg.seed * 1009 + layer
        if cfg.membership == "planted":
            groups = W.planted_partition(W.rng(cfg.seed, layer, "planted"), B, H, k)
            kfull = W.device_centroid_plus_noise(groups, k, T, d, cfg.dtype, seed)
            q5 = W.device_centroid_plus_noise(groups, k, W.N_TOK, d, cfg.dtype, seed + 2)
            q = W.device_centroid_plus_noise(groups, k, 1, d, cfg.dtype, seed + 4)[:, :, 0, :].contiguous()
            init = W.one_head_per_group(W.rng(cfg.seed, layer, "init"), groups, k)
            h2c, rep = device_membership(cfg, layer, k, kfull, q5, init)
            for b in range(B):       # k-means recovers the planted groups
                seen = {}
                assert h2c[b].cpu().tolist() == [seen.setdefault(int(a), len(seen)) for a in groups[b]]
        else:
            kfull = W.device_normal((B, H, T, d), cfg.dtype, seed)
            q = W.device_normal((B, H, d), cfg.dtype, seed + 4)
            if cfg.membership == "kmeans":
                q5 = W.device_normal((B, H, W.N_TOK, d), cfg.dtype, seed + 2)
                init = W.distinct_heads(W.rng(cfg.seed, layer, "init"), B, H, k)
                h2c, rep = device_membership(cfg, layer, k, kfull, q5, init)
            else:
                hh, rr = W.sized_membership(W.rng(cfg.seed, layer, "member"), B, H, cfg.sizes)
                h2c, rep = W.host_to_torch(hh), W.host_to_torch(rr)
        v = W.device_normal((B, H, T, d), cfg.dtype, seed + 6)
        kc = torch.empty((B, k, T, d), dtype=torch.bfloat16, device="cuda")
        C.chai_compact_kcache(kfull, rep, kc, T)
        worst = check_layer(cfg, layer, T, q, kfull, v, h2c, rep, kc, seed)
        print(f"[full-size] {name} layer {layer}: worst err/allowed over {N_SAMPLES} heads = {worst:.3f}", flush=True)
        del kfull, v, kc


def test_full_size_cfg4_prompt_then_decode():
    """OPT-66B shape, one layer at full size: 512-token prompt -> membership -> compaction -> decode steps with
    cache growth at contexts 513.., then the same at the end of the cache (context 2048)."""
    cfg = W.CONFIGS["cfg4"]
    B, H, d, k, T_cap = cfg.B, cfg.H, cfg.d, cfg.ks[0], cfg.T_cap
    seed = cfg.seed * 1009
    kfull = W.device_normal((B, H, T_cap, d), cfg.dtype, seed)
    v = W.device_normal((B, H, T_cap, d), cfg.dtype, seed + 6)
    q5 = W.device_normal((B, H, W.N_TOK, d), cfg.dtype, seed + 2)
    init = W.distinct_heads(W.rng(cfg.seed, 0, "init"), B, H, k)
    h2c, rep = device_membership(cfg, 0, k, kfull, q5, init)
    kc = torch.zeros((B, k, T_cap, d), dtype=torch.bfloat16, device="cuda")
    for start in (cfg.prompt, T_cap - 3):
        C.chai_compact_kcache(kfull, rep, kc, start)
        for step in range(3):
            pos = start + step
            qn = W.device_normal((B, H, d), cfg.dtype, seed + 100 + pos)
            kn = W.device_normal((B, H, d), cfg.dtype, seed + 200 + pos)
            vn = W.device_normal((B, H, d), cfg.dtype, seed + 300 + pos)
            C.chai_append_kv(kn, vn, rep, kc, v, pos)
            kfull[:, :, pos] = kn                      # the full cache only serves the comparison
            print(f"[full-size] cfg4 context {pos + 1}", flush=True)
            check_layer(cfg, 0, pos + 1, qn, kfull, v, h2c, rep, kc, seed + pos)
            assert torch.equal(v[:, :, pos], vn)


def test_phases_equal_the_fused_call():
    """chai_decode_scores + chai_decode_values (and their _timed forms) give bit for bit what
    chai_decode_attention gives."""
    cfg = W.CONFIGS["cfg2"].reduced(L=1, B=4, T=1500, T_cap=1536)
    x = W.layer_inputs(cfg, 0)
    B, H, d, T = cfg.B, cfg.H, cfg.d, cfg.T
    h2c_h, rep_h = W.random_membership(np.random.default_rng(3), B, H, 8)
    q, kf, v, h2c, rep = G.dev(x.q), G.dev(x.k), G.dev(x.v), G.dev(h2c_h), G.dev(rep_h)
    kc = torch.empty((B, 8, cfg.T_cap, d), dtype=torch.bfloat16, device="cuda")
    C.chai_compact_kcache(kf, rep, kc, T)
    outs = [torch.empty((B, H, d), dtype=torch.float32, device="cuda") for _ in range(3)]
    ws = G.poisoned_workspace(B, H, 8, T, d, cfg.dtype)
    C.chai_decode_attention(q, kc, v, h2c, rep, T, cfg.scale, outs[0], ws)
    ws.fill_(0xFF)
    C.chai_decode_scores(q, kc, rep, T, cfg.scale, ws)
    C.chai_decode_values(v, h2c, rep, T, outs[1], ws)
    ws.fill_(0xFF)
    C.chai_decode_scores_timed(q, kc, rep, T, cfg.scale, ws)
    C.chai_decode_values_timed(v, h2c, rep, T, outs[2], ws)
    torch.cuda.synchronize()
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
    ok, worst = G.rows_close(outs[0].cpu().numpy(), O.clustered_decode(x.q, x.k, x.v, h2c_h, rep_h, T, cfg.scale),
                             G.RTOL[cfg.dtype])
    assert ok, worst
