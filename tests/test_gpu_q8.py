"""Quantised K,V caches on the GPU (8-bit floating point E4M3 codes, one fp32 scale per row) against the CPU oracle:
codes and scales bit for bit (quantisation decides integers; both sides decide in fp32), the hardware widening of
all 254 finite codes exactly, and clustered decode attention over the same quantised bytes element by element."""
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


def _rows(seed, shape, dtype, sigma=1.0):
    x = W.normal(W.rng(seed, 0, "k"), shape, dtype, sigma=sigma)
    flat = x.reshape(-1, shape[-1])
    flat[3] = 0                                                   # an all-zero row
    f = W.as_f64(flat[5:6]).astype(np.float32)
    f[0, 7] = 1e-4 * np.abs(f).max()                              # an element deep in the subnormal codes
    f[0, 9] = np.abs(f).max() * np.float32(1.0625 / 1.75)         # lands on a tie between two codes
    flat[5:6] = W.store(f, dtype)
    return x


@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
def test_quantize_rows_bit_exact(dtype):
    x = _rows(6100, (3, 5, 77, 128), dtype, sigma=2.5)
    print(f"[q8] quantize_rows dtype={dtype}", flush=True)
    whole, codes = G.guarded(x.shape, torch.uint8, 0xAB)
    scales = torch.full(x.shape[:-1], float("nan"), dtype=torch.float32, device="cuda")
    C.chai_quantize_rows(dev(x), codes, scales)
    torch.cuda.synchronize()
    c_ref, s_ref = O.quantize_rows(x)
    assert np.array_equal(scales.cpu().numpy(), s_ref)
    assert np.array_equal(codes.cpu().numpy(), c_ref)
    assert G.guards_intact(whole, x.shape, 0xAB)
    # every code value occurs in a large enough sample, the subnormal range included
    assert len(np.unique(c_ref & 0x7F)) >= 100 and (c_ref & 0x7F).min() == 0 and ((c_ref & 0x78) == 0).any()


def test_hardware_decode_of_every_finite_code():
    """T = 1 makes the output equal to the dequantised value row: 254 codes through the kernel's widening."""
    B, H, k, d = 1, 2, 2, 128
    v8 = np.zeros((B, H, 1, d), np.uint8)
    v8[0, 0, 0] = np.arange(128) % 127            # 0 .. 126 (0x7f is the NaN code)
    v8[0, 1, 0] = 128 + np.arange(128) % 127      # the negative ones
    vs = np.full((B, H, 1), 1.0, np.float32)
    vs[0, 1, 0] = 0.75
    k8 = np.full((B, k, 1, d), 0x38, np.uint8)
    ks = np.ones((B, k, 1), np.float32)
    q = W.store(np.ones((B, H, d), np.float32), W.BF16)
    h2c = np.array([[0, 1]], np.int32)
    rep = np.array([[0, 1]], np.int32)
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    ws = torch.empty((C.chai_decode_q8_workspace_bytes(B, H, k, 1),), dtype=torch.uint8, device="cuda")
    C.chai_decode_attention_q8(dev(q), dev(k8), dev(ks), dev(v8), dev(vs), dev(h2c), dev(rep), 1, 1.0, out, ws)
    torch.cuda.synchronize()
    want = np.array([[O.e4m3_decode(int(c)) for c in v8[0, 0, 0]],
                     [O.e4m3_decode(int(c)) * 0.75 for c in v8[0, 1, 0]]])
    assert np.array_equal(out.cpu().numpy()[0].astype(np.float64), want)


def _run_case(seed, B, H, kk, T, T_cap, dtype, sized=None):
    cfg_scale = float(np.float32(1.0 / np.sqrt(128.0)))
    g = W.rng(seed, 0, "member")
    h2c, rep = (W.sized_membership(g, B, H, sized) if sized else W.random_membership(g, B, H, kk))
    q = W.normal(W.rng(seed, 0, "q"), (B, H, 128), dtype)
    kf = W.normal(W.rng(seed, 0, "k"), (B, H, T_cap, 128), W.BF16)
    vf = W.normal(W.rng(seed, 0, "v"), (B, H, T_cap, 128), W.BF16, sigma=1.5)
    k8f, ksf = O.quantize_rows(kf)
    v8, vs = O.quantize_rows(vf)
    # the compact key cache holds the representatives' quantised streams
    k8c = np.zeros((B, kk, T_cap, 128), np.uint8)
    ksc = np.zeros((B, kk, T_cap), np.float32)
    for b in range(B):
        for j in range(kk):
            if rep[b, j] >= 0:
                k8c[b, j], ksc[b, j] = k8f[b, rep[b, j]], ksf[b, rep[b, j]]
    whole, out = G.guarded((B, H, 128), torch.float32, float("nan"))
    probs = torch.full((B, kk, T), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty((C.chai_decode_q8_workspace_bytes(B, H, kk, T_cap),), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    args = (dev(q), dev(k8c), dev(ksc), dev(v8), dev(vs), dev(h2c), dev(rep), T, cfg_scale)
    C.chai_decode_attention_q8(*args, out, ws, probs_out=probs)
    out2 = torch.empty_like(out)
    ws.fill_(0xFF)
    C.chai_decode_attention_q8(*args, out2, ws)               # the instantiation without the probability copy
    torch.cuda.synchronize()
    ref, p_ref = O.clustered_decode_q8(q, k8f, ksf, v8, vs, h2c, rep, T, cfg_scale, want_probs=True)
    ok, worst = G.rows_close(out.cpu().numpy(), ref, G.RTOL[dtype])
    assert ok, f"quantised decode off: worst err/allowed {worst:.3g}"
    ok2, worst2 = G.rows_close(out2.cpu().numpy(), ref, G.RTOL[dtype])
    assert ok2, worst2
    assert G.guards_intact(whole, (B, H, 128), float("nan"))
    used = rep >= 0
    p = probs.cpu().numpy().astype(np.float64)
    assert np.abs(p[used] - p_ref[used]).max() <= G.PROB_ATOL and np.abs(p[used].sum(-1) - 1).max() <= 1e-5
    return worst


@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
@pytest.mark.parametrize("B,H,kk,T,T_cap", [
    (2, 32, 8, 1300, 1333),        # LLaMa-7B head shape, split heads + combine
    (13, 32, 8, 777, 800),         # >= 384 heads: one workgroup per head
    (3, 72, 16, 641, 700),         # OPT-66B head shape
    (1, 5, 5, 1, 4),               # a single cached token
    (2, 7, 3, 63, 64), (2, 7, 3, 64, 64), (2, 7, 3, 65, 70),      # around one batch of 64 rows
])
def test_decode_q8_matches_oracle(dtype, B, H, kk, T, T_cap):
    print(f"[q8] decode B={B} H={H} k={kk} T={T} dtype={dtype}", flush=True)
    _run_case(6200 + T, B, H, kk, T, T_cap, dtype)


def test_decode_q8_long_context_skewed_clusters():
    print("[q8] decode B=2 H=32 T=4500 sizes 20/6/4/2", flush=True)
    _run_case(6300, 2, 32, 4, 4500, 4608, W.BF16, sized=(20, 6, 4, 2))


@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
def test_append_kv_q8_bit_exact(dtype):
    B, H, kk, Tc_cap, T_cap = 3, 32, 8, 40, 48
    g = W.rng(6400, 0, "member")
    h2c, rep = W.random_membership(g, B, H, kk)
    rep[1, kk - 1] = -1                                              # an unused slot is left alone
    k_new = _rows(6401, (B, H, 128), dtype)
    v_new = _rows(6402, (B, H, 128), dtype, sigma=3.0)
    k8 = torch.full((B, kk, Tc_cap, 128), 0x11, dtype=torch.uint8, device="cuda")
    ks = torch.full((B, kk, Tc_cap), 7.0, dtype=torch.float32, device="cuda")
    v8 = torch.full((B, H, T_cap, 128), 0x22, dtype=torch.uint8, device="cuda")
    vs = torch.full((B, H, T_cap), 9.0, dtype=torch.float32, device="cuda")
    pos = 17
    C.chai_append_kv_q8(dev(k_new), dev(v_new), dev(rep), k8, ks, v8, vs, pos)
    torch.cuda.synchronize()
    kc, ksc = O.quantize_rows(k_new)
    vc, vsc = O.quantize_rows(v_new)
    k8_ref = np.full((B, kk, Tc_cap, 128), 0x11, np.uint8)
    ks_ref = np.full((B, kk, Tc_cap), 7.0, np.float32)
    for b in range(B):
        for j in range(kk):
            if rep[b, j] >= 0:
                k8_ref[b, j, pos], ks_ref[b, j, pos] = kc[b, rep[b, j]], ksc[b, rep[b, j]]
    v8_ref = np.full((B, H, T_cap, 128), 0x22, np.uint8)
    vs_ref = np.full((B, H, T_cap), 9.0, np.float32)
    v8_ref[:, :, pos], vs_ref[:, :, pos] = vc, vsc
    assert np.array_equal(k8.cpu().numpy(), k8_ref) and np.array_equal(ks.cpu().numpy(), ks_ref)
    assert np.array_equal(v8.cpu().numpy(), v8_ref) and np.array_equal(vs.cpu().numpy(), vs_ref)


def test_q8_argument_errors():
    L = C.lib()
    assert L.chai_quantize_rows(None, 1, 4, 128, None, None, None) == 1
    x = torch.zeros((4, 128), dtype=torch.bfloat16, device="cuda")
    c = torch.zeros((4, 128), dtype=torch.uint8, device="cuda")
    s = torch.zeros((4,), dtype=torch.float32, device="cuda")
    assert L.chai_quantize_rows(x.data_ptr(), 1, 4, 64, c.data_ptr(), s.data_ptr(), None) == 5      # d != 128
    assert L.chai_quantize_rows(x.data_ptr(), 9, 4, 128, c.data_ptr(), s.data_ptr(), None) == 3
    assert L.chai_quantize_rows(x.data_ptr(), 1, -1, 128, c.data_ptr(), s.data_ptr(), None) == 2
    assert L.chai_quantize_rows(x.data_ptr(), 1, 0, 128, c.data_ptr(), s.data_ptr(), None) == 0
    assert C.chai_decode_q8_workspace_bytes(4, 72, 16, 2048) >= C.chai_decode_q8_workspace_bytes(4, 72, 16, 640) > 0
    assert C.chai_decode_q8_workspace_bytes(4, 72, 73, 2048) == 0


def test_q8_full_size_sampled_heads():
    """Quantised decode at the full LLaMa-7B-shaped size, in the launch configuration bench.py times: caches
    quantised by the library, sampled (batch row, head) pairs checked against the oracle's own quantisation of the
    bf16 rows and its attention over those codes."""
    cfg = W.CONFIGS["cfg2"]
    B, H, d, T, kk = cfg.B, cfg.H, cfg.d, cfg.T, 8
    seed = cfg.seed * 4001
    kc = W.device_normal((B, kk, T, d), cfg.dtype, seed)
    v = W.device_normal((B, H, T, d), cfg.dtype, seed + 1)
    q = W.device_normal((B, H, d), cfg.dtype, seed + 2)
    h2c_h, rep_h = W.random_membership(W.rng(cfg.seed, 0, "member"), B, H, kk)
    h2c, rep = dev(h2c_h), dev(rep_h)
    print(f"[q8 full size] B={B} H={H} k={kk} T={T}", flush=True)
    k8, ks = C.chai_quantize_rows(kc)
    v8, vs = C.chai_quantize_rows(v)
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    ws = torch.empty((C.chai_decode_q8_workspace_bytes(B, H, H, T),), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    C.chai_decode_attention_q8(q, k8, ks, v8, vs, h2c, rep, T, cfg.scale, out, ws)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    g = np.random.default_rng(7)
    for _ in range(12):
        b, h = int(g.integers(B)), int(g.integers(H))
        c = int(h2c_h[b, h])
        kq, ksq = O.quantize_rows(W.torch_to_host_bits(kc[b, c]))
        vq, vsq = O.quantize_rows(W.torch_to_host_bits(v[b, h]))
        assert np.array_equal(kq, k8[b, c].cpu().numpy()) and np.array_equal(ksq, ks[b, c].cpu().numpy())
        assert np.array_equal(vq, v8[b, h].cpu().numpy()) and np.array_equal(vsq, vs[b, h].cpu().numpy())
        qr = W.torch_to_host_bits(q[b, rep_h[b, c]])
        ref = O.clustered_decode_q8(np.stack([qr, qr * 0])[None], np.stack([kq, kq * 0])[None],
                                    np.stack([ksq, ksq * 0])[None], np.stack([vq * 0, vq])[None],
                                    np.stack([vsq * 0, vsq])[None], np.zeros((1, 2), np.int32),
                                    np.zeros((1, 1), np.int32), T, cfg.scale)[0, 1]
        ok, worst = G.rows_close(out[b, h].cpu().numpy()[None], ref[None], G.RTOL[cfg.dtype])
        assert ok, f"(b={b}, h={h}): err/allowed {worst:.3g}"
