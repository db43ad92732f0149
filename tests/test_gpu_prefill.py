"""GPU parity of the clustered prefill attention (matrix-core kernel) against the CPU oracle."""
import math

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

# Probabilities are rounded to fp16 (11 significant bits) before the second product, everything else is exact
# bf16 products with fp32 accumulation: errors of ~2^-12 per term average out to a few 1e-4 per row, inside the
# 2e-3 contract for bf16 inputs.
RTOL_PREFILL = 2e-3


def run_case(B, H, kk, Tq, q_start, T_cap, seed, membership="random", sizes=None):
    g = np.random.default_rng(seed)
    q = W.normal(g, (B, H, Tq, 128), W.BF16)
    k = W.normal(g, (B, H, T_cap, 128), W.BF16)
    v = W.normal(g, (B, H, T_cap, 128), W.BF16)
    nan = np.uint16(0x7FC0)
    k[:, :, q_start + Tq:], v[:, :, q_start + Tq:] = nan, nan          # positions past the block are never read
    if membership == "sized":
        h2c, rep = W.sized_membership(g, B, H, sizes)
    else:
        h2c, rep = W.random_membership(g, B, H, kk)
    scale = float(np.float32(1 / math.sqrt(128)))
    kd, vd, qd, hd, rd = dev(k), dev(v), dev(q), dev(h2c), dev(rep)
    kc = torch.zeros((B, kk, T_cap, 128), dtype=torch.bfloat16, device="cuda")
    C.chai_compact_kcache(kd, rd, kc, q_start + Tq)
    whole, out = G.guarded((B, H, Tq, 128), torch.float32, float("nan"))
    ws = torch.full((max(C.chai_prefill_workspace_bytes(B, H, kk, q_start + Tq), 256),), 0xFF, dtype=torch.uint8, device="cuda")
    C.chai_prefill_attention(qd, kc, vd, hd, rd, q_start, scale, out, ws)
    torch.cuda.synchronize()
    ref = O.clustered_prefill(q, k, v, h2c, rep, q_start, scale)
    ok, worst = G.rows_close(out.cpu().numpy(), ref, RTOL_PREFILL)
    assert ok, f"prefill off: worst err/allowed {worst:.3g}"
    assert G.guards_intact(whole, (B, H, Tq, 128), float("nan"))
    return worst, (q, k, v, qd, kd, vd)


@pytest.mark.parametrize("B,H,kk,Tq,q_start,T_cap", [
    (2, 8, 3, 200, 5, 256),        # ragged last query tile, odd group sizes
    (1, 32, 8, 300, 5, 305),       # LLaMa-7B head structure, cache exactly full
    (1, 32, 32, 130, 0, 160),      # every head alone, block starts at position 0
    (2, 52, 4, 64, 100, 200),      # block in the middle of the sequence
    (1, 72, 16, 1, 40, 64),        # a single query row
    (1, 4, 1, 129, 31, 192),       # one cluster for all heads
    (16, 32, 8, 640, 5, 645),      # three query tiles sent singly, the largest first
    (22, 32, 8, 640, 5, 645),      # enough workgroups for paired query tiles, odd tile count (the middle one alone)
])
def test_prefill_matches_oracle(B, H, kk, Tq, q_start, T_cap):
    worst, _ = run_case(B, H, kk, Tq, q_start, T_cap, seed=B * 31 + H * 7 + Tq)
    print(f"worst err/allowed = {worst:.3f}")


def test_prefill_skewed_clusters():
    run_case(2, 32, 4, 260, 5, 272, seed=5, membership="sized", sizes=(20, 6, 4, 2))


def test_dense_prefill_and_one_head_per_cluster():
    B, H, Tq, q_start, T_cap = 1, 8, 190, 5, 200
    worst, (q, k, v, qd, kd, vd) = run_case(B, H, H, Tq, q_start, T_cap, seed=9)
    scale = float(np.float32(1 / math.sqrt(128)))
    out = torch.empty((B, H, Tq, 128), dtype=torch.float32, device="cuda")
    ws = torch.empty((max(C.chai_prefill_workspace_bytes(B, H, H, q_start + Tq), 256),), dtype=torch.uint8, device="cuda")
    C.chai_dense_prefill_attention(qd, kd, vd, q_start, scale, out, ws)
    torch.cuda.synchronize()
    ident = np.tile(np.arange(H, dtype=np.int32), (B, 1))
    ref = O.clustered_prefill(q, k, v, ident, ident, q_start, scale)
    ok, worst = G.rows_close(out.cpu().numpy(), ref, RTOL_PREFILL)
    assert ok, worst


def test_prefill_rows_equal_decode_steps():
    """Row i of the prefill block is what the decode kernels give at context q_start + i + 1 (to fp16 rounding)."""
    B, H, kk, Tq, q_start, T_cap = 1, 32, 8, 140, 5, 160
    g = np.random.default_rng(77)
    q = W.normal(g, (B, H, Tq, 128), W.BF16)
    k = W.normal(g, (B, H, T_cap, 128), W.BF16)
    v = W.normal(g, (B, H, T_cap, 128), W.BF16)
    h2c, rep = W.random_membership(g, B, H, kk)
    qd, kd, vd, hd, rd = dev(q), dev(k), dev(v), dev(h2c), dev(rep)
    kc = torch.zeros((B, kk, T_cap, 128), dtype=torch.bfloat16, device="cuda")
    C.chai_compact_kcache(kd, rd, kc, q_start + Tq)
    out = torch.empty((B, H, Tq, 128), dtype=torch.float32, device="cuda")
    ws = torch.empty((max(C.chai_prefill_workspace_bytes(B, H, kk, q_start + Tq), 256),), dtype=torch.uint8, device="cuda")
    C.chai_prefill_attention(qd, kc, vd, hd, rd, q_start, 0.0884, out, ws)
    dws = C.alloc_workspace(B, H, kk, T_cap, 128, C.CHAI_BF16)
    for i in (0, 63, 139):
        o = torch.empty((B, H, 128), dtype=torch.float32, device="cuda")
        C.chai_decode_attention(qd[:, :, i].contiguous(), kc, vd, hd, rd, q_start + i + 1, 0.0884, o, dws)
        torch.cuda.synchronize()
        ok, worst = G.rows_close(out[:, :, i].cpu().numpy(), o.cpu().numpy().astype(np.float64), RTOL_PREFILL)
        assert ok, (i, worst)


def test_prefill_argument_errors():
    B, H, kk, Tq = 1, 8, 2, 16
    q = torch.zeros((B, H, Tq, 128), dtype=torch.bfloat16, device="cuda")
    kc = torch.zeros((B, kk, 32, 128), dtype=torch.bfloat16, device="cuda")
    v = torch.zeros((B, H, 32, 128), dtype=torch.bfloat16, device="cuda")
    h2c = torch.zeros((B, H), dtype=torch.int32, device="cuda")
    rep = torch.zeros((B, kk), dtype=torch.int32, device="cuda")
    out = torch.zeros((B, H, Tq, 128), dtype=torch.float32, device="cuda")
    ws = torch.empty((max(C.chai_prefill_workspace_bytes(B, H, kk, 32), 256),), dtype=torch.uint8, device="cuda")

    def status(*a):
        with pytest.raises(C.ChaiError) as e:
            C.chai_prefill_attention(*a)
        return e.value.status

    assert status(q, kc, v, h2c, rep, 17, 0.1, out, ws) == 2              # block runs past the cache
    assert status(q, kc, v, h2c, rep, -1, 0.1, out, ws) == 2
    assert status(q, kc, v, h2c, rep, 0, 0.1, out, ws[:64]) == 4
    qf = torch.zeros((B, H, Tq, 128), dtype=torch.float32, device="cuda")
    kf = torch.zeros((B, kk, 32, 128), dtype=torch.float32, device="cuda")
    vf = torch.zeros((B, H, 32, 128), dtype=torch.float32, device="cuda")
    assert status(qf, kf, vf, h2c, rep, 0, 0.1, out, ws) == 5              # fp32 inputs not supported here


@pytest.mark.parametrize("name,T", [("cfg2", 2048), ("cfg4", 512), ("cfg5", 32768)])
def test_prefill_full_size_sampled(name, T):
    """Prefill at the sizes bench.py --mode prefill times (same B, H, k, prompt length, positions 5..T-1, same
    workspace sizing).  The oracle computes sampled (batch row, head, query rows) one by one from the bytes
    downloaded from the device; properties that hold at any size: finite everywhere, members of a cluster with
    identical values get identical rows."""
    cfg = W.CONFIGS[name]
    B, H, d = cfg.B, cfg.H, cfg.d
    kk = cfg.ks[-1]
    q_start, Tq = W.N_TOK, T - W.N_TOK
    print(f"[full-size prefill] {name}: B={B} H={H} k={kk} T={T}", flush=True)
    g = W.rng(cfg.seed, 0, "member", extra=7)
    if cfg.membership == "skewed":
        h2c, rep = W.sized_membership(g, B, H, cfg.sizes)
    else:
        h2c, rep = W.random_membership(g, B, H, kk)
    seed = cfg.seed * 4001
    q = W.device_normal((B, H, Tq, d), cfg.dtype, seed + 1)
    kfull = W.device_normal((B, H, T, d), cfg.dtype, seed + 2)
    v = W.device_normal((B, H, T, d), cfg.dtype, seed + 3)
    # two members of one cluster share their values: their output rows must then be equal bit for bit
    b0 = 0
    members = [np.nonzero(h2c[b0] == c)[0] for c in range(kk)]
    pair = next(m for m in members if len(m) >= 2)
    v[b0, pair[1]] = v[b0, pair[0]]
    hd, rd = W.host_to_torch(h2c), W.host_to_torch(rep)
    kc = torch.empty((B, kk, T, d), dtype=torch.bfloat16, device="cuda")
    C.chai_compact_kcache(kfull, rd, kc, T)
    out = torch.full((B, H, Tq, d), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.full((C.chai_prefill_workspace_bytes(B, H, H, T),), 0xFF, dtype=torch.uint8, device="cuda")
    C.chai_prefill_attention(q, kc, v, hd, rd, q_start, cfg.scale, out, ws)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    assert torch.equal(out[b0, pair[0]], out[b0, pair[1]])
    gs = np.random.default_rng(cfg.seed + T)
    rows = 6
    worst = 0.0
    for s in range(10):
        b, h = int(gs.integers(B)), int(gs.integers(H))
        # blocks of rows at the start, around tile edges and at the end of the prompt
        i0 = [0, 250, Tq - rows, int(gs.integers(Tq - rows)), int(gs.integers(Tq - rows))][s % 5]
        i0 = max(min(i0, Tq - rows), 0)
        c = int(h2c[b, h]); r = int(rep[b, c])
        n = q_start + i0 + rows                                # keys the last sampled row sees
        qh = W.torch_to_host_bits(q[b, r, i0:i0 + rows])       # [rows, d]
        kh = W.torch_to_host_bits(kfull[b, r, :n])
        vh = W.torch_to_host_bits(v[b, h, :n])
        q2 = np.stack([qh, np.zeros_like(qh)])[None]           # head 0 = representative, head 1 = the sampled head
        k2 = np.stack([kh, np.zeros_like(kh)])[None]
        v2 = np.stack([np.zeros_like(vh), vh])[None]
        ref = O.clustered_prefill(q2, k2, v2, np.zeros((1, 2), np.int32), np.zeros((1, 1), np.int32), q_start + i0,
                                  cfg.scale)[0, 1]
        ok, ratio = G.rows_close(out[b, h, i0:i0 + rows].cpu().numpy(), ref, RTOL_PREFILL)
        assert ok, f"{name} (b={b}, h={h}, rows {i0}..): err/allowed {ratio:.3g}"
        worst = max(worst, ratio)
    print(f"worst err/allowed = {worst:.3f}")


def _random_prefill_shapes(n, seed):
    g = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        H = int(g.choice([2, 5, 8, 32, 52]))
        B = int(g.choice([1, 2, 3]))
        kk = int(g.integers(1, min(H, 16) + 1))
        Tq = int(g.choice([1, 31, 33, 64, 65, 255, 257, 300, 513]))
        q_start = int(g.choice([0, 1, 5, 63, 64, 200]))
        out.append((B, H, kk, Tq, q_start, q_start + Tq + int(g.integers(0, 5))))
    return out


@pytest.mark.parametrize("B,H,kk,Tq,q_start,T_cap", _random_prefill_shapes(10, 77001))
def test_prefill_random_shapes(B, H, kk, Tq, q_start, T_cap):
    run_case(B, H, kk, Tq, q_start, T_cap, seed=B + 3 * H + 7 * kk + Tq + q_start)
