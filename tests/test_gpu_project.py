"""GPU parity of the pruned query/key projection (matrix-core kernel) against the CPU oracle."""
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


def bf16_ulp(ref):
    """Spacing of bf16 numbers around |ref| (8 significant bits), never below the smallest normal's spacing."""
    a = np.maximum(np.abs(ref), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(a)) - 7)


def check_rounded(gpu_bits, ref, sum_abs, what):
    """The device accumulates exact bf16 products in fp32 and rounds ONCE to bf16; the oracle gives the unrounded
    fp64 value.  A correct result is a bf16 neighbour of the exact value: within half a bf16 spacing plus the
    fp32 accumulation error (D terms, a few 2^-24 of the sum of magnitudes)."""
    got = W.bf16_bits_to_f32(gpu_bits).astype(np.float64)
    allowed = 0.5 * bf16_ulp(ref) + 3e-6 * sum_abs
    bad = np.abs(got - ref) > allowed
    assert not bad.any(), f"{what}: {int(bad.sum())} of {bad.size} values off; worst {np.max(np.abs(got - ref) / allowed):.3f} of allowed"
    # and it is not systematically one-sided: most values are the nearest bf16
    nearest = np.abs(got - ref) <= 0.5 * bf16_ulp(ref) * (1 + 1e-9)
    assert nearest.mean() > 0.98, f"{what}: only {nearest.mean():.3f} of the values are the nearest bf16"


def run_case(B, H, kk, Tn, D, pos0, Tc_cap, seed, holes=False):
    g = np.random.default_rng(seed)
    d = 128
    x = W.normal(g, (B, Tn, D), W.BF16)
    w_q, w_k = W.normal(g, (H * d, D), W.BF16), W.normal(g, (H * d, D), W.BF16)
    _, rep = W.random_membership(g, B, H, kk)
    if holes and kk > 2:
        rep[0, kk - 1] = -1                                   # an unused slot
    q_whole, q_out = G.guarded((B, H, Tn, d), torch.bfloat16, 3.0)
    k_whole, kc = G.guarded((B, kk, Tc_cap, d), torch.bfloat16, 5.0)
    q_out.fill_(7.0)
    kc.fill_(9.0)
    C.chai_project_qk(dev(x), dev(w_q), dev(w_k), dev(rep), q_out, kc, pos0)
    torch.cuda.synchronize()
    q_ref, k_ref = O.project_qk(x, w_q, w_k, rep, d)
    x64 = np.abs(W.as_f64(x))
    aq, ak = np.abs(W.as_f64(w_q)).reshape(H, d, D), np.abs(W.as_f64(w_k)).reshape(H, d, D)
    qh, kh = W.torch_to_host_bits(q_out), W.torch_to_host_bits(kc)
    seven, nine = W.store(np.array([7.0], np.float32), W.BF16)[0], W.store(np.array([9.0], np.float32), W.BF16)[0]
    for b in range(B):
        used = set()
        for j in range(kk):
            r = int(rep[b, j])
            if r < 0:
                assert np.all(kh[b, j] == nine), "unused slot touched"
                continue
            used.add(r)
            check_rounded(qh[b, r], q_ref[b, j], np.einsum("te,ce->tc", x64[b], aq[r]), f"q b={b} j={j}")
            check_rounded(kh[b, j, pos0:pos0 + Tn], k_ref[b, j], np.einsum("te,ce->tc", x64[b], ak[r]), f"k b={b} j={j}")
            assert np.all(kh[b, j, :pos0] == nine) and np.all(kh[b, j, pos0 + Tn:] == nine), "rows outside the block touched"
        for h in range(H):
            if h not in used:
                assert np.all(qh[b, h] == seven), "query rows of a pruned head touched"
    assert G.guards_intact(q_whole, (B, H, Tn, d), 3.0) and G.guards_intact(k_whole, (B, kk, Tc_cap, d), 5.0)


@pytest.mark.parametrize("B,H,kk,Tn,D,pos0,Tc_cap", [
    (2, 8, 3, 300, 1024, 5, 320),      # two token tiles, the second ragged
    (1, 32, 8, 256, 4096, 0, 256),     # LLaMa-7B width, exactly one tile
    (3, 4, 4, 1, 512, 17, 32),         # decode step: one token per row
    (1, 6, 2, 513, 192, 0, 600),       # three tiles, short contraction
    (2, 72, 16, 37, 576, 100, 140),    # many heads, block in the middle of the cache
])
def test_projection_matches_oracle(B, H, kk, Tn, D, pos0, Tc_cap):
    run_case(B, H, kk, Tn, D, pos0, Tc_cap, seed=B * 5 + H * 3 + Tn, holes=True)


@pytest.mark.parametrize("name", ["cfg2", "cfg4"])
def test_projection_full_size_sampled(name):
    """The projection at the sizes bench.py --mode project times (all batch rows, positions 5..T-1, the model's
    width, the benchmark's 0.05-scaled weights).  The oracle computes sampled (batch row, slot, token block) pieces
    from the bytes downloaded from the device; what holds at any size: every written value is finite, pruned heads'
    query rows and the cache rows outside the block stay untouched."""
    cfg = W.CONFIGS[name]
    B, H, d, T = cfg.B, cfg.H, cfg.d, cfg.T
    D, kk = H * d, cfg.ks[-1]
    pos0, Tn = W.N_TOK, T - W.N_TOK
    print(f"[full-size projection] {name}: B={B} H={H} k={kk} tokens={Tn} width={D}", flush=True)
    g = W.rng(cfg.seed, 0, "member", extra=11)
    _, rep = W.random_membership(g, B, H, kk)
    seed = cfg.seed * 6007
    x = W.device_normal((B, Tn, D), cfg.dtype, seed + 1)
    w_q = (W.device_normal((H * d, D), cfg.dtype, seed + 2) * 0.05).to(torch.bfloat16)
    w_k = (W.device_normal((H * d, D), cfg.dtype, seed + 3) * 0.05).to(torch.bfloat16)
    q_out = torch.full((B, H, Tn, d), 7.0, dtype=torch.bfloat16, device="cuda")
    kc = torch.full((B, kk, T, d), 9.0, dtype=torch.bfloat16, device="cuda")
    C.chai_project_qk(x, w_q, w_k, W.host_to_torch(rep), q_out, kc, pos0)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(q_out.float()).all()) and bool(torch.isfinite(kc.float()).all())
    assert bool((kc[:, :, :pos0] == 9.0).all())
    for b in range(B):
        pruned = sorted(set(range(H)) - set(int(r) for r in rep[b] if r >= 0))
        if pruned:
            assert bool((q_out[b, pruned] == 7.0).all()), "query rows of a pruned head touched"
    gs = np.random.default_rng(cfg.seed + 17)
    rows = 8
    for s in range(8):
        b, j = int(gs.integers(B)), int(gs.integers(kk))
        r = int(rep[b, j])
        if r < 0:
            continue
        t0 = [0, 250, Tn - rows, int(gs.integers(Tn - rows))][s % 4]       # first tile, a tile edge, the ragged end
        xh = W.torch_to_host_bits(x[b:b + 1, t0:t0 + rows])
        wqh = W.torch_to_host_bits(w_q[r * d:(r + 1) * d])
        wkh = W.torch_to_host_bits(w_k[r * d:(r + 1) * d])
        q_ref, k_ref = O.project_qk(xh, wqh, wkh, np.zeros((1, 1), np.int32), d)      # one head: its own weights
        x64 = np.abs(W.as_f64(xh))[0]
        check_rounded(W.torch_to_host_bits(q_out[b, r, t0:t0 + rows]), q_ref[0, 0],
                      np.einsum("te,ce->tc", x64, np.abs(W.as_f64(wqh))), f"{name} q b={b} j={j} rows {t0}..")
        check_rounded(W.torch_to_host_bits(kc[b, j, pos0 + t0:pos0 + t0 + rows]), k_ref[0, 0],
                      np.einsum("te,ce->tc", x64, np.abs(W.as_f64(wkh))), f"{name} k b={b} j={j} rows {t0}..")


def test_projection_feeds_the_attention_kernels():
    """Projection -> clustered prefill attention, against the oracle fed with the oracle's projections rounded to
    bf16: the layouts the projection writes are the ones the attention kernels read."""
    B, H, kk, Tn, D, d = 1, 8, 3, 200, 512, 128
    g = np.random.default_rng(11)
    x = W.store(0.2 * g.standard_normal((B, Tn, D)).astype(np.float32), W.BF16)
    w_q = W.store(0.2 * g.standard_normal((H * d, D)).astype(np.float32), W.BF16)
    w_k = W.store(0.2 * g.standard_normal((H * d, D)).astype(np.float32), W.BF16)
    v = W.normal(g, (B, H, Tn, d), W.BF16)
    h2c, rep = W.random_membership(g, B, H, kk)
    q_out = torch.zeros((B, H, Tn, d), dtype=torch.bfloat16, device="cuda")
    kc = torch.zeros((B, kk, Tn, d), dtype=torch.bfloat16, device="cuda")
    C.chai_project_qk(dev(x), dev(w_q), dev(w_k), dev(rep), q_out, kc, 0)
    out = torch.empty((B, H, Tn, d), dtype=torch.float32, device="cuda")
    ws = torch.empty((C.chai_prefill_workspace_bytes(B, H, kk, Tn),), dtype=torch.uint8, device="cuda")
    scale = float(np.float32(d ** -0.5))
    C.chai_prefill_attention(q_out, kc, dev(v), dev(h2c), dev(rep), 0, scale, out, ws)
    torch.cuda.synchronize()
    # the oracle attends over full caches: place the device's (rounded) projections at the representatives' rows
    q_full = np.zeros((B, H, Tn, d), np.uint16)
    k_full = np.zeros((B, H, Tn, d), np.uint16)
    qh, kh = W.torch_to_host_bits(q_out), W.torch_to_host_bits(kc)
    for j in range(kk):
        q_full[0, rep[0, j]] = qh[0, rep[0, j]]
        k_full[0, rep[0, j]] = kh[0, j]
    ref = O.clustered_prefill(q_full, k_full, v, h2c, rep, 0, scale)
    ok, worst = G.rows_close(out.cpu().numpy(), ref, 2e-3)
    assert ok, worst


def test_projection_argument_errors():
    x = torch.zeros((1, 4, 128), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((2 * 128, 128), dtype=torch.bfloat16, device="cuda")
    rep = torch.zeros((1, 1), dtype=torch.int32, device="cuda")
    q = torch.full((1, 2, 4, 128), 7.0, dtype=torch.bfloat16, device="cuda")
    kc = torch.full((1, 1, 8, 128), 7.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(C.ChaiError) as e:
        C.chai_project_qk(x, w, w, rep, q, kc, 5)                   # block runs past the cache
    assert e.value.status == 2
    x96 = torch.zeros((1, 4, 96), dtype=torch.bfloat16, device="cuda")
    w96 = torch.zeros((2 * 128, 96), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(C.ChaiError) as e:
        C.chai_project_qk(x96, w96, w96, rep, q, kc, 0)             # contraction length not a multiple of 64
    assert e.value.status == 5
    with pytest.raises(C.ChaiError) as e:
        C.chai_project_qk(x.float(), w, w, rep, q, kc, 0)           # fp32 activations
    assert e.value.status == 5
    torch.cuda.synchronize()
    assert bool((q == 7.0).all()) and bool((kc == 7.0).all())


def test_mfma_rate_probe_runs_and_checks_arguments():
    data = torch.randn((1 << 16,), device="cuda").to(torch.bfloat16)
    sink = torch.full((1,), 7.0, dtype=torch.float32, device="cuda")
    flops = C.chai_mfma_rate_probe(data, 10, sink)
    torch.cuda.synchronize()
    assert flops == 512 * 8 * 10 * 8 * 2.0 * 32 * 32 * 16 and float(sink[0]) == 7.0
    with pytest.raises(C.ChaiError) as e:
        C.chai_mfma_rate_probe(data, 0, sink)
    assert e.value.status == 2
