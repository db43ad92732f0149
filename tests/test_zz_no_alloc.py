"""chai_decode_attention_static (the entry point for callers that cannot allocate: scratch is a fixed array inside
the library) against chai_decode_attention with a caller-provided workspace, through the C ABI, on two calls in a
row of which the second is smaller (stale contents of the first call's scratch must not matter), plus the size
limit.  Both entry points run the same kernels, so the results are compared bit for bit."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

if not torch.cuda.is_available():
    pytest.skip("needs a GPU", allow_module_level=True)

import paper_2403_08058_amd as C
import workloads as W

from gpu_util import dev, guarded, guards_intact


def _case(seed, B, H, k, T, T_cap, dtype):
    g = W.rng(seed, 0, "member")
    h2c, rep = W.random_membership(g, B, H, k)
    q = W.normal(W.rng(seed, 0, "q"), (B, H, 128), dtype)
    kc = W.normal(W.rng(seed, 0, "k"), (B, k, T_cap, 128), dtype)
    v = W.normal(W.rng(seed, 0, "v"), (B, H, T_cap, 128), dtype)
    return dev(q), dev(kc), dev(v), dev(h2c), dev(rep)


def _raw_static(q, kc, v, h2c, rep, T, scale, out, probs):
    """The raw C ABI call: plain pointers and sizes, no workspace argument."""
    B, H, d = q.shape
    k, Tc_cap, T_cap = kc.shape[1], kc.shape[2], v.shape[2]
    return C.lib().chai_decode_attention_static(
        ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(kc.data_ptr()), ctypes.c_void_p(v.data_ptr()),
        ctypes.c_void_p(h2c.data_ptr()), ctypes.c_void_p(rep.data_ptr()), B, H, k, T, Tc_cap, T_cap, d,
        C.binding.dtype_code(q), ctypes.c_float(scale), ctypes.c_void_p(out.data_ptr()),
        ctypes.c_void_p(probs.data_ptr()) if probs is not None else None,
        ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))


@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
def test_static_scratch_matches_workspace_call_twice_in_a_row(dtype):
    scale = 1.0 / np.sqrt(128.0)
    # first a call with split heads (partial rows + combine), then a smaller one of another chunking
    shapes = [(3, 32, 8, 2500, 2560), (2, 20, 5, 333, 384)]
    for i, (B, H, k, T, T_cap) in enumerate(shapes):
        print(f"[no-alloc] call {i}: B={B} H={H} k={k} T={T} dtype={dtype}", flush=True)
        q, kc, v, h2c, rep = _case(4100 + i, B, H, k, T, T_cap, dtype)
        ws = C.alloc_workspace(B, H, k, T, 128, dtype)
        ws.fill_(0xFF)
        ref = torch.empty((B, H, 128), dtype=torch.float32, device="cuda")
        ref_p = torch.empty((B, k, T), dtype=torch.float32, device="cuda")
        C.chai_decode_attention(q, kc, v, h2c, rep, T, scale, ref, ws, probs_out=ref_p)
        whole, out = guarded((B, H, 128), torch.float32, float("nan"))
        probs = torch.empty((B, k, T), dtype=torch.float32, device="cuda")
        free_before = torch.cuda.mem_get_info()[0]
        st = _raw_static(q, kc, v, h2c, rep, T, scale, out, probs)
        assert st == C.CHAI_OK, C.chai_status_string(st)
        torch.cuda.synchronize()
        if i > 0:       # the first call on a device may load the code object; later calls must not move memory
            assert torch.cuda.mem_get_info()[0] == free_before
        assert torch.equal(out, ref), float((out - ref).abs().max())
        assert torch.equal(probs, ref_p)
        assert guards_intact(whole, (B, H, 128), float("nan"))
        assert bool(torch.isfinite(out).all())


def test_static_scratch_refuses_sizes_beyond_its_limit_and_bad_arguments():
    B, H, k, T = 2, 32, 8, 64
    q, kc, v, h2c, rep = _case(4200, B, H, k, T, T, W.BF16)
    out = torch.zeros((B, H, 128), dtype=torch.float32, device="cuda")
    # a size whose workspace exceeds the built-in array: refused on the host, nothing launched, out untouched
    big_B, big_T = 64, 1 << 16
    assert C.chai_decode_workspace_bytes(big_B, H, k, big_T, 128, W.BF16) > C.binding.CHAI_STATIC_SCRATCH_BYTES
    st = C.lib().chai_decode_attention_static(
        ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(kc.data_ptr()), ctypes.c_void_p(v.data_ptr()),
        ctypes.c_void_p(h2c.data_ptr()), ctypes.c_void_p(rep.data_ptr()), big_B, H, k, big_T, big_T, big_T, 128,
        W.BF16, ctypes.c_float(1.0), ctypes.c_void_p(out.data_ptr()), None, None)
    assert st == 8 and "static" in C.chai_status_string(st)
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
    # ordinary argument errors are answered as by chai_decode_attention
    st = C.lib().chai_decode_attention_static(None, ctypes.c_void_p(kc.data_ptr()), ctypes.c_void_p(v.data_ptr()),
                                              ctypes.c_void_p(h2c.data_ptr()), ctypes.c_void_p(rep.data_ptr()), B, H, k, T,
                                              T, T, 128, W.BF16, ctypes.c_float(1.0), ctypes.c_void_p(out.data_ptr()),
                                              None, None)
    assert st == 1
    st = C.lib().chai_decode_attention_static(ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(kc.data_ptr()),
                                              ctypes.c_void_p(v.data_ptr()), ctypes.c_void_p(h2c.data_ptr()),
                                              ctypes.c_void_p(rep.data_ptr()), B, H, k, T + 1, T, T, 128, W.BF16,
                                              ctypes.c_float(1.0), ctypes.c_void_p(out.data_ptr()), None, None)
    assert st == 2
