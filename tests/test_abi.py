"""The C-ABI library loads without a GPU, exports every symbol include/chai.h declares, and its host-side
argument checks answer before anything touches the device (no compute call is made here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INCLUDE = os.path.join(ROOT, "include")


@pytest.fixture(scope="module")
def chai():
    import paper_2403_08058_amd as C
    return C


def declared_functions():
    names = set()
    for header in sorted(os.listdir(INCLUDE)):
        if header.endswith(".h"):
            text = open(os.path.join(INCLUDE, header)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(chai_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_header_symbols_exported(chai):
    names = declared_functions()
    assert len(names) >= 28 and "chai_decode_attention_static" in names and "chai_assign_clusters" in names and "chai_compact_kcache" in names \
        and "chai_decode_attention" in names
    L = ctypes.CDLL(chai.LIB_PATH)
    for n in names:
        assert hasattr(L, n), f"{n} declared in chai.h but not exported"
    # the Python binding carries the same names
    assert sorted(chai.EXPORTS) == names
    for n in names:
        assert callable(getattr(chai, n))


def test_status_strings_and_version(chai):
    assert chai.chai_version() >= 100
    seen = {chai.chai_status_string(s) for s in range(9)}
    assert len(seen) == 9 and chai.chai_status_string(0) == "ok"
    assert chai.chai_status_string(99) == "unknown status"


def test_workspace_query_is_host_only(chai):
    q = chai.chai_decode_workspace_bytes
    assert q(16, 32, 8, 2048, 128, chai.CHAI_BF16) > 16 * 8 * 2048 * 4
    assert q(16, 32, 8, 2048, 64, chai.CHAI_BF16) == 0          # unsupported head dim
    assert q(16, 32, 33, 2048, 128, chai.CHAI_BF16) == 0        # k > H
    assert q(16, 32, 8, 0, 128, chai.CHAI_BF16) == 0            # nothing to attend to
    assert q(16, 32, 8, 2048, 128, 5) == 0
    assert q(4, 32, 4, 32768, 128, 1) % 256 == 0
    # monotone in T: a workspace sized for the capacity serves every shorter context
    sizes = [q(4, 72, 16, T, 128, 1) for T in (1, 100, 513, 1024, 2048)]
    assert sizes == sorted(sizes)


def test_argument_checks_run_before_any_launch(chai):
    """Invalid calls return their error code on a machine without a GPU: the checks precede every HIP call."""
    L = chai.lib()
    fake = 0x1000            # a non-NULL, 16-byte aligned address that is never dereferenced on the host
    assert L.chai_decode_attention(None, fake, fake, fake, fake, 1, 32, 8, 64, 64, 64, 128, 1, 0.1, fake, None, fake,
                                   1 << 30, None) == 1
    assert L.chai_decode_attention(fake, fake, fake, fake, fake, 1, 32, 8, 65, 64, 64, 128, 1, 0.1, fake, None, fake,
                                   1 << 30, None) == 2
    assert L.chai_decode_attention(fake, fake, fake, fake, fake, 1, 32, 8, 64, 64, 64, 128, 2, 0.1, fake, None, fake,
                                   1 << 30, None) == 3
    assert L.chai_decode_attention(fake, fake, fake, fake, fake, 1, 32, 8, 64, 64, 64, 128, 1, 0.1, fake, None, fake,
                                   16, None) == 4
    assert L.chai_decode_attention(fake, fake, fake, fake, fake, 1, 32, 8, 64, 64, 64, 96, 1, 0.1, fake, None, fake,
                                   1 << 30, None) == 5
    assert L.chai_decode_attention(fake + 2, fake, fake, fake, fake, 1, 32, 8, 64, 64, 64, 128, 1, 0.1, fake, None,
                                   fake, 1 << 30, None) == 7
    assert L.chai_dense_decode_attention(fake, fake, None, 1, 32, 64, 64, 128, 1, 0.1, fake, fake, 1 << 30, None) == 1
    assert L.chai_compact_kcache(fake, fake, fake, 1, 32, 8, 65, 64, 128, 128, 1, None) == 2
    assert L.chai_compact_kcache(fake, fake, fake, 1, 32, 8, 0, 64, 128, 128, 1, None) == 0      # T = 0: no-op
    assert L.chai_append_kv(fake, fake, fake, fake, fake, 1, 32, 8, 64, 64, 64, 128, 1, None) == 2
    assert L.chai_assign_clusters(fake, 1, 32, 25, 33, fake, 50, fake, fake, fake, None, None) == 2
    assert L.chai_assign_clusters(fake, 1, 300, 25, 8, fake, 50, fake, fake, fake, None, None) == 5
    assert L.chai_assign_clusters(fake, 0, 32, 25, 8, fake, 50, fake, fake, fake, None, None) == 0  # B = 0: no-op
    assert L.chai_score_features(fake, fake, 1, 32, 9, 128, 1, 9 * 128, 9 * 128, 0.1, fake, None) == 5
    assert L.chai_score_features(fake, fake, 1, 32, 5, 128, 1, 4 * 128, 5 * 128, 0.1, fake, None) == 2
    # prefill: positions [q_start, q_start + Tq) of a bf16 cache; scale must be positive
    big = 1 << 34
    pf = lambda **kw: L.chai_prefill_attention(*[kw.get(n, dflt) for n, dflt in (
        ("q", fake), ("kc", fake), ("v", fake), ("h2c", fake), ("rep", fake), ("B", 1), ("H", 32), ("k", 8), ("Tq", 64),
        ("q_start", 0), ("Tc_cap", 64), ("T_cap", 64), ("d", 128), ("dtype", 1), ("scale", 0.1), ("out", fake),
        ("ws", 0x1000), ("ws_bytes", big), ("stream", None))])
    assert pf(h2c=None) == 1
    assert pf(Tq=65) == 2                       # runs past the cache
    assert pf(q_start=1) == 2
    assert pf(dtype=2) == 3
    assert pf(ws_bytes=16) == 4
    assert pf(dtype=0) == 5                     # fp32 prefill is not built
    assert pf(scale=0.0) == 5 and pf(scale=-0.1) == 5 and pf(scale=float("nan")) == 5
    assert pf(q=fake + 2) == 7
    assert pf(B=0) == 0                         # empty batch: no-op
    assert pf(Tq=1 << 23, Tc_cap=1 << 23, T_cap=1 << 23, ws_bytes=1 << 60) == 5     # beyond 32-bit key offsets
    assert L.chai_dense_prefill_attention(fake, fake, fake, 1, 32, 64, 0, 64, 128, 1, -1.0, fake, 0x1000, big, None) == 5
    # projections of the representatives: x [B,Tn,D], weights [H*d, D]
    pj = lambda **kw: L.chai_project_qk(*[kw.get(n, dflt) for n, dflt in (
        ("x", fake), ("w_q", fake), ("w_k", fake), ("rep", fake), ("B", 1), ("H", 32), ("k", 8), ("Tn", 16), ("D", 4096),
        ("d", 128), ("dtype", 1), ("q_out", fake), ("kc", fake), ("pos0", 0), ("Tc_cap", 64), ("stream", None))])
    assert pj(w_k=None) == 1
    assert pj(pos0=60) == 2                     # block runs past the compact cache
    assert pj(dtype=7) == 3
    assert pj(dtype=0) == 5 and pj(D=4000) == 5 and pj(d=64) == 5
    assert pj(x=fake + 8) == 7
    assert pj(B=0) == 0
    assert chai.chai_prefill_workspace_bytes(4, 32, 8, 100) == chai.chai_prefill_workspace_bytes(4, 32, 8, 128)
    assert chai.chai_prefill_workspace_bytes(4, 32, 8, 129) > chai.chai_prefill_workspace_bytes(4, 32, 8, 128)


def test_pick_cluster_count_runs_on_the_host(chai):
    """The plateau rule is host code with host pointers: checked here against the hand-worked cases."""
    import json
    cases = json.load(open(os.path.join(ROOT, "tests", "golden", "cluster_count_worked.json")))["pick_cases"]
    for c in cases:
        assert chai.chai_pick_cluster_count(c["err"], c["ks"], c["tol"]) == c["k"], c["how"]
    with pytest.raises(chai.ChaiError):
        chai.chai_pick_cluster_count([3.0, 2.0], [4, 4], 0.1)        # ks not ascending
    with pytest.raises(chai.ChaiError):
        chai.chai_pick_cluster_count([3.0, 2.0], [2, 4], -1.0)


def test_product_does_not_import_the_oracle():
    """The product package never reaches into oracle/ (and the oracle never into the product)."""
    pkg = os.path.join(ROOT, "paper_2403_08058_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2403_08058_amd" not in text and "libchai.so" not in text


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: bench.py --gpus N with N > 1 exits with a message before touching any device."""
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode == 2 and "ONE GPU" in res.stderr and res.stdout.strip() == ""
