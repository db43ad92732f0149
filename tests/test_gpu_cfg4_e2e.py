"""The OPT-66B-shaped configuration as it is stated: 512-token prompt -> score features of the first five positions
-> k-means (k = 16) -> K-cache compaction -> 128 decode steps with cache growth (chai_decode_step), per layer at the
full width (72 heads, batch 4, capacity 2048), through the same code path bench.py times (`bench.e2e_bench`), on
a few layers.  Parity inside that flow: oracle on sampled (batch row, head) pairs at steps 1, 64 and 128 from the
FULL prompt key cache plus the appended rows; grown caches byte-equal to chai_append_kv's; both for the pass that
starts at the prompt and the pass that ends at the cache capacity."""
import argparse
import dataclasses

import pytest
import torch

pytestmark = pytest.mark.gpu

if not torch.cuda.is_available():
    pytest.skip("needs a GPU", allow_module_level=True)

import bench
import paper_2403_08058_amd as C
import workloads as W


def test_cfg4_flow_as_stated_on_three_layers():
    cfg = dataclasses.replace(W.CONFIGS["cfg4"], L=3, ks=(16,) * 3)
    assert cfg.prompt == 512 and cfg.decode_steps == 128 and cfg.T_cap == 2048 and cfg.H == 72 and cfg.B == 4
    print("[cfg4 e2e] 3 layers x 128 steps, two passes", flush=True)
    rec = bench.e2e_bench(cfg, argparse.Namespace(), torch, C, W, steps_timed=1)
    for name, first in (("from_prompt", 513), ("to_capacity", 1921)):
        r = rec[name]
        assert r["contexts"] == [first, first + 127] and r["decode_steps"] == 128
        assert r["parity"]["grown_caches_equal_chai_append_kv"] is True
        assert r["parity"]["at_steps"] == [1, 64, 128] and r["parity"]["sampled_heads"] >= 27
        assert r["parity"]["worst_normwise_err"] <= 2e-5
        assert r["tokens_per_s"] > 0
    assert rec["membership_and_compaction_ms"] > 0
