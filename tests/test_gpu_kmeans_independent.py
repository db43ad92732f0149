"""chai_assign_clusters checked WITHOUT the CPU oracle: against scikit-learn's Lloyd iterations from the same
starting centres, against the optimum over all partitions on tiny planted inputs, against the hand-worked examples
of tests/golden/kmeans_worked.json, and against the fixed-point property of Lloyd's algorithm.  (Section 3.5:
membership by K-Means; Section 3.2: the clustering error is the sum of squared distances to the closest centre.)
The oracle is not imported here, so an error shared by the kernel and the oracle's transcription of the same rules
cannot hide."""
import itertools
import json
import os
import warnings

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

if not torch.cuda.is_available():
    pytest.skip("needs a GPU", allow_module_level=True)

import paper_2403_08058_amd as C
import workloads as W

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _gpu_kmeans(X, init, max_iter=50):
    """X [B,H,F] fp32, init [B,k] -> (head_to_cluster, rep_heads, n_clusters, iters) as numpy arrays."""
    feat = W.host_to_torch(np.ascontiguousarray(X, np.float32), "cuda")
    h2c, rep, n, it = C.chai_assign_clusters(feat, W.host_to_torch(np.ascontiguousarray(init, np.int32), "cuda"),
                                             max_iter=max_iter)
    torch.cuda.synchronize()
    return h2c.cpu().numpy(), rep.cpu().numpy(), n.cpu().numpy(), it.cpu().numpy()


def _canon(labels):
    seen, out = {}, []
    for a in labels:
        out.append(seen.setdefault(int(a), len(seen)))
    return np.asarray(out, np.int32)


def _sse(X, lab):
    X = X.astype(np.float64)
    return sum(((X[lab == j] - X[lab == j].mean(0)) ** 2).sum() for j in np.unique(lab))


def test_matches_sklearn_lloyd_from_the_same_start():
    from sklearn.cluster import KMeans
    checked = 0
    for seed in range(16):
        g = np.random.default_rng(7300 + seed)
        H, F, kk = [(32, 25, 8), (52, 25, 4), (72, 25, 16), (32, 5, 8)][seed % 4]
        X = g.random((H, F)).astype(np.float32)
        init = W.distinct_heads(g, 1, H, kk)
        print(f"[kmeans/sklearn] seed {seed} H={H} F={F} k={kk}", flush=True)
        h2c, rep, n, it = _gpu_kmeans(X[None], init, max_iter=100)
        with warnings.catch_warnings():
            warnings.simplefilter("ignore")
            km = KMeans(n_clusters=kk, init=X[init[0]].astype(np.float64), n_init=1, algorithm="lloyd", tol=0.0,
                        max_iter=100).fit(X.astype(np.float64))
        if len(np.unique(km.labels_)) < kk or int(n[0]) < kk:
            continue        # the library treats an empty centre differently: not comparable
        assert np.array_equal(h2c[0], _canon(km.labels_)), seed
        assert km.n_iter_ == int(it[0]), (seed, km.n_iter_, it)
        assert rep[0].tolist() == [int(np.nonzero(h2c[0] == j)[0][0]) for j in range(kk)]
        checked += 1
    assert checked >= 10


def test_reaches_the_brute_force_optimum_on_planted_tiny_inputs():
    for seed in range(5):
        g = np.random.default_rng(7200 + seed)
        H, F, kk = 9, 4, 3
        groups = W.planted_partition(g, 1, H, kk)
        cent = 10.0 * g.standard_normal((kk, F))
        X = (cent[groups[0]] + 0.05 * g.standard_normal((H, F))).astype(np.float32)
        best_lab = min(itertools.product(range(kk), repeat=H), key=lambda lab: _sse(X, np.asarray(lab)))
        init = W.one_head_per_group(g, groups, kk)
        print(f"[kmeans/brute] planted seed {seed}", flush=True)
        h2c, rep, n, it = _gpu_kmeans(X[None], init)
        assert np.array_equal(h2c[0], _canon(best_lab)) and np.array_equal(h2c[0], _canon(groups[0]))
        assert int(n[0]) == kk
    # unstructured tiny inputs: Lloyd never beats the optimum, and its partition is a fixed point
    for seed in range(6):
        g = np.random.default_rng(7100 + seed)
        H, F, kk = 8, 3, 3
        X = g.standard_normal((H, F)).astype(np.float32)
        best = min(_sse(X, np.asarray(lab)) for lab in itertools.product(range(kk), repeat=H))
        init = W.distinct_heads(g, 1, H, kk)
        print(f"[kmeans/brute] random seed {seed}", flush=True)
        h2c, rep, n, it = _gpu_kmeans(X[None], init)
        assert _sse(X, h2c[0]) >= best - 1e-10
        means = np.stack([X[h2c[0] == j].astype(np.float64).mean(0) for j in range(int(n[0]))])
        dist = ((X[:, None, :].astype(np.float64) - means[None]) ** 2).sum(-1)
        assert np.array_equal(np.argmin(dist, 1), h2c[0])


def test_hand_worked_examples():
    """Every case of the golden file (worked by hand under the completion rules, the repair-donor cases included)."""
    with open(os.path.join(GOLDEN, "kmeans_worked.json")) as f:
        cases = json.load(f)["cases"]
    for case in cases:
        X = np.asarray(case["feat"], np.float32)[None]
        init = np.asarray(case["init_heads"], np.int32)[None]
        print(f"[kmeans/golden] {case['name']}", flush=True)
        h2c, rep, n, it = _gpu_kmeans(X, init)
        assert h2c[0].tolist() == case["head_to_cluster"], case["name"]
        assert rep[0].tolist() == case["rep_heads"], case["name"]
        assert int(n[0]) == case["n_clusters"] and int(it[0]) == case["iters"], case["name"]
        assert abs(_sse(X[0], h2c[0]) - case["sse"]) < 1e-9, case["name"]


def test_clustering_error_never_rises_and_rows_are_independent():
    g = np.random.default_rng(7400)
    B, H, F, kk = 4, 72, 25, 16
    X = g.random((B, H, F)).astype(np.float32)
    init = W.distinct_heads(g, B, H, kk)
    full, _, _, it = _gpu_kmeans(X, init)
    prev = None
    for m in range(1, int(it.max()) + 1):
        h, _, _, its = _gpu_kmeans(X, init, max_iter=m)
        assert np.all(its == np.minimum(it, m))
        s = np.array([_sse(X[b], h[b]) for b in range(B)])
        if prev is not None:
            assert np.all(s <= prev + 1e-9)
        prev = s
    assert np.array_equal(h, full)
    one, _, _, _ = _gpu_kmeans(X[2:3], init[2:3])
    assert np.array_equal(one[0], full[2])
