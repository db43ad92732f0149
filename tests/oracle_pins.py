"""Pins of the CPU oracle: checks against what the paper and the mathematics fix.

Every function here takes no arguments, calls ``oracle.chai_oracle`` and raises AssertionError when the oracle
disagrees with a value it did not produce itself: a hand-worked example (tests/golden), a library routine
(scipy softmax + numpy contraction, scikit-learn Lloyd, numpy gathers, torch's bf16 cast), a closed form, an
invariant of the definition, or brute force over all partitions.  ``test_oracle_pins.py`` runs them against
the oracle as committed, and ``test_oracle_mutants.py`` runs them against deliberately broken copies of the C
file to show that each planted mistake is caught by at least one pin.
"""
from __future__ import annotations

import itertools
import json
import math
import os

import numpy as np
import scipy.special

import workloads as W
from oracle import chai_oracle as O

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _golden(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return json.load(f)


def _ln(a):
    return np.log(np.asarray(a, np.float64)).astype(np.float32)


# ----------------------------------------------------------------------------------------------
# library re-statement used as an independent pin: scipy softmax + numpy einsum in fp64
# ----------------------------------------------------------------------------------------------
def lib_dense(q, k, v, T, scale):
    q64, k64, v64 = W.as_f64(q), W.as_f64(k)[:, :, :T], W.as_f64(v)[:, :, :T]
    s = scale * np.einsum("bhd,bhtd->bht", q64, k64)
    p = scipy.special.softmax(s, axis=-1)
    return np.einsum("bht,bhtd->bhd", p, v64), p


def lib_clustered(q, k, v, h2c, rep, T, scale):
    B, H, d = q.shape
    _, p_dense = lib_dense(q, k, v, T, scale)
    v64 = W.as_f64(v)[:, :, :T]
    out = np.empty((B, H, d))
    for b in range(B):
        for h in range(H):
            out[b, h] = p_dense[b, rep[b, h2c[b, h]]] @ v64[b, h]
    return out


def _rand_case(seed, B, H, T, T_cap, d, dtype):
    g = np.random.default_rng(seed)
    q = W.normal(g, (B, H, d), dtype)
    k = W.normal(g, (B, H, T_cap, d), dtype)
    v = W.normal(g, (B, H, T_cap, d), dtype)
    return q, k, v


# ----------------------------------------------------------------------------------------------
# attention pins
# ----------------------------------------------------------------------------------------------
def pin_bf16_bits():
    import torch
    x = np.random.default_rng(1).standard_normal(4096).astype(np.float32)
    x[:6] = [1.0, -2.0, 0.0, 1.00390625, 1.01171875, 3.0e38]   # 1+2^-8 is a tie -> even (1.0); 1+3*2^-8 ties up
    bits = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    assert bits[0] == 0x3F80 and bits[1] == 0xC000 and bits[3] == 0x3F80 and bits[4] == 0x3F82
    # the oracle widens exactly: a one-token attention returns V unchanged
    v = W.f32_to_bf16_bits(x[:128]).reshape(1, 1, 1, 128)
    out = O.dense_decode(v[:, :, 0], v, v, 1, 1.0)
    assert np.array_equal(out[0, 0], W.bf16_bits_to_f32(v[0, 0, 0]).astype(np.float64))


def pin_attention_worked_example():
    gd = _golden("attention_worked.json")
    q = np.asarray(gd["q"], np.float32)
    k = _ln(gd["k_ln"])
    v = np.asarray(gd["v"], np.float32)
    out, p = O.dense_decode(q, k, v, 2, gd["scale"], want_probs=True)
    assert np.allclose(p, gd["dense_probs"], rtol=0, atol=1e-7)
    assert np.allclose(out, gd["dense_out"], rtol=0, atol=1e-6)
    h2c = np.asarray(gd["clustered_head_to_cluster"], np.int32)
    rep = np.asarray(gd["clustered_rep_heads"], np.int32)
    outc, pc = O.clustered_decode(q, k, v, h2c, rep, 2, gd["scale"], want_probs=True)
    assert np.allclose(outc, gd["clustered_out"], rtol=0, atol=1e-6)
    assert np.allclose(pc[0, 0], gd["dense_probs"][0][0], rtol=0, atol=1e-7)


def pin_dense_matches_library():
    for seed, (B, H, T, T_cap, d, dt) in enumerate([(2, 3, 17, 17, 8, W.F32), (1, 4, 33, 40, 128, W.BF16),
                                                    (2, 2, 1, 5, 16, W.F32)]):
        q, k, v = _rand_case(seed, B, H, T, T_cap, d, dt)
        if T_cap > T:   # rows past T must never be read
            if dt == W.F32:
                k[:, :, T:], v[:, :, T:] = np.nan, np.nan
            else:
                k[:, :, T:], v[:, :, T:] = 0x7FC0, 0x7FC0
        scale = float(np.float32(1.0 / math.sqrt(d)))
        out, p = O.dense_decode(q, k, v, T, scale, want_probs=True)
        ref, pref = lib_dense(q, k, v, T, scale)
        assert np.allclose(p, pref, rtol=1e-12, atol=1e-15)
        assert np.allclose(out, ref, rtol=1e-12, atol=1e-13)
        # the scale really multiplies the scores
        out2 = O.dense_decode(q, k, v, T, 0.375)
        assert np.allclose(out2, lib_dense(q, k, v, T, 0.375)[0], rtol=1e-12, atol=1e-13)


def pin_dense_closed_forms():
    g = np.random.default_rng(7)
    B, H, T, d = 1, 2, 9, 16
    q = W.normal(g, (B, H, d), W.F32)
    v = W.normal(g, (B, H, T, d), W.F32)
    # equal keys -> uniform probabilities -> mean of the value rows
    k = np.broadcast_to(W.normal(g, (B, H, 1, d), W.F32), (B, H, T, d)).copy()
    out, p = O.dense_decode(q, k, v, T, 0.25, want_probs=True)
    assert np.allclose(p, 1.0 / T, rtol=0, atol=1e-15)
    assert np.allclose(out, v.astype(np.float64).mean(axis=2), rtol=0, atol=1e-14)
    # one key aligned with q and huge -> that token's value row
    k = np.zeros((B, H, T, d), np.float32)
    k[:, :, 4] = 1000.0 * q
    out = O.dense_decode(q, k, v, T, 1.0)
    assert np.allclose(out, v[:, :, 4].astype(np.float64), rtol=0, atol=1e-12)
    assert np.all(np.isfinite(out))
    # one cached token -> its value row exactly
    out = O.dense_decode(q, k, v, 1, 1.0)
    assert np.array_equal(out, v[:, :, 0].astype(np.float64))


def pin_softmax_properties():
    q, k, v = _rand_case(11, 2, 4, 50, 50, 32, W.F32)
    scale = float(np.float32(1.0 / math.sqrt(32)))
    _, p = O.dense_decode(q, k, v, 50, scale, want_probs=True)
    assert np.all(p >= 0) and np.allclose(p.sum(-1), 1.0, rtol=0, atol=1e-14)
    # adding one vector u to every key shifts all scores of a head by the same constant
    u = W.normal(np.random.default_rng(3), (1, 1, 1, 32), W.F32)
    _, p2 = O.dense_decode(q, (k.astype(np.float64) + u).astype(np.float32), v, 50, scale, want_probs=True)
    assert np.allclose(p, p2, rtol=0, atol=2e-6)
    # very large scores of both signs stay finite and normalised
    _, p3 = O.dense_decode(q, k, v, 50, 80.0, want_probs=True)
    assert np.all(np.isfinite(p3)) and np.allclose(p3.sum(-1), 1.0, rtol=0, atol=1e-14)
    # probabilities order like the scores
    s = 80.0 * np.einsum("bhd,bhtd->bht", q.astype(np.float64), k.astype(np.float64))
    assert np.array_equal(np.argmax(s, -1), np.argmax(p3, -1))


def pin_clustered_reduces_to_dense():
    for seed, dt in [(21, W.F32), (22, W.BF16)]:
        B, H, T, T_cap, d = 2, 6, 23, 29, 64
        q, k, v = _rand_case(seed, B, H, T, T_cap, d, dt)
        scale = float(np.float32(1.0 / math.sqrt(d)))
        dense = O.dense_decode(q, k, v, T, scale)
        # one head per cluster (any labelling) is dense attention
        g = np.random.default_rng(seed)
        perm = np.stack([g.permutation(H) for _ in range(B)]).astype(np.int32)      # head -> cluster label
        rep = np.empty_like(perm)
        for b in range(B):
            rep[b, perm[b]] = np.arange(H)
        out = O.clustered_decode(q, k, v, perm, rep, T, scale)
        assert np.array_equal(out, dense)


def pin_clustered_matches_library():
    for seed, dt in [(31, W.F32), (32, W.BF16)]:
        B, H, T, T_cap, d, kk = 2, 7, 19, 19, 32, 3
        q, k, v = _rand_case(seed, B, H, T, T_cap, d, dt)
        h2c, rep = W.random_membership(np.random.default_rng(seed), B, H, kk)
        scale = float(np.float32(1.0 / math.sqrt(d)))
        out, p = O.clustered_decode(q, k, v, h2c, rep, T, scale, want_probs=True)
        ref = lib_clustered(q, k, v, h2c, rep, T, scale)
        assert np.allclose(out, ref, rtol=1e-12, atol=1e-13)
        _, pd = lib_dense(q, k, v, T, scale)
        for b in range(B):
            for j in range(kk):
                assert np.allclose(p[b, j], pd[b, rep[b, j]], rtol=1e-12, atol=1e-15)


def pin_clustered_identical_qk_is_exact():
    # members with identical Q and K: the clustered result is dense attention for every head, whatever V is,
    # and whichever member is taken as representative
    B, H, T, d, kk = 2, 8, 31, 32, 3
    g = np.random.default_rng(41)
    h2c, rep = W.random_membership(g, B, H, kk)
    qc = W.normal(g, (B, kk, d), W.F32)
    kc = W.normal(g, (B, kk, T, d), W.F32)
    q = np.stack([qc[b, h2c[b]] for b in range(B)])
    k = np.stack([kc[b, h2c[b]] for b in range(B)])
    v = W.normal(g, (B, H, T, d), W.F32)
    scale = float(np.float32(1.0 / math.sqrt(d)))
    dense = O.dense_decode(q, k, v, T, scale)
    out, p = O.clustered_decode(q, k, v, h2c, rep, T, scale, want_probs=True)
    assert np.array_equal(out, dense)
    # another representative (the highest member instead of the lowest)
    rep_hi = np.full_like(rep, -1)
    for b in range(B):
        for h in range(H):
            rep_hi[b, h2c[b, h]] = h
    assert np.array_equal(O.clustered_decode(q, k, v, h2c, rep_hi, T, scale), dense)
    # members share the probability row but not the output: values are never shared
    for b in range(B):
        for j in range(kk):
            members = np.nonzero(h2c[b] == j)[0]
            if len(members) >= 2:
                a, c = members[:2]
                assert not np.allclose(out[b, a], out[b, c])
                assert np.allclose(out[b, a], p[b, j] @ v[b, a].astype(np.float64), rtol=1e-12, atol=1e-13)
                assert np.allclose(out[b, c], p[b, j] @ v[b, c].astype(np.float64), rtol=1e-12, atol=1e-13)


def pin_clustered_ignores_pruned_qk():
    # queries and keys of non-representative heads are pruned: poisoning them changes nothing
    B, H, T, d, kk = 1, 9, 13, 16, 4
    q, k, v = _rand_case(51, B, H, T, T, d, W.F32)
    h2c, rep = W.random_membership(np.random.default_rng(51), B, H, kk)
    out = O.clustered_decode(q, k, v, h2c, rep, T, 0.25)
    q2, k2 = q.copy(), k.copy()
    for h in range(H):
        if h not in rep[0]:
            q2[0, h], k2[0, h] = np.nan, np.nan
    assert np.array_equal(O.clustered_decode(q2, k2, v, h2c, rep, T, 0.25), out)
    # permuting the heads (with their maps) permutes the outputs
    perm = np.random.default_rng(52).permutation(H)
    inv = np.argsort(perm)
    rep_p = inv[rep].astype(np.int32)
    out_p = O.clustered_decode(q[:, perm], k[:, perm], v[:, perm], h2c[:, perm], rep_p, T, 0.25)
    assert np.allclose(out_p, out[:, perm], rtol=1e-13, atol=1e-14)


def pin_shared_v_takes_the_whole_representative():
    # the ablation that prunes values too: every head's output is the dense attention output of its
    # representative (library re-statement), whatever the pruned heads hold in Q, K and V
    for seed, dt in [(61, W.F32), (62, W.BF16)]:
        B, H, T, T_cap, d, kk = 2, 9, 21, 25, 32, 4
        q, k, v = _rand_case(seed, B, H, T, T_cap, d, dt)
        h2c, rep = W.random_membership(np.random.default_rng(seed), B, H, kk)
        scale = float(np.float32(1.0 / math.sqrt(d)))
        out = O.shared_v_decode(q, k, v, h2c, rep, T, scale)
        ref, _ = lib_dense(q, k, v, T, scale)
        for b in range(B):
            for h in range(H):
                assert np.allclose(out[b, h], ref[b, rep[b, h2c[b, h]]], rtol=1e-12, atol=1e-13)
        own = O.clustered_decode(q, k, v, h2c, rep, T, scale)
        for b in range(B):
            for h in range(H):
                same = np.allclose(out[b, h], own[b, h], rtol=1e-9, atol=1e-12)
                assert same == (h in rep[b]), "only representatives agree with the variant that keeps every V"
        q2, k2, v2 = q.copy(), k.copy(), v.copy()
        for b in range(B):
            for h in range(H):
                if h not in rep[b]:
                    for a in (q2, k2, v2):
                        a[b, h] = 0x7FC0 if dt == W.BF16 else np.nan
        assert np.array_equal(O.shared_v_decode(q2, k2, v2, h2c, rep, T, scale), out)


def pin_closest_representatives():
    for c in _golden("representative_worked.json")["cases"]:
        X = np.asarray(c["feat"], np.float32)[None]
        lab = np.asarray(c["labels"], np.int32)[None]
        assert O.closest_representatives(X, lab, c["k"])[0].tolist() == c["rep"], c["how"]
    # numpy re-statement on random partitions (distinct distances with probability 1)
    g = np.random.default_rng(801)
    B, H, F, kk = 5, 24, 25, 7
    X = g.random((B, H, F)).astype(np.float32)
    lab = g.integers(0, kk, size=(B, H)).astype(np.int32)
    lab[0][lab[0] == 3] = 2                                    # an empty slot
    rep = O.closest_representatives(X, lab, kk)
    for b in range(B):
        for j in range(kk):
            members = np.nonzero(lab[b] == j)[0]
            if len(members) == 0:
                assert rep[b, j] == -1
                continue
            pts = X[b, members].astype(np.float64)
            dist = ((pts - pts.mean(axis=0)) ** 2).sum(axis=1)
            assert rep[b, j] == members[np.argmin(dist)]
    # one head per cluster: every head represents itself; identical members: the lowest one
    assert np.array_equal(O.closest_representatives(X, np.tile(np.arange(H, dtype=np.int32), (B, 1)), H),
                          np.tile(np.arange(H, dtype=np.int32), (B, 1)))
    same = np.repeat(X[:, :1], H, axis=1)
    assert np.all(O.closest_representatives(same, np.zeros((B, H), np.int32), 1) == 0)


def pin_prefill_matches_library_and_decode():
    for seed, dt in [(71, W.F32), (72, W.BF16)]:
        B, H, Tq, q_start, T_cap, d, kk = 2, 6, 9, 5, 16, 32, 3
        g = np.random.default_rng(seed)
        q = W.normal(g, (B, H, Tq, d), dt)
        k = W.normal(g, (B, H, T_cap, d), dt)
        v = W.normal(g, (B, H, T_cap, d), dt)
        nan = np.nan if dt == W.F32 else 0x7FC0
        k[:, :, q_start + Tq:], v[:, :, q_start + Tq:] = nan, nan           # never read
        h2c, rep = W.random_membership(g, B, H, kk)
        scale = float(np.float32(1.0 / math.sqrt(d)))
        out = O.clustered_prefill(q, k, v, h2c, rep, q_start, scale)
        # library statement: causal mask + scipy softmax + einsum, probabilities of the representative
        T = q_start + Tq
        s = scale * np.einsum("bhid,bhtd->bhit", W.as_f64(q), W.as_f64(k)[:, :, :T])
        mask = np.arange(T)[None, :] <= (q_start + np.arange(Tq))[:, None]
        p = scipy.special.softmax(np.where(mask, s, -np.inf), axis=-1)
        ref = np.empty_like(out)
        for b in range(B):
            for h in range(H):
                ref[b, h] = p[b, rep[b, h2c[b, h]]] @ W.as_f64(v)[b, h, :T]
        assert np.allclose(out, ref, rtol=1e-12, atol=1e-13)
        # row i of the block is the decode step at context q_start + i + 1
        for i in (0, 4, Tq - 1):
            dec = O.clustered_decode(np.ascontiguousarray(q[:, :, i]), k, v, h2c, rep, q_start + i + 1, scale)
            assert np.array_equal(out[:, :, i], dec)


# ----------------------------------------------------------------------------------------------
# feature pins
# ----------------------------------------------------------------------------------------------
def pin_features_worked_example():
    gd = _golden("features_worked.json")
    q = np.asarray(gd["q"], np.float32)
    k = _ln(gd["k_ln"])
    feat = O.score_features(q, k, gd["scale"])
    assert np.allclose(feat, gd["feat"], rtol=0, atol=2e-7)


def pin_features_match_library():
    for seed, dt in [(61, W.F32), (62, W.BF16)]:
        B, H, n, d = 2, 5, 5, 128
        g = np.random.default_rng(seed)
        q5 = W.normal(g, (B, H, n, d), dt)
        kc = W.normal(g, (B, H, 11, d), dt)          # keys read in place from a longer cache
        scale = float(np.float32(1.0 / math.sqrt(d)))
        feat = O.score_features(q5, kc, scale, n_tok=n)
        s = scale * np.einsum("bhid,bhjd->bhij", W.as_f64(q5), W.as_f64(kc)[:, :, :n])
        s = np.where(np.tril(np.ones((n, n), bool)), s, -np.inf)
        ref = scipy.special.softmax(s, axis=-1).reshape(B, H, n * n)
        assert np.allclose(feat, ref, rtol=0, atol=6e-8)          # fp32 rounding of values <= 1
        f = feat.reshape(B, H, n, n)
        assert np.all(f[..., 0, 0] == 1.0)
        assert np.all(f[np.broadcast_to(np.triu(np.ones((n, n), bool), 1), f.shape)] == 0.0)
        assert np.allclose(f.sum(-1), 1.0, rtol=0, atol=3e-7)


# ----------------------------------------------------------------------------------------------
# k-means pins
# ----------------------------------------------------------------------------------------------
def _sse(X, labels):
    X = X.astype(np.float64)
    tot = 0.0
    for j in np.unique(labels):
        m = X[labels == j]
        tot += ((m - m.mean(0)) ** 2).sum()
    return tot


def _canon(labels):
    seen, out = {}, []
    for a in labels:
        out.append(seen.setdefault(int(a), len(seen)))
    return np.asarray(out, np.int32)


def pin_kmeans_worked_examples():
    for case in _golden("kmeans_worked.json")["cases"]:
        X = np.asarray(case["feat"], np.float32)[None]
        init = np.asarray(case["init_heads"], np.int32)[None]
        h2c, rep, n, it, sse = O.kmeans(X, init, want_sse=True)
        assert h2c[0].tolist() == case["head_to_cluster"], case["name"]
        assert rep[0].tolist() == case["rep_heads"], case["name"]
        assert int(n[0]) == case["n_clusters"] and int(it[0]) == case["iters"], case["name"]
        assert abs(sse[0] - case["sse"]) < 1e-12, case["name"]


def pin_kmeans_brute_force():
    # tiny problems: Lloyd never beats the optimum over all partitions, and attains it on separated data
    for seed in range(6):
        g = np.random.default_rng(100 + seed)
        H, F, kk = 8, 3, 3
        X = g.standard_normal((H, F)).astype(np.float32)
        best = min(_sse(X, np.asarray(lab)) for lab in itertools.product(range(kk), repeat=H))
        init = W.distinct_heads(g, 1, H, kk)
        h2c, rep, n, it, sse = O.kmeans(X[None], init, want_sse=True)
        assert abs(sse[0] - _sse(X, h2c[0])) < 1e-10
        assert sse[0] >= best - 1e-10
    for seed in range(4):
        g = np.random.default_rng(200 + seed)
        H, F, kk = 9, 4, 3
        groups = W.planted_partition(g, 1, H, kk)
        cent = 10.0 * g.standard_normal((kk, F))
        X = (cent[groups[0]] + 0.05 * g.standard_normal((H, F))).astype(np.float32)
        best_lab = min(itertools.product(range(kk), repeat=H), key=lambda lab: _sse(X, np.asarray(lab)))
        init = W.one_head_per_group(g, groups, kk)
        h2c, rep, n, it = O.kmeans(X[None], init)
        assert np.array_equal(h2c[0], _canon(best_lab)) and np.array_equal(h2c[0], _canon(groups[0]))
        assert int(n[0]) == kk


def pin_kmeans_matches_sklearn_lloyd():
    from sklearn.cluster import KMeans
    import warnings
    checked = 0
    for seed in range(12):
        g = np.random.default_rng(300 + seed)
        H, F, kk = [(32, 25, 8), (52, 25, 4), (72, 25, 16), (32, 5, 8)][seed % 4]
        X = g.random((H, F)).astype(np.float32)
        init = W.distinct_heads(g, 1, H, kk)
        h2c, rep, n, it = O.kmeans(X[None], init, max_iter=100)
        with warnings.catch_warnings():
            warnings.simplefilter("ignore")
            km = KMeans(n_clusters=kk, init=X[init[0]].astype(np.float64), n_init=1, algorithm="lloyd", tol=0.0,
                        max_iter=100).fit(X.astype(np.float64))
        if len(np.unique(km.labels_)) < kk or int(n[0]) < kk:
            continue        # library and oracle treat empty centres differently; not comparable
        assert np.array_equal(h2c[0], _canon(km.labels_)), seed
        assert km.n_iter_ == int(it[0]), (km.n_iter_, it)
        checked += 1
    assert checked >= 8


def pin_kmeans_properties():
    g = np.random.default_rng(400)
    B, H, F, kk = 3, 32, 25, 8
    X = g.random((B, H, F)).astype(np.float32)
    init = W.distinct_heads(g, B, H, kk)
    h2c, rep, n, it, sse = O.kmeans(X, init, want_sse=True)
    for b in range(B):
        assert it[b] < 50
        # fixed point: every head is nearest to the mean of its own cluster
        means = np.stack([X[b][h2c[b] == j].astype(np.float64).mean(0) for j in range(n[b])])
        dist = ((X[b][:, None, :].astype(np.float64) - means[None]) ** 2).sum(-1)
        assert np.array_equal(np.argmin(dist, 1), h2c[b])
        # canonical labels and representatives
        assert np.array_equal(h2c[b], _canon(h2c[b]))
        assert rep[b, :n[b]].tolist() == [int(np.nonzero(h2c[b] == j)[0][0]) for j in range(n[b])]
        assert np.all(np.diff(rep[b, :n[b]]) > 0) and np.all(rep[b, n[b]:] == -1)
        assert abs(sse[b] - _sse(X[b], h2c[b])) < 1e-10
    # clustering error does not go up from one pass to the next; iters reports the cap when it is hit
    prev = None
    for m in range(1, int(it.max()) + 1):
        h, _, _, its, s = O.kmeans(X, init, max_iter=m, want_sse=True)
        assert np.all(its == np.minimum(it, m))
        if prev is not None:
            assert np.all(s <= prev + 1e-12)
        prev = s
    assert np.array_equal(h, h2c)
    # k = H: every head alone; k = 1: one cluster led by head 0
    init_all = np.stack([g.permutation(H) for _ in range(B)]).astype(np.int32)
    h, r, nn, _ = O.kmeans(X, init_all)
    assert np.all(h == np.arange(H)) and np.all(r == np.arange(H)) and np.all(nn == H)
    h, r, nn, _ = O.kmeans(X, np.zeros((B, 1), np.int32) + 5)
    assert np.all(h == 0) and np.all(r == 0) and np.all(nn == 1)
    # duplicate points never separate
    Xd = X.copy()
    Xd[:, 7] = Xd[:, 3]
    Xd[:, 20] = Xd[:, 3]
    h, _, _, _ = O.kmeans(Xd, init)
    assert np.all(h[:, 7] == h[:, 3]) and np.all(h[:, 20] == h[:, 3])
    # batch rows are independent problems
    h1, r1, _, _ = O.kmeans(X[1:2], init[1:2])
    assert np.array_equal(h1[0], h2c[1]) and np.array_equal(r1[0], rep[1])


def pin_kmeans_recovers_planted_features():
    # heads built as centroid + small noise (the cfg3 recipe): features cluster by planted group
    cfg = W.CONFIGS["cfg3"].reduced(L=3, B=2, T=8)
    for layer in range(cfg.L):
        x = W.layer_inputs(cfg, layer)
        feat = O.score_features(x.q5, x.k, cfg.scale, n_tok=W.N_TOK)
        h2c, rep, n, it = O.kmeans(feat, x.init_heads)
        for b in range(cfg.B):
            assert np.array_equal(h2c[b], _canon(x.groups[b])), (layer, b)
            assert int(n[b]) == cfg.ks[layer]


def pin_cluster_error_and_count():
    gd = _golden("cluster_count_worked.json")
    for c in gd["error_cases"]:
        X = np.asarray(c["feat"], np.float32)[None]
        lab = np.asarray(c["labels"], np.int32)[None]
        assert abs(O.cluster_error(X, lab, c["k"])[0] - c["sse"]) < 1e-12, c["how"]
    for c in gd["pick_cases"]:
        assert O.pick_cluster_count(c["err"], c["ks"], c["tol"]) == c["k"], c["how"]
    # against numpy on random partitions with arbitrary labels; extremes k = H and k = 1
    g = np.random.default_rng(700)
    B, H, F = 4, 32, 25
    X = g.random((B, H, F)).astype(np.float32)
    lab = g.integers(0, 11, size=(B, H)).astype(np.int32)
    e = O.cluster_error(X, lab, 11)
    for b in range(B):
        assert abs(e[b] - _sse(X[b], lab[b])) < 1e-10
    assert np.all(O.cluster_error(X, np.tile(np.arange(H, dtype=np.int32), (B, 1)), H) == 0.0)
    one = O.cluster_error(X, np.zeros((B, H), np.int32), 1)
    assert np.allclose(one, [H * X[b].astype(np.float64).var(axis=0).sum() for b in range(B)], rtol=1e-12)
    # the error curve of planted groups falls to its plateau at the planted count
    kk, ks = 6, [1, 2, 3, 4, 6, 8, 12, 16]
    groups = W.planted_partition(g, B, H, kk)
    cent = g.standard_normal((B, kk, F))
    Xp = np.stack([cent[b, groups[b]] for b in range(B)]) + 0.01 * g.standard_normal((B, H, F))
    Xp = Xp.astype(np.float32)
    curve = []
    for k_try in ks:
        init = W.one_head_per_group(g, groups, kk)[:, :k_try] if k_try <= kk else np.concatenate(
            [W.one_head_per_group(g, groups, kk),
             np.stack([g.choice(np.setdiff1d(np.arange(H), W.one_head_per_group(g, groups, kk)[b]), k_try - kk,
                                replace=False) for b in range(B)])], axis=1)
        h2c, _, _, _ = O.kmeans(Xp, init.astype(np.int32))
        curve.append(O.cluster_error(Xp, h2c, k_try).mean())
    assert all(curve[i + 1] <= curve[i] + 1e-9 for i in range(len(ks) - 1))
    assert O.pick_cluster_count(curve, ks, 0.02) == kk


# ----------------------------------------------------------------------------------------------
# projection pins
# ----------------------------------------------------------------------------------------------
def pin_projection_of_representatives():
    # hand-worked: D = 2, d = 1, H = 3: w_q rows (1,0),(0,1),(1,1); w_k rows (2,0),(0,3),(1,-1); token x = (5,7)
    x = np.array([[[5.0, 7.0], [1.0, -1.0]]], np.float32)
    w_q = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]], np.float32)
    w_k = np.array([[2.0, 0.0], [0.0, 3.0], [1.0, -1.0]], np.float32)
    q, k = O.project_qk(x, w_q, w_k, np.array([[2, 0]], np.int32), 1)
    assert q[0, :, :, 0].tolist() == [[12.0, 0.0], [5.0, 1.0]]          # slot 0 = head 2, slot 1 = head 0
    assert k[0, :, :, 0].tolist() == [[-2.0, 2.0], [10.0, 2.0]]
    # library contraction, fp32 and bf16 storage, an unused slot, heads that are nobody's representative poisoned
    for seed, dt in [(71, W.F32), (72, W.BF16)]:
        g = np.random.default_rng(seed)
        B, H, kk, Tn, D, d = 2, 6, 3, 5, 24, 4
        x = W.normal(g, (B, Tn, D), dt)
        w_q, w_k = W.normal(g, (H * d, D), dt), W.normal(g, (H * d, D), dt)
        _, rep = W.random_membership(g, B, H, kk)
        rep[1, 2] = -1
        q, k = O.project_qk(x, w_q, w_k, rep, d)
        x64 = W.as_f64(x)
        wq64, wk64 = W.as_f64(w_q).reshape(H, d, D), W.as_f64(w_k).reshape(H, d, D)
        for b in range(B):
            for j in range(kk):
                if rep[b, j] < 0:
                    assert np.all(np.isnan(q[b, j])) and np.all(np.isnan(k[b, j]))
                    continue
                assert np.allclose(q[b, j], np.einsum("te,ce->tc", x64[b], wq64[rep[b, j]]), rtol=1e-13, atol=1e-13)
                assert np.allclose(k[b, j], np.einsum("te,ce->tc", x64[b], wk64[rep[b, j]]), rtol=1e-13, atol=1e-13)
        used = {int(r) for r in rep.ravel() if r >= 0}
        w_q2, w_k2 = w_q.copy().reshape(H, d, D), w_k.copy().reshape(H, d, D)
        for h in range(H):
            if h not in used:
                w_q2[h], w_k2[h] = (0x7FC0 if dt == W.BF16 else np.nan), (0x7FC0 if dt == W.BF16 else np.nan)
        q2, k2 = O.project_qk(x, w_q2.reshape(H * d, D), w_k2.reshape(H * d, D), rep, d)
        assert np.array_equal(q2, q, equal_nan=True) and np.array_equal(k2, k, equal_nan=True)


# ----------------------------------------------------------------------------------------------
# cache pins
# ----------------------------------------------------------------------------------------------
def pin_compaction_is_a_gather():
    for dt in (W.F32, W.BF16):
        g = np.random.default_rng(500 + dt)
        B, H, T, T_cap, Tc_cap, d, kk = 2, 6, 11, 14, 12, 16, 3
        kf = W.normal(g, (B, H, T_cap, d), dt)
        _, rep = W.random_membership(g, B, H, kk)
        rep[1, 2] = -1                                   # an unused slot stays untouched
        sentinel = np.full((B, kk, Tc_cap, d), 7, kf.dtype)
        kc, src = O.compact_kcache(kf, rep, T, k_compact=sentinel.copy(), want_src_rows=True)
        for b in range(B):
            for j in range(kk):
                if rep[b, j] < 0:
                    assert np.all(kc[b, j] == 7) and np.all(src[b, j] == -1)
                    continue
                assert np.array_equal(kc[b, j, :T], kf[b, rep[b, j], :T])
                assert np.all(kc[b, j, T:] == 7)
                assert np.array_equal(src[b, j], (b * H + rep[b, j]) * T_cap + np.arange(T))
        # with every head its own representative the compact cache is the cache
        ident = np.tile(np.arange(H, dtype=np.int32), (B, 1))
        assert np.array_equal(O.compact_kcache(kf, ident, T_cap), kf)
        # attention over the gathered keys with identity maps equals clustered attention over the full cache
        rep[1, 2] = 5
        kc = O.compact_kcache(kf, rep, T, Tc_cap=T_cap)
        q = W.normal(g, (B, H, d), dt)
        v = W.normal(g, (B, H, T_cap, d), dt)
        h2c = np.stack([g.integers(0, kk, H) for _ in range(B)]).astype(np.int32)
        full = O.clustered_decode(q, kf, v, h2c, rep, T, 0.25)
        qc = np.stack([q[b, rep[b]] for b in range(B)])
        _, p = O.dense_decode(qc, kc, kc, T, 0.25, want_probs=True)
        ref = np.stack([np.stack([p[b, h2c[b, h]] @ W.as_f64(v)[b, h, :T] for h in range(H)]) for b in range(B)])
        assert np.allclose(full, ref, rtol=1e-12, atol=1e-13)


def pin_append_writes_one_row():
    g = np.random.default_rng(600)
    B, H, T_cap, Tc_cap, d, kk, pos = 2, 5, 9, 8, 8, 2, 6
    _, rep = W.random_membership(g, B, H, kk)
    kc0 = W.normal(g, (B, kk, Tc_cap, d), W.BF16)
    v0 = W.normal(g, (B, H, T_cap, d), W.BF16)
    kn, vn = W.normal(g, (B, H, d), W.BF16), W.normal(g, (B, H, d), W.BF16)
    kc, v = kc0.copy(), v0.copy()
    O.append_kv(kn, vn, rep, kc, v, pos)
    ek, ev = kc0.copy(), v0.copy()
    for b in range(B):
        ek[b, :, pos] = kn[b, rep[b]]
    ev[:, :, pos] = vn
    assert np.array_equal(kc, ek) and np.array_equal(v, ev)


# ----------------------------------------------------------------------------------------------
# quantised caches: 8-bit floating point codes, per-row scales, attention over dequantised tensors
# ----------------------------------------------------------------------------------------------
def _finite_e4m3():
    """(code, value) of every finite code, from the field layout written out here (not from the oracle)."""
    out = []
    for code in range(256):
        sgn, e, m = code >> 7, (code >> 3) & 15, code & 7
        if e == 15 and m == 7:
            continue
        mag = (m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7)
        out.append((code, -mag if sgn else mag))
    return out


def pin_e4m3_codes_match_the_format():
    import torch
    g = _golden("e4m3_worked.json")
    for c in g["codes"]:
        assert O.e4m3_decode(c["code"]) == c["value"], c
    for c in g["nan_codes"]:
        assert math.isnan(O.e4m3_decode(c))
    vals = [O.e4m3_decode(c) for c in range(0x7f)]
    assert all(b > a for a, b in zip(vals, vals[1:])) and vals[0] == 0.0          # positive codes ascend
    assert all(O.e4m3_decode(c | 0x80) == -O.e4m3_decode(c) for c in range(0x7f))
    # a library's decoder of the same format, all 256 codes
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    mine = np.array([O.e4m3_decode(c) for c in range(256)])
    assert np.array_equal(np.isnan(lib), np.isnan(mine)) and np.array_equal(lib[~np.isnan(lib)], mine[~np.isnan(mine)])
    for code, value in _finite_e4m3():
        assert mine[code] == value


def pin_e4m3_encode_is_nearest_even():
    import torch
    g = _golden("e4m3_worked.json")
    for c in g["encode"]:
        assert O.e4m3_encode(c["y"]) == c["code"], c
    table = _finite_e4m3()
    codes = np.array([c for c, _ in table])
    vals = np.array([v for _, v in table])
    rng = np.random.default_rng(5150)
    ys = np.concatenate([rng.standard_normal(3000) * 100, rng.standard_normal(3000), rng.standard_normal(3000) * 0.01,
                         rng.uniform(-448, 448, 3000), [448.0, -448.0, 0.0, 2.0 ** -9, 2.0 ** -10]]).astype(np.float32)
    ys = np.clip(ys, -448, 448)
    # brute force: the finite value at the smallest distance; on a tie the code with an even mantissa
    for y in ys[:4000]:
        dist = np.abs(vals - np.float64(y))
        best = np.flatnonzero(dist == dist.min())
        want = {int(codes[i]) for i in best}
        if len(want) > 1 and not (want == {0, 0x80}):
            want = {c for c in want if c % 2 == 0}
        got = O.e4m3_encode(y)
        assert got in want or (y == 0 and got in (0, 0x80)), (float(y), got, want)
    # a library's conversion of the same format
    lib = torch.from_numpy(ys).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    mine = np.array([O.e4m3_encode(y) for y in ys], np.uint8)
    assert np.array_equal(lib, mine)
    # decode(encode(v)) returns every representable value
    for code, value in table:
        assert O.e4m3_decode(O.e4m3_encode(value)) == value


def pin_quantized_rows():
    g = _golden("e4m3_worked.json")
    for row in g["rows"]:
        codes, scale = O.quantize_rows(np.asarray(row["x"], np.float32)[None])
        assert codes[0].tolist() == row["codes"], row
        assert scale[0] == np.float32(row["scale"]), (row, scale)
    rng = np.random.default_rng(5151)
    for dtype in (W.F32, W.BF16):
        x = W.normal(rng, (7, 33, 128), dtype, sigma=3.0)
        xf = W.as_f64(x)
        codes, scales = O.quantize_rows(x)
        amax = np.abs(xf).max(-1)
        assert np.array_equal(scales, (amax.astype(np.float32) / np.float32(448)).astype(np.float32))
        deq = O.dequantize_rows(codes, scales)
        # the element with the largest magnitude maps to +-448; nothing is off by more than half a spacing:
        # 2^-4 relative for normal codes, half of the smallest step (2^-10 of the scale) below that
        assert np.all(np.abs(np.vectorize(O.e4m3_decode)(codes)).max(-1) == 448.0)
        bound = np.maximum(np.abs(xf) * 2.0 ** -4, scales[..., None].astype(np.float64) * 2.0 ** -10) * (1 + 1e-5)
        assert np.all(np.abs(deq - xf) <= bound)
        # scaling a row by a power of two leaves the codes alone and scales the scale
        x4 = W.store(W.as_f64(x).astype(np.float32) * 4.0, dtype)
        c4, s4 = O.quantize_rows(x4)
        assert np.array_equal(c4, codes) and np.array_equal(s4, scales * np.float32(4))
    # dequantisation is decode(code) * scale, against the library decoder
    import torch
    lib = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy() * scales[..., None].astype(np.float64)
    assert np.array_equal(lib, deq)


def pin_quantized_attention_matches_library():
    import torch
    rng = np.random.default_rng(5152)
    B, H, kk, T, T_cap, d = 2, 6, 3, 37, 40, 16
    scale = 0.25
    for dtype in (W.F32, W.BF16):
        q = W.normal(rng, (B, H, d), dtype)
        kf = W.normal(rng, (B, H, T_cap, d), dtype)
        vf = W.normal(rng, (B, H, T_cap, d), dtype, sigma=2.0)
        h2c, rep = W.random_membership(rng, B, H, kk)
        k8, ks = O.quantize_rows(kf)
        v8, vs = O.quantize_rows(vf)
        out, probs = O.clustered_decode_q8(q, k8, ks, v8, vs, h2c, rep, T, scale, want_probs=True)
        # library: decode the codes with torch, scale per row, then softmax + contraction in numpy fp64
        kd = torch.from_numpy(k8.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy() * ks[..., None].astype(np.float64)
        vd = torch.from_numpy(v8.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy() * vs[..., None].astype(np.float64)
        q64 = W.as_f64(q)
        sc = np.float64(np.float32(scale))
        for b in range(B):
            for j in range(kk):
                r = rep[b, j]
                p = scipy.special.softmax(sc * kd[b, r, :T] @ q64[b, r])
                assert np.abs(p - probs[b, j]).max() < 1e-13
            for h in range(H):
                p = scipy.special.softmax(sc * kd[b, rep[b, h2c[b, h]], :T] @ q64[b, rep[b, h2c[b, h]]])
                assert np.abs(p @ vd[b, h, :T] - out[b, h]).max() < 1e-12
        # the quantised result stays near the unquantised one (error of a few percent of the row scale at most)
        plain = O.clustered_decode(q, kf, vf, h2c, rep, T, scale)
        assert np.abs(out - plain).max() < 0.15 * np.abs(plain).max()
        # scales that are all 1 and codes that are exact: identical to plain attention on the decoded values
        ones = np.ones_like(ks)
        kx = torch.from_numpy(k8.copy()).view(torch.float8_e4m3fn).to(torch.float32).numpy()
        vx = torch.from_numpy(v8.copy()).view(torch.float8_e4m3fn).to(torch.float32).numpy()
        a = O.clustered_decode_q8(q if dtype == W.F32 else W.as_f64(q).astype(np.float32), k8, ones, v8, ones, h2c, rep, T, scale)
        bb = O.clustered_decode(W.as_f64(q).astype(np.float32), kx, vx, h2c, rep, T, scale)
        assert np.abs(a - bb).max() < 1e-12 * max(1.0, np.abs(bb).max())


ALL_PINS = [v for n, v in sorted(globals().items()) if n.startswith("pin_") and callable(v)]
