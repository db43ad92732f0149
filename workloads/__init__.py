"""Seeded synthetic inputs and the registry of the five benchmark configurations.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds NO arithmetic of the method: it draws random tensors,
draws random partitions of heads, converts fp32 to bf16 bit patterns, and
records shapes.  Scores, softmax, k-means, compaction and attention live
elsewhere (once in ``oracle/``, once in the HIP library).

The inputs stand in for the paper's workloads (LLaMa-7B / LLaMa-33B / OPT-66B
decode at sequence lengths up to 2048, skewed cluster sizes, few clusters in
late layers and none in the first ones); no trained weights, prompts or
benchmark items are involved.

bf16 tensors are numpy ``uint16`` arrays of bit patterns (host) or
``torch.bfloat16`` tensors (device filler).
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

F32, BF16 = 0, 1
N_TOK = 5  # tokens whose attention scores decide cluster membership (Section 3.3)

_TAGS = {"q": 1, "k": 2, "v": 3, "q5": 4, "init": 5, "member": 6, "ck": 7, "cq": 8, "knew": 9, "vnew": 10,
         "qstep": 11, "kcount": 12, "planted": 13, "cq5": 14}


# --------------------------------------------------------------------------------------
# configurations
# --------------------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class Config:
    """One benchmark configuration (shapes only; tensors come from the generators below)."""
    name: str
    L: int                 # layers
    H: int                 # heads per layer
    d: int                 # head dimension
    B: int                 # batch rows (independent requests)
    T: int                 # cached tokens attended to (current token included)
    T_cap: int             # capacity of the caches along the token axis
    dtype: int             # F32 or BF16 (storage type of q, K, V)
    ks: Tuple[int, ...]    # clusters per layer
    membership: str        # "random" | "kmeans" | "planted" | "skewed"
    seed: int
    sizes: Optional[Tuple[int, ...]] = None   # cluster sizes for "skewed"
    prompt: int = 0        # end-to-end config: prompt length
    decode_steps: int = 0  # end-to-end config: decode steps after the prompt

    @property
    def scale(self) -> float:
        return float(np.float32(1.0 / math.sqrt(self.d)))

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == F32 else 2

    def clustered_bytes_per_step(self, T: Optional[int] = None) -> int:
        """Bytes the method itself must move for one decode step over all layers."""
        T = self.T if T is None else T
        e, tot = self.elem_bytes, 0
        for k in self.ks:
            tot += self.B * k * T * self.d * e + self.B * self.H * T * self.d * e   # compact K + all V
            tot += self.B * k * self.d * e + 2 * self.B * self.H * 4                # q of representatives + maps
            tot += self.B * self.H * self.d * 4                                     # output
        return tot

    def dense_bytes_per_step(self, T: Optional[int] = None) -> int:
        T = self.T if T is None else T
        e = self.elem_bytes
        per = 2 * self.B * self.H * T * self.d * e + self.B * self.H * self.d * e + self.B * self.H * self.d * 4
        return per * self.L

    def k_bytes_saved(self, T: Optional[int] = None) -> int:
        T = self.T if T is None else T
        return sum(self.B * (self.H - k) * T * self.d * self.elem_bytes for k in self.ks)

    def reduced(self, L: int, B: int, T: int, T_cap: Optional[int] = None) -> "Config":
        """Same head structure at a size the oracle finishes in seconds; layers are sampled evenly."""
        idx = sorted(set(int(round(i * (self.L - 1) / max(L - 1, 1))) for i in range(L))) if self.L > 1 else [0]
        ks = tuple(self.ks[i] for i in idx)
        return dataclasses.replace(self, name=self.name + "-reduced", L=len(ks), B=B, T=T,
                                   T_cap=T if T_cap is None else T_cap, ks=ks)


def _cfg3_ks(L: int, seed: int) -> Tuple[int, ...]:
    g = np.random.Generator(np.random.Philox(key=[seed, _TAGS["kcount"]]))
    return tuple(int(x) for x in g.choice([4, 8, 16], size=L))


CONFIGS = {
    # single layer, fp32, random membership
    "cfg1": Config("cfg1", L=1, H=32, d=128, B=1, T=256, T_cap=256, dtype=F32, ks=(8,), membership="random",
                   seed=101),
    # LLaMa-7B shape: first 4 layers unclustered, the rest 8 clusters from k-means on 5-token features
    "cfg2": Config("cfg2", L=32, H=32, d=128, B=16, T=2048, T_cap=2048, dtype=BF16, ks=(32,) * 4 + (8,) * 28,
                   membership="kmeans", seed=202),
    # LLaMa-33B shape: per-layer k in {4,8,16}; heads are planted centroids + noise
    "cfg3": Config("cfg3", L=60, H=52, d=128, B=8, T=2048, T_cap=2048, dtype=BF16, ks=_cfg3_ks(60, 303),
                   membership="planted", seed=303),
    # OPT-66B shape, end to end: 512-token prompt, k-means, compaction, 128 decode steps
    "cfg4": Config("cfg4", L=64, H=72, d=128, B=4, T=2048, T_cap=2048, dtype=BF16, ks=(16,) * 64,
                   membership="kmeans", seed=404, prompt=512, decode_steps=128),
    # long context, skewed clusters
    "cfg5": Config("cfg5", L=8, H=32, d=128, B=4, T=32768, T_cap=32768, dtype=BF16, ks=(4,) * 8,
                   membership="skewed", seed=505, sizes=(20, 6, 4, 2)),
}


# --------------------------------------------------------------------------------------
# bf16 bit patterns
# --------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even) and return the uint16 bit patterns."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32)


def as_f64(a: np.ndarray) -> np.ndarray:
    """Exact fp64 view of a stored tensor (fp32 array or bf16 bit patterns)."""
    return (bf16_bits_to_f32(a) if a.dtype == np.uint16 else a).astype(np.float64)


# --------------------------------------------------------------------------------------
# host generators (numpy, counter-based Philox streams)
# --------------------------------------------------------------------------------------
def rng(seed: int, layer: int, tag: str, extra: int = 0) -> np.random.Generator:
    key = [np.uint64(seed), (np.uint64(layer) << np.uint64(40)) | (np.uint64(extra) << np.uint64(8)) |
           np.uint64(_TAGS[tag])]
    return np.random.Generator(np.random.Philox(key=key))


def store(x: np.ndarray, dtype: int) -> np.ndarray:
    """fp32 values -> storage type (fp32 unchanged, or bf16 bit patterns)."""
    x = np.ascontiguousarray(x, np.float32)
    return x if dtype == F32 else f32_to_bf16_bits(x)


def normal(g: np.random.Generator, shape: Sequence[int], dtype: int, sigma: float = 1.0) -> np.ndarray:
    x = g.standard_normal(size=tuple(shape), dtype=np.float32)
    if sigma != 1.0:
        x *= np.float32(sigma)
    return store(x, dtype)


def random_membership(g: np.random.Generator, B: int, H: int, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """Uniformly random head->cluster maps with every cluster non-empty; representative = lowest member."""
    h2c = np.empty((B, H), np.int32)
    for b in range(B):
        # k randomly chosen heads seed the k clusters (so none is empty), the others fall uniformly
        a = g.integers(0, k, size=H)
        a[g.choice(H, size=k, replace=False)] = np.arange(k)
        h2c[b] = a
    return h2c, representatives(h2c, k)


def sized_membership(g: np.random.Generator, B: int, H: int, sizes: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """Partitions with prescribed cluster sizes; which heads fall where is drawn per batch row."""
    assert sum(sizes) == H
    k = len(sizes)
    h2c = np.empty((B, H), np.int32)
    labels = np.repeat(np.arange(k, dtype=np.int32), sizes)
    for b in range(B):
        h2c[b] = labels[g.permutation(H)]
    return h2c, representatives(h2c, k)


def representatives(h2c: np.ndarray, k: int) -> np.ndarray:
    """Lowest-index member of each cluster ([B,k], -1 where a cluster has no member)."""
    B, H = h2c.shape
    rep = np.full((B, k), -1, np.int32)
    for b in range(B):
        for h in range(H - 1, -1, -1):
            rep[b, h2c[b, h]] = h
    return rep


def distinct_heads(g: np.random.Generator, B: int, H: int, k: int) -> np.ndarray:
    """k distinct head ids per batch row: the caller-chosen k-means starting points."""
    return np.stack([g.choice(H, size=k, replace=False) for _ in range(B)]).astype(np.int32)


def planted_partition(g: np.random.Generator, B: int, H: int, k: int) -> np.ndarray:
    """Random partition of the heads into k non-empty groups with skewed sizes, [B,H] group ids."""
    out = np.empty((B, H), np.int32)
    for b in range(B):
        w = g.dirichlet(np.full(k, 0.7))
        a = np.concatenate([np.arange(k), g.choice(k, size=H - k, p=w)])
        out[b] = a[g.permutation(H)]
    return out


def one_head_per_group(g: np.random.Generator, groups: np.ndarray, k: int) -> np.ndarray:
    """One random member of every planted group: starting points that cover all groups."""
    B, H = groups.shape
    init = np.empty((B, k), np.int32)
    for b in range(B):
        for j in range(k):
            init[b, j] = g.choice(np.nonzero(groups[b] == j)[0])
    return init


def centroid_plus_noise(g_cent: np.random.Generator, g_noise: np.random.Generator, groups: np.ndarray, k: int,
                        rows: int, d: int, dtype: int, sigma: float = 0.1) -> np.ndarray:
    """x[b,h,t,:] = centroid[b, groups[b,h], t, :] + sigma * N(0,1)  (heads of a group nearly coincide)."""
    B, H = groups.shape
    cent = g_cent.standard_normal(size=(B, k, rows, d), dtype=np.float32)
    x = np.empty((B, H, rows, d), np.float32)
    for b in range(B):
        x[b] = cent[b, groups[b]]
    x += np.float32(sigma) * g_noise.standard_normal(size=(B, H, rows, d), dtype=np.float32)
    return store(x, dtype)


@dataclasses.dataclass
class LayerInputs:
    """Host tensors of one layer.  ``groups``/``h2c``/``rep`` are inputs (drawn), never computed here."""
    q: np.ndarray                  # [B,H,d]       query of the decode token
    k: np.ndarray                  # [B,H,T_cap,d] full key cache
    v: np.ndarray                  # [B,H,T_cap,d] value cache
    q5: np.ndarray                 # [B,H,N_TOK,d] queries of the first N_TOK positions
    k_layer: int                   # clusters in this layer
    init_heads: Optional[np.ndarray] = None   # [B,k] k-means starting heads ("kmeans", "planted")
    h2c: Optional[np.ndarray] = None          # [B,H] drawn membership ("random", "skewed")
    rep: Optional[np.ndarray] = None          # [B,k]
    groups: Optional[np.ndarray] = None       # [B,H] planted groups ("planted")


def layer_inputs(cfg: Config, layer: int) -> LayerInputs:
    """All host tensors of one layer of a configuration (sized by cfg: use cfg.reduced() for the oracle)."""
    B, H, d, Tc, dt, s = cfg.B, cfg.H, cfg.d, cfg.T_cap, cfg.dtype, cfg.seed
    k = cfg.ks[layer]
    out = LayerInputs(q=None, k=None, v=None, q5=None, k_layer=k)
    out.v = normal(rng(s, layer, "v"), (B, H, Tc, d), dt)
    if cfg.membership == "planted":
        groups = planted_partition(rng(s, layer, "planted"), B, H, k)
        out.groups = groups
        out.k = centroid_plus_noise(rng(s, layer, "ck"), rng(s, layer, "k"), groups, k, Tc, d, dt)
        out.q5 = centroid_plus_noise(rng(s, layer, "cq5"), rng(s, layer, "q5"), groups, k, N_TOK, d, dt)
        out.q = centroid_plus_noise(rng(s, layer, "cq"), rng(s, layer, "q"), groups, k, 1, d, dt)[:, :, 0, :].copy()
        out.init_heads = one_head_per_group(rng(s, layer, "init"), groups, k)
        return out
    out.k = normal(rng(s, layer, "k"), (B, H, Tc, d), dt)
    out.q = normal(rng(s, layer, "q"), (B, H, d), dt)
    out.q5 = normal(rng(s, layer, "q5"), (B, H, N_TOK, d), dt)
    if cfg.membership == "kmeans":
        out.init_heads = distinct_heads(rng(s, layer, "init"), B, H, k)
    elif cfg.membership == "random":
        out.h2c, out.rep = random_membership(rng(s, layer, "member"), B, H, k)
    elif cfg.membership == "skewed":
        out.h2c, out.rep = sized_membership(rng(s, layer, "member"), B, H, cfg.sizes)
    else:
        raise ValueError(cfg.membership)
    return out


def step_inputs(cfg: Config, layer: int, step: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """q, k_new, v_new [B,H,d] of decode step `step` (end-to-end configuration)."""
    shp = (cfg.B, cfg.H, cfg.d)
    return (normal(rng(cfg.seed, layer, "qstep", step), shp, cfg.dtype),
            normal(rng(cfg.seed, layer, "knew", step), shp, cfg.dtype),
            normal(rng(cfg.seed, layer, "vnew", step), shp, cfg.dtype))


# --------------------------------------------------------------------------------------
# device filler for full-size tensors (timing runs and sampled parity)
# --------------------------------------------------------------------------------------
def device_normal(shape: Sequence[int], dtype: int, seed: int, device="cuda", sigma: float = 1.0):
    """N(0, sigma^2) tensor drawn on the device by torch's seeded generator (fp32 -> bf16 by torch's RNE cast)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    x = torch.randn(tuple(shape), generator=g, device=device, dtype=torch.float32)
    if sigma != 1.0:
        x *= sigma
    return x if dtype == F32 else x.to(torch.bfloat16)


def device_centroid_plus_noise(groups: np.ndarray, k: int, rows: int, d: int, dtype: int, seed: int,
                               device="cuda", sigma: float = 0.1):
    """Device version of centroid_plus_noise for full-size planted caches."""
    import torch
    B, H = groups.shape
    cent = device_normal((B, k, rows, d), F32, seed, device)
    idx = torch.as_tensor(groups.astype(np.int64), device=device)
    x = torch.stack([cent[b].index_select(0, idx[b]) for b in range(B)])
    x += device_normal((B, H, rows, d), F32, seed + 1, device, sigma)
    return x if dtype == F32 else x.to(torch.bfloat16)


def torch_to_host_bits(t) -> np.ndarray:
    """Device/host torch tensor -> numpy array the oracle accepts (fp32, or uint16 bit patterns for bf16)."""
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def host_to_torch(a: np.ndarray, device="cuda"):
    """numpy array (fp32 / bf16 bits / int32) -> device tensor holding the same bytes."""
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).to(device)
    return torch.from_numpy(np.ascontiguousarray(a).copy()).to(device)
