"""Seeded synthetic inputs for the Clover-2 speculative step.

This module only *generates inputs*: model shapes, random-init weights, static
tree topologies and prompts.  It holds none of the method's arithmetic (no
norms, no attention, no draft head, no acceptance) so that both the CPU oracle
and the HIP path can be fed from it without sharing any computation.

Recipes
-------
* Weights: every tensor is drawn N(0, std=0.02) from its own SFC64 stream
  seeded by (key, seed, crc32(tensor name)), so a tensor's values do not
  depend on which other tensors were generated or in what order.
  Norm gains are 1.0 (optionally 1 + gain_jitter*N(0,1) for stronger tests).
  For bf16 models each tensor is rounded once to bf16 (round-to-nearest-even)
  and handed out as uint16 bit patterns; `bf16_bits_to_f32` widens them.
* Trees: `make_tree` enumerates the full k_1 x k_2 x ... tree, scores a node by
  the product over its path of 1/(1+rank) and keeps the root plus the heaviest
  nodes, renumbered in breadth-first order.
* Prompts: token ids uniform in [0, vocab).
"""
from __future__ import annotations

import zlib
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from fractions import Fraction
from typing import Dict, Iterable, List, Sequence, Tuple

import numpy as np

WEIGHT_KEY = 240800264  # seed word shared by all weight streams


@dataclass(frozen=True)
class ModelShape:
    """Shape of a LLaMA-style target plus its Clover-2 draft head."""
    name: str
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rope_base: float
    rms_eps: float = 1e-5
    bf16: bool = False
    aug_layers: int = 1
    ad_heads: int = 0          # 0 -> n_q_heads
    draft_depths: int = 3      # D: deepest tree level
    tree_k: Tuple[int, ...] = (4, 3, 2)
    tree_nodes: int = 16
    batch: int = 1
    prompt_len: Tuple[int, int] = (64, 64)   # inclusive range, per sequence
    steps: int = 8
    seed: int = 1

    @property
    def heads_ad(self) -> int:
        return self.ad_heads or self.n_q_heads


# The five workloads (model shape + tree + batch/prompt recipe).
CONFIGS: Dict[int, ModelShape] = {
    1: ModelShape("tiny-fp32", 2, 256, 4, 4, 64, 688, 1024, 1e4, bf16=False,
                  draft_depths=3, tree_k=(4, 3, 2), tree_nodes=16,
                  batch=1, prompt_len=(64, 64), steps=8, seed=1),
    2: ModelShape("vicuna7b-shape-bf16", 32, 4096, 32, 32, 128, 11008, 32000, 1e4, bf16=True,
                  draft_depths=4, tree_k=(8, 6, 4, 3), tree_nodes=64,
                  batch=1, prompt_len=(512, 512), steps=128, seed=2),
    3: ModelShape("llama3-8b-shape-bf16", 32, 4096, 32, 8, 128, 14336, 128256, 5e5, bf16=True,
                  draft_depths=4, tree_k=(8, 6, 4, 3), tree_nodes=64,
                  batch=1, prompt_len=(1024, 1024), steps=32, seed=3),
    4: ModelShape("llama3-8b-shape-bf16-b8", 32, 4096, 32, 8, 128, 14336, 128256, 5e5, bf16=True,
                  draft_depths=4, tree_k=(6, 4, 3, 2), tree_nodes=32,
                  batch=8, prompt_len=(256, 2048), steps=16, seed=4),
    5: ModelShape("llama3-8b-shape-bf16-long", 32, 4096, 32, 8, 128, 14336, 128256, 5e5, bf16=True,
                  draft_depths=5, tree_k=(8, 6, 4, 3, 2), tree_nodes=96,
                  batch=1, prompt_len=(8192, 8192), steps=16, seed=5),
}


def scaled(shape: ModelShape, **kw) -> ModelShape:
    """A copy of `shape` with some fields replaced (reduced-size test cases)."""
    return replace(shape, **kw)


# ----------------------------------------------------------------------------
# bf16 bit patterns
# ----------------------------------------------------------------------------
def _f32_to_bf16_bits_np(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return r.astype(np.uint16)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits.
    Large arrays go through torch's CPU conversion (same rounding, much faster)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if x.size >= (1 << 20):
        try:
            import torch
            return torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        except ImportError:
            pass
    return _f32_to_bf16_bits_np(x)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# weights
# ----------------------------------------------------------------------------
def _stream(name: str, seed: int) -> np.random.Generator:
    ss = np.random.SeedSequence([WEIGHT_KEY, int(seed), zlib.crc32(name.encode())])
    return np.random.Generator(np.random.SFC64(ss))


def tensor_normal(name: str, shape: Sequence[int], seed: int, std: float = 0.02) -> np.ndarray:
    g = _stream(name, seed)
    out = g.standard_normal(size=tuple(shape), dtype=np.float32)
    out *= np.float32(std)
    return out


def layer_tensor_shapes(s: ModelShape) -> Dict[str, Tuple[int, ...]]:
    H, d = s.hidden, s.head_dim
    return {
        "attn_norm": (H,), "wq": (s.n_q_heads * d, H), "wk": (s.n_kv_heads * d, H),
        "wv": (s.n_kv_heads * d, H), "wo": (H, s.n_q_heads * d), "ffn_norm": (H,),
        "w_gate": (s.ffn, H), "w_up": (s.ffn, H), "w_down": (H, s.ffn),
    }


def weight_shapes(s: ModelShape) -> Dict[str, Tuple[int, ...]]:
    """Name -> shape for every tensor of the target and the draft head.
    Linear weights are [out_features, in_features]."""
    H = s.hidden
    out: Dict[str, Tuple[int, ...]] = {"embed": (s.vocab, H)}
    for i in range(s.n_layers):
        for k, v in layer_tensor_shapes(s).items():
            out[f"layers.{i}.{k}"] = v
    out["final_norm"] = (H,)
    out["lm_head"] = (s.vocab, H)
    for ad in ("ad1", "ad2"):
        out[f"{ad}.norm"] = (H,)
        for p in ("q", "k", "v"):
            out[f"{ad}.w{p}"] = (H, H)
            out[f"{ad}.b{p}"] = (H,)
    for i in range(s.aug_layers):
        for k, v in layer_tensor_shapes(s).items():
            out[f"aug.{i}.{k}"] = v
    out["fc0.w"] = (H, H)
    out["fc0.b"] = (H,)
    for j in range(1, s.draft_depths):
        out[f"fc.{j}.w"] = (H, 2 * H)
        out[f"fc.{j}.b"] = (H,)
    out["head_norm"] = (H,)
    return out


def _is_norm(name: str) -> bool:
    return name.endswith("norm")


class WeightStore:
    """Lazily generated, cached weights of one model.

    `get(name)` returns float32 for fp32 models and uint16 bf16 bit patterns
    for bf16 models.  `get_f32(name)` always returns float32 values (the bf16
    ones widened exactly)."""

    def __init__(self, shape: ModelShape, seed: int | None = None, gain_jitter: float = 0.0,
                 overrides: Dict[str, np.ndarray] | None = None):
        self.shape = shape
        self.seed = shape.seed if seed is None else seed
        self.gain_jitter = float(gain_jitter)
        self.shapes = weight_shapes(shape)
        self._cache: Dict[str, np.ndarray] = {}
        self._overrides = dict(overrides or {})

    def names(self) -> List[str]:
        return list(self.shapes.keys())

    def _make_f32(self, name: str) -> np.ndarray:
        if name in self._overrides:
            a = np.asarray(self._overrides[name], dtype=np.float32)
            assert a.shape == self.shapes[name], (name, a.shape, self.shapes[name])
            return a
        shp = self.shapes[name]
        if _is_norm(name):
            if self.gain_jitter == 0.0:
                return np.ones(shp, dtype=np.float32)
            return (1.0 + tensor_normal(name, shp, self.seed, self.gain_jitter)).astype(np.float32)
        return tensor_normal(name, shp, self.seed, 0.02)

    def get(self, name: str) -> np.ndarray:
        a = self._cache.get(name)
        if a is None:
            a = self._make_f32(name)
            if self.shape.bf16:
                a = f32_to_bf16_bits(a)
            self._cache[name] = a
        return a

    def get_f32(self, name: str) -> np.ndarray:
        a = self.get(name)
        return bf16_bits_to_f32(a) if a.dtype == np.uint16 else a

    def drop(self, name: str) -> None:
        self._cache.pop(name, None)

    def prefetch(self, names: Iterable[str], threads: int = 8) -> None:
        """Generate several tensors concurrently (numpy releases the GIL)."""
        todo = [n for n in names if n not in self._cache]
        if not todo:
            return
        with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
            list(ex.map(self.get, todo))


# ----------------------------------------------------------------------------
# static trees
# ----------------------------------------------------------------------------
def make_tree(k: Sequence[int], n_nodes: int) -> Tuple[np.ndarray, np.ndarray]:
    """Static draft tree: (parent[N], rank[N]) int32 in breadth-first order.

    Node 0 is the root (parent -1, rank 0).  A node at depth j >= 1 is the
    rank-th best continuation of its parent, rank in [0, k[j-1]).  Of the full
    tree, the root and the n_nodes-1 heaviest nodes are kept, where a node's
    weight is the product of 1/(1+rank) along its path; ties prefer the
    shallower node, then the lexicographically smaller rank path."""
    full: List[Tuple[Fraction, int, Tuple[int, ...]]] = []
    frontier: List[Tuple[Tuple[int, ...], Fraction]] = [((), Fraction(1))]
    for kj in k:
        nxt = []
        for path, w in frontier:
            for r in range(kj):
                p2 = path + (r,)
                w2 = w / (1 + r)
                full.append((w2, len(p2), p2))
                nxt.append((p2, w2))
        frontier = nxt
    if n_nodes - 1 > len(full):
        raise ValueError("tree has fewer nodes than requested")
    full.sort(key=lambda t: (-t[0], t[1], t[2]))
    kept = {(): 0}
    chosen = [t[2] for t in full[: n_nodes - 1]]
    for p in chosen:                       # closure: a parent always outranks its child
        assert p[:-1] == () or p[:-1] in set(chosen)
    order = sorted(chosen, key=lambda p: (len(p), p))   # breadth-first, siblings by rank
    parent = np.full(n_nodes, -1, dtype=np.int32)
    rank = np.zeros(n_nodes, dtype=np.int32)
    for i, p in enumerate(order, start=1):
        kept[p] = i
    for p in order:
        parent[kept[p]] = kept[p[:-1]]
        rank[kept[p]] = p[-1]
    return parent, rank


def chain_tree(n: int) -> Tuple[np.ndarray, np.ndarray]:
    """A path: node i's parent is i-1.  Verifying it is plain decoding of n tokens."""
    parent = np.arange(-1, n - 1, dtype=np.int32)
    rank = np.zeros(n, dtype=np.int32)
    return parent, rank


def tree_for(shape: ModelShape) -> Tuple[np.ndarray, np.ndarray]:
    return make_tree(shape.tree_k, shape.tree_nodes)


# ----------------------------------------------------------------------------
# prompts
# ----------------------------------------------------------------------------
def make_prompts(shape: ModelShape, seed: int | None = None) -> List[np.ndarray]:
    """One int32 id array per sequence; lengths drawn first, then the ids."""
    rng = np.random.Generator(np.random.Philox(key=np.uint64(1000003 * (shape.seed if seed is None else seed) + 17)))
    lo, hi = shape.prompt_len
    lens = [int(rng.integers(lo, hi + 1)) for _ in range(shape.batch)]
    return [rng.integers(0, shape.vocab, size=n, dtype=np.int64).astype(np.int32) for n in lens]
