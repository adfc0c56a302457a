"""Seeded synthetic inputs for the DSD verify step (data only, no method arithmetic).

This module serves both the CPU oracle's tests and the HIP path's tests/bench.  It
produces weights, KV caches, hidden states, draft noise and uniforms as plain numpy
arrays, with the shapes of the workloads the paper evaluates (Llama-3-8B / 70B style
decoder stages split over 4-8 nodes, draft window up to 8; paper section 3.1
"Experimental Setup").  Nothing here computes a norm, a projection, a softmax or an
acceptance test: those live in the oracle and in the HIP kernels, separately.

bf16 tensors are carried as uint16 bit patterns (numpy has no bf16 type).
"""
from __future__ import annotations

import zlib
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

# random streams (one per kind of input, so that changing one never shifts another)
STREAM_WEIGHTS = 0
STREAM_STATE = 1      # KV cache contents, hidden states, prompt token ids
STREAM_DRAFT = 2      # draft-logit noise, draft token draws
STREAM_UNIFORM = 3    # acceptance / resampling uniforms
STREAM_CALIB = 100    # calibration batch for the key-token thresholds


# --------------------------------------------------------------------------- bf16 bits
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round to nearest even); returns uint16 bit patterns."""
    u = np.array(x, dtype=np.float32, order="C", copy=True).view(np.uint32)
    lsb = u >> np.uint32(16)
    lsb &= np.uint32(1)
    u += np.uint32(0x7FFF)
    u += lsb
    del lsb
    # the high half of each little-endian 32-bit word is the bf16 pattern
    return np.ascontiguousarray(u.view(np.uint16).reshape(u.shape + (2,))[..., 1])


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def rng_for(seed: int, stream: int, name: str) -> np.random.Generator:
    """Counter-based generator keyed by (seed, stream, tensor name)."""
    ss = np.random.SeedSequence([int(seed), int(stream), zlib.crc32(name.encode())])
    return np.random.Generator(np.random.Philox(ss))


def normal(seed: int, stream: int, name: str, shape, std: float, mean: float = 0.0,
           dtype: str = "f32") -> np.ndarray:
    """N(mean, std^2) samples; dtype 'f32' -> float32, 'bf16' -> uint16 bit patterns."""
    g = rng_for(seed, stream, name)
    x = g.standard_normal(size=shape, dtype=np.float32)
    x *= np.float32(std)
    if mean != 0.0:
        x += np.float32(mean)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    return x


# --------------------------------------------------------------------------- configs
@dataclass(frozen=True)
class ModelCfg:
    name: str
    L: int
    d: int
    Hq: int
    Hkv: int
    hd: int
    F: int
    V: int            # 0 when the stage has neither embedding nor LM head
    dtype: str        # 'f32' | 'bf16' (weights, hidden states and KV cache)
    has_embed: bool
    has_head: bool
    rope_theta: float
    eps: float = 1e-5

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv


@dataclass(frozen=True)
class WorkCfg:
    name: str
    model: ModelCfg
    B: int
    C: int                      # committed context length per sequence
    k: int                      # drafted rows per sequence (tree: nodes)
    tree: bool = False
    adaptive: bool = False
    tau: float = 0.0
    top_m: int = 8
    temperature: float = 1.0
    seed: int = 0
    noise_std: float = 0.5      # draft logits = target logits + N(0, noise_std^2)


_M8B = dict(L=8, d=4096, Hq=32, Hkv=8, hd=128, F=14336, dtype="bf16", rope_theta=5e5)

MODELS = {
    "tiny": ModelCfg("tiny", L=2, d=256, Hq=4, Hkv=2, hd=64, F=688, V=4096, dtype="f32",
                     has_embed=True, has_head=True, rope_theta=1e4),
    "8b_mid": ModelCfg("8b_mid", V=0, has_embed=False, has_head=False, **_M8B),
    "8b_final": ModelCfg("8b_final", V=128256, has_embed=False, has_head=True, **_M8B),
    "70b_mid": ModelCfg("70b_mid", L=10, d=8192, Hq=64, Hkv=8, hd=128, F=28672, V=0, dtype="bf16",
                        has_embed=False, has_head=False, rope_theta=5e5),
}

CONFIGS = {
    "c1": WorkCfg("c1", MODELS["tiny"], B=1, C=128, k=4),
    "c2": WorkCfg("c2", MODELS["8b_mid"], B=1, C=2048, k=5),
    "c3": WorkCfg("c3", MODELS["8b_final"], B=16, C=4096, k=8, adaptive=True, tau=0.2),
    "c4": WorkCfg("c4", MODELS["70b_mid"], B=8, C=8192, k=6),
    "c5": WorkCfg("c5", MODELS["8b_final"], B=4, C=4096, k=32, tree=True, adaptive=True, tau=0.2),
}


def scaled(cfg: WorkCfg, **kw) -> WorkCfg:
    """A reduced copy of a workload (fewer layers, narrower, shorter context) for
    parity cases a CPU finishes in seconds.  Keys of ModelCfg go to the model."""
    mkeys = {k: kw.pop(k) for k in list(kw) if k in ModelCfg.__dataclass_fields__ and k != "name"}
    model = replace(cfg.model, **mkeys) if mkeys else cfg.model
    return replace(cfg, model=model, **kw)


# --------------------------------------------------------------------------- weights
def weight_specs(m: ModelCfg) -> List[Tuple[str, Tuple[int, ...], str]]:
    """(name, shape, kind) in the order the C ABI expects; kind 'w' = matrix, 'g' = gain.
    Matrices are [out_features, in_features], row-major."""
    out = []
    if m.has_embed:
        out.append(("embed", (m.V, m.d), "w"))
    for l in range(m.L):
        p = f"l{l}."
        out += [
            (p + "g1", (m.d,), "g"),
            (p + "wq", (m.Hq * m.hd, m.d), "w"),
            (p + "wk", (m.Hkv * m.hd, m.d), "w"),
            (p + "wv", (m.Hkv * m.hd, m.d), "w"),
            (p + "wo", (m.d, m.Hq * m.hd), "w"),
            (p + "g2", (m.d,), "g"),
            (p + "wg", (m.F, m.d), "w"),
            (p + "wu", (m.F, m.d), "w"),
            (p + "wd", (m.d, m.F), "w"),
        ]
    if m.has_head:
        out += [("gf", (m.d,), "g"), ("lm", (m.V, m.d), "w")]
    return out


def make_weight(m: ModelCfg, seed: int, name: str, shape, kind: str) -> np.ndarray:
    """Matrices N(0, 0.02^2); RMSNorm gains 1 + N(0, 0.02^2)."""
    return normal(seed, STREAM_WEIGHTS, name, shape, 0.02, 1.0 if kind == "g" else 0.0, m.dtype)


def make_weights(m: ModelCfg, seed: int = 0, threads: int = 8) -> Dict[str, np.ndarray]:
    specs = weight_specs(m)
    with ThreadPoolExecutor(max_workers=threads) as ex:
        arrs = list(ex.map(lambda s: make_weight(m, seed, *s), specs))
    return {s[0]: a for s, a in zip(specs, arrs)}


# --------------------------------------------------------------------------- state
def kv_std(m: ModelCfg) -> float:
    """Spread of a projection of a unit-RMS input through N(0, 0.02^2) weights."""
    return 0.02 * float(np.sqrt(m.d))


def make_kv(cfg: WorkCfg, threads: int = 8) -> Tuple[np.ndarray, np.ndarray]:
    """Random K (treated as already rotated) and V, [L, B, Hkv, C, hd] each."""
    m = cfg.model
    shape = (m.L, cfg.B, m.Hkv, cfg.C, m.hd)

    def one(which_l):
        which, l = which_l
        return normal(cfg.seed, STREAM_STATE, f"kv.{which}.{l}", shape[1:], kv_std(m), 0.0, m.dtype)

    jobs = [(w, l) for w in "kv" for l in range(m.L)]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        parts = list(ex.map(one, jobs))
    K = np.stack(parts[: m.L])
    V = np.stack(parts[m.L:])
    return K, V


def make_hidden(cfg: WorkCfg, rows: Optional[int] = None, tag: str = "hidden") -> np.ndarray:
    """N(0,1) input hidden states [B, rows, d] in the model dtype."""
    m = cfg.model
    rows = cfg.k if rows is None else rows
    return normal(cfg.seed, STREAM_STATE, tag, (cfg.B, rows, m.d), 1.0, 0.0, m.dtype)


def make_prompt_tokens(cfg: WorkCfg) -> np.ndarray:
    g = rng_for(cfg.seed, STREAM_STATE, "prompt")
    return g.integers(0, cfg.model.V, size=(cfg.B, cfg.C), dtype=np.int32)


def make_draft_noise(cfg: WorkCfg, rows: int, V: int, tag: str = "noise") -> np.ndarray:
    return normal(cfg.seed, STREAM_DRAFT, tag, (cfg.B, rows, V), cfg.noise_std, 0.0, "f32")


def make_uniforms(cfg: WorkCfg, rows: int, tag: str = "u", stream: int = STREAM_UNIFORM) -> np.ndarray:
    """U[0,1) float32, [B, rows]."""
    g = rng_for(cfg.seed, stream, tag)
    u = g.random(size=(cfg.B, rows), dtype=np.float32)
    return np.minimum(u, np.float32(1.0 - 2.0 ** -24))


def draw_categorical(prob_row: np.ndarray, u: float) -> int:
    """Index drawn from a probability row by walking its cumulative sum with one
    uniform (how the synthetic draft picks its tokens)."""
    c = np.cumsum(prob_row.astype(np.float64))
    i = int(np.searchsorted(c, u * c[-1], side="right"))
    return min(i, prob_row.shape[0] - 1)


# --------------------------------------------------------------------------- draft trees
def chain_parents(k: int) -> np.ndarray:
    """parent[i-1] for node i = 1..k of a chain: node i hangs under node i-1 (0 = root)."""
    return np.arange(0, k, dtype=np.int32)


def ranked_tree_parents(branching=(4, 3, 2, 2, 1, 1), n_nodes: int = 32) -> np.ndarray:
    """Token tree of the tree-draft workload: the full tree with the given per-depth
    branching is enumerated, every node is keyed by (sum of child ranks along its path,
    depth, path) and the n_nodes smallest are kept, which keeps the set ancestor-closed
    (a parent's key is never larger than its child's).  Nodes are numbered 1..n in
    (depth, path) order; returns parent ids (0 = root) for nodes 1..n."""
    paths = [()]
    allp = []
    for b in branching:
        nxt = [p + (r,) for p in paths for r in range(b)]
        allp += nxt
        paths = nxt
    allp.sort(key=lambda p: (sum(p), len(p), p))
    kept = sorted(allp[:n_nodes], key=lambda p: (len(p), p))
    ids = {(): 0}
    for i, p in enumerate(kept):
        ids[p] = i + 1
    return np.array([ids[p[:-1]] for p in kept], dtype=np.int32)


def tree_depths(parent: np.ndarray) -> np.ndarray:
    """depth[i-1] of node i, counted from 0 for children of the root."""
    k = len(parent)
    d = np.zeros(k, dtype=np.int32)
    for i in range(1, k + 1):
        p = int(parent[i - 1])
        d[i - 1] = 0 if p == 0 else d[p - 1] + 1
    return d


def tree_mask_bits(parent: np.ndarray) -> np.ndarray:
    """uint64 row t-1 has bit s-1 set when node s is node t or one of its ancestors."""
    k = len(parent)
    assert k <= 64
    bits = np.zeros(k, dtype=np.uint64)
    for i in range(1, k + 1):
        p = int(parent[i - 1])
        b = np.uint64(1) << np.uint64(i - 1)
        if p != 0:
            b |= bits[p - 1]
        bits[i - 1] = b
    return bits


def children_of(parent: np.ndarray) -> Dict[int, List[int]]:
    ch: Dict[int, List[int]] = {}
    for i in range(1, len(parent) + 1):
        ch.setdefault(int(parent[i - 1]), []).append(i)
    return ch
