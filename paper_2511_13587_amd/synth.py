"""Seeded synthetic inputs for the verify pass: model shapes, random-init weights, prefixes,
draft trees, draft distributions, drafted tokens, uniforms and the VQ-codebook neighbour table.

This module only *produces arrays*.  It holds none of the verification arithmetic (no transformer
forward, no CFG mix, no acceptance rule); the HIP path and the CPU checker both consume what it
returns, so that the two are compared on identical inputs.  Everything is NumPy on the host.

The workloads stand in for the paper's LlamaGen-XL / Lumina-mGPT-7B targets with MS-COCO captions and
LANTERN/EAGLE-2 drafters (Section 5, experimental setup), none of which can be loaded here: weights
are random-init, the caption prefix is a random dense tensor, and draft distributions are Gaussian
logits through a normalised exponential.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

import numpy as np

DTYPE_FP32 = 0
DTYPE_BF16 = 1

PREFIX_CLASS = 0   # prefix = class-id embeddings (a table of n_classes + 1 rows; last row = "null")
PREFIX_DENSE = 1   # prefix = dense [P, d] vectors handed in by the caller


@dataclass(frozen=True)
class Shape:
    """One workload: model shape + generation geometry + draft geometry."""
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    d_ff: int
    vocab: int
    logit_lo: int
    logit_hi: int
    grid_h: int
    grid_w: int
    prefix_len: int
    prefix_kind: int
    n_prompts: int
    n_nodes: int              # draft nodes per verify call (chain: K)
    tree_widths: Optional[Tuple[int, ...]]  # None = chain; else nodes per depth 1..D
    dtype: int
    cfg_scale: float
    n_classes: int = 1000
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    relax_k: int = 0
    relax_delta: float = 0.0
    draft_std: float = 2.0        # std of the "target-like" Gaussian draft logits
    draft_noise_std: float = 0.0  # std of the extra noise added on top
    seed: int = 0

    @property
    def d_head(self) -> int:
        return self.d_model // self.n_heads

    @property
    def v_eff(self) -> int:
        return self.logit_hi - self.logit_lo

    @property
    def n_rows(self) -> int:
        return 2 * self.n_prompts

    @property
    def grid(self) -> int:
        return self.grid_h * self.grid_w

    def replace(self, **kw) -> "Shape":
        return dataclasses.replace(self, **kw)


# The five workloads (tiny fp32 reference, LlamaGen-B shape, LlamaGen-XL shape with a 26-node tree,
# 7B shape with a masked 8192-id slice, XL stress with a 60-node tree and relaxed acceptance).
TINY = Shape("tiny", 2, 128, 4, 344, 1024, 0, 1024, 8, 8, 1, PREFIX_CLASS, 1, 4, None,
             DTYPE_FP32, 4.0, draft_std=2.0, seed=1001)
B_SHAPE = Shape("llamagen_b", 12, 768, 12, 2048, 16384, 0, 16384, 16, 16, 1, PREFIX_CLASS, 4, 5, None,
                DTYPE_BF16, 7.5, draft_std=3.0, draft_noise_std=1.0, seed=1002)
XL_TREE = Shape("llamagen_xl_tree26", 36, 1280, 20, 3456, 16384, 0, 16384, 24, 24, 120, PREFIX_DENSE,
                8, 26, (4, 6, 6, 4, 3, 3), DTYPE_BF16, 7.5, draft_std=3.0, draft_noise_std=1.0, seed=1003)
SEVEN_B = Shape("7b_slice", 32, 4096, 32, 11008, 65536, 4096, 4096 + 8192, 32, 32, 64, PREFIX_DENSE,
                2, 6, None, DTYPE_BF16, 7.5, draft_std=3.0, draft_noise_std=1.0, seed=1004)
XL_STRESS = Shape("llamagen_xl_tree60", 36, 1280, 20, 3456, 16384, 0, 16384, 24, 24, 120, PREFIX_DENSE,
                  32, 60, (8, 12, 12, 10, 8, 6, 4), DTYPE_BF16, 7.5, relax_k=50, relax_delta=0.2,
                  draft_std=3.0, draft_noise_std=1.0, seed=1005)

SHAPES: Dict[str, Shape] = {s.name: s for s in (TINY, B_SHAPE, XL_TREE, SEVEN_B, XL_STRESS)}


# ----------------------------------------------------------------------------- bf16 helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------- weights
def weight_names(shape: Shape) -> List[str]:
    """Canonical tensor order (this is also the order the library's weight loader expects)."""
    names = ["embed", "prefix_embed"]
    for l in range(shape.n_layers):
        names += [f"l{l}.{k}" for k in ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")]
    names += ["gf", "wout"]
    return names


def weight_dims(shape: Shape, name: str) -> Tuple[int, ...]:
    d, f, v = shape.d_model, shape.d_ff, shape.vocab
    if name == "embed":
        return (v, d)
    if name == "prefix_embed":
        return (shape.n_classes + 1, d)
    if name == "wout":
        return (d, v)
    key = name.split(".")[-1]
    return {"g1": (d,), "g2": (d,), "gf": (d,), "wq": (d, d), "wk": (d, d), "wv": (d, d), "wo": (d, d),
            "wg": (d, f), "wu": (d, f), "wd": (f, d)}[key]


def make_weights(shape: Shape, std: float = 0.02, gain_jitter: float = 0.0) -> Dict[str, np.ndarray]:
    """Random-init weights, float32 arrays.  Matrices are [in, out] (activations multiply from the
    left).  For bf16 shapes every value is already bf16-representable.  Norm gains are 1 (+ optional
    jitter so that a dropped gain is visible to tests)."""
    rng = np.random.default_rng(shape.seed)
    out: Dict[str, np.ndarray] = {}
    for name in weight_names(shape):
        dims = weight_dims(shape, name)
        if len(dims) == 1:
            w = np.ones(dims, dtype=np.float32)
            if gain_jitter:
                w = w + gain_jitter * rng.standard_normal(dims, dtype=np.float32)
        else:
            w = rng.standard_normal(dims, dtype=np.float32)
            w *= np.float32(std)
        if shape.dtype == DTYPE_BF16:
            w = bf16_bits_to_f32(f32_to_bf16_bits(w))
        out[name] = w
    return out


def make_drafter_weights(shape: Shape, target_weights: Dict[str, np.ndarray], std: float = 0.02,
                         gain_jitter: float = 0.0, seed_offset: int = 104729) -> Dict[str, np.ndarray]:
    """Random-init weights of a one-block drafter for `shape`: its own block (l0.*), final gain gf and
    input map fc [2 d, d]; the token embedding table, class table and output head are the target's
    (the same arrays).  float32, bf16-representable for bf16 shapes."""
    one = shape.replace(n_layers=1, seed=shape.seed + seed_offset)
    own = make_weights(one, std=std, gain_jitter=gain_jitter)
    out = {k: v for k, v in own.items() if k.startswith("l0.") or k == "gf"}
    for k in ("embed", "prefix_embed", "wout"):
        out[k] = target_weights[k]
    rng = np.random.default_rng(one.seed + 17)
    fc = rng.standard_normal((2 * shape.d_model, shape.d_model), dtype=np.float32) * np.float32(std * 8)
    if shape.dtype == DTYPE_BF16:
        fc = bf16_bits_to_f32(f32_to_bf16_bits(fc))
    out["fc"] = fc
    return out


def drafter_weight_names() -> List[str]:
    """Canonical tensor order of a drafter context: the one-layer list followed by fc."""
    return ["embed", "prefix_embed"] + [f"l0.{k}" for k in ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")] + ["gf", "wout", "fc"]


# ----------------------------------------------------------------------------- prefixes
def make_prefix(shape: Shape, seed_offset: int = 0):
    """Returns (cond, uncond).
    class kind : cond int32 [B, P] ids in [0, n_classes); uncond None (the null id is used).
    dense kind : cond float32 [B, P, d] (std 1, bf16-representable for bf16 shapes);
                 uncond float32 [P, d], one shared "null" prefix."""
    rng = np.random.default_rng(shape.seed + 7919 + seed_offset)
    B, P, d = shape.n_prompts, shape.prefix_len, shape.d_model
    if shape.prefix_kind == PREFIX_CLASS:
        return rng.integers(0, shape.n_classes, size=(B, P)).astype(np.int32), None
    cond = rng.standard_normal((B, P, d), dtype=np.float32)
    unc = rng.standard_normal((P, d), dtype=np.float32)
    if shape.dtype == DTYPE_BF16:
        cond = bf16_bits_to_f32(f32_to_bf16_bits(cond))
        unc = bf16_bits_to_f32(f32_to_bf16_bits(unc))
    return cond, unc


# ----------------------------------------------------------------------------- draft topology
def tree_parents(widths: Optional[Tuple[int, ...]], n_nodes: int, seed: int = 0) -> np.ndarray:
    """parent[j-1] = parent of node j (nodes 1..N, root 0), topological (parent index < child index).
    Chain when widths is None.  For a tree: widths[k] nodes at depth k+1; each node's parent is drawn
    among the nodes of the previous depth, the first of them always gets a child (so the depth is
    reached) and sibling groups are contiguous in node id."""
    if widths is None:
        return np.arange(0, n_nodes, dtype=np.int32)
    assert sum(widths) == n_nodes
    rng = np.random.default_rng(seed + 31337)
    parent: List[int] = []
    prev = [0]
    nxt = 1
    for w in widths:
        picks = sorted([prev[0]] + [prev[int(i)] for i in rng.integers(0, len(prev), size=w - 1)])
        cur = []
        for p in picks:
            parent.append(p)
            cur.append(nxt)
            nxt += 1
        prev = cur
    return np.asarray(parent, dtype=np.int32)


def ancestor_mask(parent: np.ndarray) -> np.ndarray:
    """uint8 [T, T]; mask[i, j] = 1 iff j is i or an ancestor of i (root = index 0)."""
    T = len(parent) + 1
    m = np.zeros((T, T), dtype=np.uint8)
    for i in range(T):
        j = i
        while True:
            m[i, j] = 1
            if j == 0:
                break
            j = int(parent[j - 1])
    return m


def node_depths(parent: np.ndarray) -> np.ndarray:
    T = len(parent) + 1
    dep = np.zeros(T, dtype=np.int32)
    for j in range(1, T):
        dep[j] = dep[int(parent[j - 1])] + 1
    return dep


# ----------------------------------------------------------------------------- draft distributions
def _normalised_exp(logits: np.ndarray) -> np.ndarray:
    z = logits - logits.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def make_draft(shape: Shape, parent: np.ndarray, call_index: int = 0,
               base_logits: Optional[np.ndarray] = None):
    """Draft distributions and drafted tokens for one verify call.

    Returns (q float32 [B, T, V_eff], tokens int32 [B, N]).  q[b, j] is the draft distribution over
    the children of node j: normalised exp of Gaussian logits (std draft_std) plus Gaussian noise
    (std draft_noise_std); `base_logits` [B, T, V_eff] replaces the first Gaussian when given (used
    for the "correlated draft" coverage cases).  Children of one parent are drawn from q[b, parent]
    without replacement, in node-id order, so sibling tokens are distinct.  Token ids are full
    vocabulary ids (logit_lo added)."""
    rng = np.random.default_rng(shape.seed + 104729 * (call_index + 1))
    B, N, V = shape.n_prompts, len(parent), shape.v_eff
    T = N + 1
    if base_logits is None:
        logits = rng.standard_normal((B, T, V), dtype=np.float32) * np.float32(shape.draft_std)
    else:
        logits = np.asarray(base_logits, dtype=np.float32).copy()
    if shape.draft_noise_std:
        logits += rng.standard_normal((B, T, V), dtype=np.float32) * np.float32(shape.draft_noise_std)
    q = _normalised_exp(logits.astype(np.float64)).astype(np.float32)
    tokens = np.zeros((B, N), dtype=np.int32)
    children: Dict[int, List[int]] = {}
    for j in range(1, T):
        children.setdefault(int(parent[j - 1]), []).append(j)
    for b in range(B):
        for p, kids in children.items():
            w = q[b, p].astype(np.float64)
            w /= w.sum()
            picks = rng.choice(V, size=len(kids), replace=False, p=w)
            for c, x in zip(kids, picks):
                tokens[b, c - 1] = shape.logit_lo + int(x)
    return q, tokens


def make_uniforms(shape: Shape, n_nodes: int, call_index: int = 0) -> np.ndarray:
    """float32 [B, T, 2] in [0, 1): [.., 0] drives the accept test of a node, [.., 1] the terminal
    sample taken at a node."""
    rng = np.random.default_rng(shape.seed + 1000003 * (call_index + 1))
    return rng.random((shape.n_prompts, n_nodes + 1, 2), dtype=np.float32)


def make_forced_tokens(shape: Shape, n_forced: int) -> np.ndarray:
    """int32 [B, n_forced] image tokens inside the allowed slice, used to bring the KV cache to a
    chosen length with real forward outputs."""
    rng = np.random.default_rng(shape.seed + 15485863)
    return rng.integers(shape.logit_lo, shape.logit_hi, size=(shape.n_prompts, n_forced)).astype(np.int32)


# ----------------------------------------------------------------------------- codebook neighbours
def make_codebook_embeddings(vocab: int, dim: int = 8, seed: int = 4242) -> np.ndarray:
    """float32 [vocab, dim]: the random unit-norm latent embeddings behind make_codebook_neighbours
    (same seed, same vectors), standing in for the VQ codebook of the image tokenizer."""
    rng = np.random.default_rng(seed)
    e = rng.standard_normal((vocab, dim))
    e /= np.linalg.norm(e, axis=1, keepdims=True)
    return e.astype(np.float32)


def make_codebook_neighbours(vocab: int, k: int, dim: int = 8, seed: int = 4242) -> np.ndarray:
    """int32 [vocab, k]: for every code, its k nearest other codes by cosine distance on random
    unit-norm `dim`-d embeddings, ascending distance, ties broken by the lower id."""
    rng = np.random.default_rng(seed)
    e = rng.standard_normal((vocab, dim))
    e /= np.linalg.norm(e, axis=1, keepdims=True)
    out = np.zeros((vocab, k), dtype=np.int32)
    step = 2048
    for s in range(0, vocab, step):
        sim = e[s:s + step] @ e.T
        for i in range(sim.shape[0]):
            sim[i, s + i] = -np.inf  # self excluded
        # stable sort on (-sim) keeps the lower id first among equal distances
        order = np.argsort(-sim, axis=1, kind="stable")[:, :k]
        out[s:s + step] = order.astype(np.int32)
    return out
