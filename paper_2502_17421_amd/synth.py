"""Seeded synthetic inputs shaped like the paper's long-context verification workloads.

This module only DRAWS inputs (random numbers, random trees, rounding of the
drawn values to the storage type).  It holds none of the method's arithmetic
and imports neither the GPU binding nor the CPU oracle, so both sides can be
fed from it.  numpy only.

Shapes follow Section 4.1 / Appendix "Experiments Details" of the paper:
prefixes of up to 32k tokens (64k for the long-reasoning shape), and a
speculation tree grown over at most five beam-search steps with beam widths
[4, 16, 16, 16, 16], i.e. a few tens of nodes, shallow and bushy.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str              # "bf16" | "f16" | "f32"
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_tree: int
    prefix_lo: int          # prefix length drawn uniformly in [prefix_lo, prefix_hi] per sequence
    prefix_hi: int
    max_depth: Optional[int]      # None: unconstrained uniform parents
    max_children: Optional[int]
    seed: int
    kind: str = "verify"    # "verify": hybrid tree attention; "cross": cached keys only; "accept": acceptance + KV commit

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


# The five benchmark shapes.
WORKLOADS = {
    "C1": Workload("C1", "f32", 1, 4, 1, 64, 16, 1024, 1024, None, None, 1001),
    "C2": Workload("C2", "bf16", 1, 32, 8, 128, 64, 8192, 8192, 8, 4, 1002),
    "C3": Workload("C3", "bf16", 1, 32, 8, 128, 64, 32768, 32768, 8, 4, 1003),
    "C4": Workload("C4", "bf16", 1, 32, 32, 128, 32, 16384, 16384, 6, None, 1004),
    "C5": Workload("C5", "bf16", 4, 40, 8, 128, 128, 16384, 65536, 10, 4, 1005),
    # Draft-side cross-attention over the target model's KV cache (Section 3.1): one drafting
    # step of beam width 16 resp. 4 (Appendix "Experiments Details") on the 8B-class GQA shape.
    "D1": Workload("D1", "bf16", 1, 32, 8, 128, 16, 32768, 32768, None, None, 1011, "cross"),
    "D2": Workload("D2", "bf16", 1, 32, 8, 128, 4, 32768, 32768, None, None, 1012, "cross"),
    # The draft model's own self-attention (Section 3.1): a sliding window of 512 cached rows plus
    # the tokens drafted so far (68 nodes after the five beam steps of the appendix).
    "W1": Workload("W1", "bf16", 1, 32, 8, 128, 68, 512, 512, 5, 16, 1041),
    # The headline shape with IEEE half inputs, the precision of the paper's own experiments.
    "H3": Workload("H3", "f16", 1, 32, 8, 128, 64, 32768, 32768, 8, 4, 1033),
    # The steps after the attention in a verification round (greedy acceptance + KV commit) on
    # the C3 and C5 shapes; "kind" accept.
    "A3": Workload("A3", "bf16", 1, 32, 8, 128, 64, 32768, 32768, 8, 4, 1023, "accept"),
    "A5": Workload("A5", "bf16", 4, 40, 8, 128, 128, 16384, 65536, 10, 4, 1025, "accept"),
    # The C3 shape under the paper's own tree: five beam steps of widths 4, 16, 16, 16, 16 (Appendix
    # "Experiments Details") = 68 nodes, 272 query rows per KV head: one full query block + 16 rows.
    "B3": Workload("B3", "bf16", 1, 32, 8, 128, 68, 32768, 32768, 5, 16, 1063),
    # The C3 shape under a speculation tree four times the size (256 nodes, 1024 query rows per
    # KV head): the regime of large static trees, bound by the matrix cores rather than by HBM.
    "L3": Workload("L3", "bf16", 1, 32, 8, 128, 256, 32768, 32768, 12, 4, 1053),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result is float32
    holding exactly representable bf16 values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    bias = ((u >> 16) & 1) + 0x7FFF
    r = ((u + bias) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(x.shape)


def round_to_f16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest IEEE half (ties to even); result is float32."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).astype(np.float32)


def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    """x rounded to the storage type named dtype ("bf16", "f16" or "f32"), held as float32."""
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "f16":
        return round_to_f16(x)
    return np.ascontiguousarray(x, dtype=np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    assert not np.any(u & 0xFFFF), "values are not bf16-representable"
    return (u >> 16).astype(np.uint16).reshape(x.shape)


# ---------------------------------------------------------------- trees ----

def tree_uniform(rng: np.random.Generator, n: int) -> np.ndarray:
    """parents[0] = -1, parents[i] uniform in [0, i)."""
    p = np.full(n, -1, dtype=np.int32)
    for i in range(1, n):
        p[i] = rng.integers(0, i)
    return p


def tree_constrained(rng: np.random.Generator, n: int, max_depth: Optional[int],
                     max_children: Optional[int]) -> np.ndarray:
    """Random tree in topological order: node i picks its parent uniformly among earlier
    nodes whose depth is below max_depth and that have fewer than max_children children.
    The root has depth 0."""
    p = np.full(n, -1, dtype=np.int32)
    depth = np.zeros(n, dtype=np.int64)
    kids = np.zeros(n, dtype=np.int64)
    for i in range(1, n):
        ok = np.ones(i, dtype=bool)
        if max_depth is not None:
            ok &= depth[:i] < max_depth
        if max_children is not None:
            ok &= kids[:i] < max_children
        cand = np.nonzero(ok)[0]
        if cand.size == 0:
            raise ValueError("tree constraints cannot hold this many nodes")
        j = int(cand[rng.integers(0, cand.size)])
        p[i] = j
        depth[i] = depth[j] + 1
        kids[j] += 1
    return p


def tree_chain(n: int) -> np.ndarray:
    return np.arange(-1, n - 1, dtype=np.int32)


def tree_star(n: int) -> np.ndarray:
    p = np.zeros(n, dtype=np.int32)
    p[0] = -1
    return p


def tree_beam(rng: np.random.Generator, widths=(4, 16, 16, 16, 16)) -> np.ndarray:
    """A root plus one level per beam step: every node of a level hangs under a random
    node of the level above (the paper's beam widths by default: 1 + 68 nodes)."""
    parents = [-1]
    prev = [0]
    for w in widths:
        cur = []
        for _ in range(w):
            parents.append(int(prev[rng.integers(0, len(prev))]))
            cur.append(len(parents) - 1)
        prev = cur
    return np.asarray(parents, dtype=np.int32)


def tree_depths(parents: np.ndarray) -> np.ndarray:
    d = np.zeros(len(parents), dtype=np.int64)
    for i, p in enumerate(parents):
        d[i] = 0 if p < 0 else d[p] + 1
    return d


# --------------------------------------------------------------- tensors ----

@dataclass
class Sequence:
    """One sequence's inputs, float32 arrays holding values exact in the storage dtype."""
    q: np.ndarray         # [Hq, T, D]
    k_cache: np.ndarray   # [Hkv, P, D]
    v_cache: np.ndarray   # [Hkv, P, D]
    k_tree: np.ndarray    # [Hkv, T, D]
    v_tree: np.ndarray    # [Hkv, T, D]
    parents: np.ndarray   # [T] int32
    prefix_len: int


@dataclass
class Batch:
    workload: Workload
    variant: str
    seqs: list = field(default_factory=list)

    @property
    def prefix_lens(self) -> np.ndarray:
        return np.asarray([s.prefix_len for s in self.seqs], dtype=np.int32)

    @property
    def max_prefix_len(self) -> int:
        return int(max(s.prefix_len for s in self.seqs))


def _normal(rng, shape, dtype):
    x = rng.standard_normal(shape, dtype=np.float32)
    return round_to(x, dtype)


def make_sequence(rng: np.random.Generator, *, dtype: str, n_q_heads: int, n_kv_heads: int,
                  head_dim: int, n_tree: int, prefix_len: int, parents: np.ndarray,
                  variant: str = "iid") -> Sequence:
    """Draw one sequence.

    variant "iid":   Q, K, V i.i.d. N(0,1) (the benchmark recipe).
    variant "peaked": as iid with Q multiplied by 6, so a few keys take most of the
                      weight and outputs are O(1) instead of an average of ~P rows.
    variant "tree":  as iid, but every tree key is replaced by 4x the mean query of its
                      KV group at that tree row, so tree keys out-weigh the prefix.
    """
    g = n_q_heads // n_kv_heads
    q = rng.standard_normal((n_q_heads, n_tree, head_dim), dtype=np.float32)
    if variant == "peaked":
        q = q * np.float32(6.0)
    k_cache = _normal(rng, (n_kv_heads, prefix_len, head_dim), dtype)
    v_cache = _normal(rng, (n_kv_heads, prefix_len, head_dim), dtype)
    k_tree = rng.standard_normal((n_kv_heads, n_tree, head_dim), dtype=np.float32)
    v_tree = _normal(rng, (n_kv_heads, n_tree, head_dim), dtype)
    if variant == "tree":
        k_tree = np.float32(4.0) * q.reshape(n_kv_heads, g, n_tree, head_dim).mean(axis=1)
    elif variant not in ("iid", "peaked"):
        raise ValueError(variant)
    q = round_to(q, dtype)
    k_tree = round_to(k_tree, dtype)
    return Sequence(q.astype(np.float32), k_cache, v_cache, k_tree.astype(np.float32), v_tree,
                    np.asarray(parents, dtype=np.int32), int(prefix_len))


def make_batch(w: Workload, variant: str = "iid", *, prefix_override: Optional[int] = None,
               n_tree_override: Optional[int] = None) -> Batch:
    """All sequences of a workload; sequence b uses seed w.seed + b.  The overrides shrink
    a workload for parity cases that the oracle must finish in seconds."""
    batch = Batch(w, variant)
    n_tree = n_tree_override or w.n_tree
    for b in range(w.batch):
        rng = np.random.default_rng(w.seed + b)
        if prefix_override is not None:
            plen = int(prefix_override)
        elif w.prefix_lo == w.prefix_hi:
            plen = w.prefix_lo
        else:
            plen = int(rng.integers(w.prefix_lo, w.prefix_hi + 1))
        if w.max_depth is None and w.max_children is None:
            parents = tree_uniform(rng, n_tree)
        else:
            parents = tree_constrained(rng, n_tree, w.max_depth, w.max_children)
        batch.seqs.append(make_sequence(rng, dtype=w.dtype, n_q_heads=w.n_q_heads,
                                        n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                                        n_tree=n_tree, prefix_len=plen, parents=parents,
                                        variant=variant))
    return batch


def make_tokens(rng: np.random.Generator, parents: np.ndarray, vocab: int = 32000, p_follow: float = 0.6):
    """Token ids for a verification round over a tree: (draft_tokens [T], target_tokens [T]).
    target_tokens[i] stands for the target model's prediction after node i and is drawn
    uniformly; a non-root node repeats its parent's prediction with probability p_follow
    (so accepted paths of several nodes occur) and is drawn uniformly otherwise."""
    t = len(parents)
    target = rng.integers(0, vocab, size=t).astype(np.int32)
    draft = rng.integers(0, vocab, size=t).astype(np.int32)
    for i in range(1, t):
        if parents[i] >= 0 and rng.random() < p_follow:
            draft[i] = target[parents[i]]
    return draft, target
