"""Seeded synthetic verify-stage workloads (inputs only: no part of the method's arithmetic lives here).

The paper evaluates on real prompts and trained LLaMA/OPT/BLOOM weights (Section 6.1, Appendix A); none of
that is used.  These generators stand in for it with LLaMA-2-*shaped* tensors: a layered draft DAG per
sequence (the token graph of Section 5.3, nodes packed in topological order), draft tokens, Q/K/V ~ N(0,1)
and verifier logits ~ N(0,1) with a +5 "planted" bump on one child's token so that deterministic acceptance
(Section 3) is non-trivial.

Both the CPU oracle's tests and the GPU path's tests/benchmark draw their inputs from here, so that both see
identical bytes.  bf16 tensors are drawn in fp32, rounded to nearest-even once, and stored as uint16 bit
patterns; everything is numpy on the host.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

SEED_BASE = 20240716 * 10


@dataclass(frozen=True)
class VerifyConfig:
    """Shape of one synthetic verify step (one attention layer + the LM-head logits)."""

    name: str
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    prefix_min: int          # KV prefix length per sequence is uniform in [prefix_min, prefix_max]
    prefix_max: int
    layers: int              # DAG layers
    width: int               # nodes per layer
    max_parents: int         # parents per node uniform in 1..max_parents (drawn from the previous layer)
    vocab: int
    plant_p: float           # probability that a non-leaf node's logits get the +5 bump on a child's token
    dtype: str               # "f32" or "bf16"

    @property
    def nodes(self) -> int:
        return self.layers * self.width


CONFIGS = {
    1: VerifyConfig("cfg1-tiny-f32", 1, 4, 4, 64, 128, 128, 4, 4, 2, 1000, 0.7, "f32"),
    2: VerifyConfig("cfg2-llama2-7b-shaped", 1, 32, 32, 128, 1024, 1024, 8, 8, 2, 32000, 0.7, "bf16"),
    3: VerifyConfig("cfg3-llama2-13b-shaped", 4, 40, 40, 128, 2048, 2048, 16, 8, 3, 32000, 0.75, "bf16"),
    4: VerifyConfig("cfg4-llama2-70b-shaped-gqa", 8, 64, 8, 128, 4096, 4096, 32, 8, 3, 32000, 0.8, "bf16"),
    5: VerifyConfig("cfg5-70b-stress-ragged", 32, 64, 8, 128, 1024, 8192, 64, 8, 4, 32000, 0.8, "bf16"),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 bit patterns.  No NaN inputs expected."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Workload:
    cfg: VerifyConfig
    seed: int
    # DAG, CSR over packed nodes; parent ids are sequence-local, -1 = root (the context)
    node_offsets: np.ndarray          # [B+1] int32
    parent_offsets: np.ndarray        # [T+1] int32
    parent_idx: np.ndarray            # [E]   int32
    tokens: np.ndarray                # [T]   int32
    root_pred: np.ndarray             # [B]   int32
    prefix_lens: np.ndarray           # [B]   int32
    kv_offsets: np.ndarray            # [B]   int64  first K/V row of sequence b (prefix rows, then draft rows)
    q: np.ndarray                     # [T, Hq, D]      f32, or uint16 bf16 bits
    k: np.ndarray                     # [R, Hkv, D]     R = sum_b (P_b + N_b)
    v: np.ndarray                     # [R, Hkv, D]
    logits: np.ndarray                # [T, V]
    softmax_scale: float
    extras: dict = field(default_factory=dict)

    @property
    def total_nodes(self) -> int:
        return int(self.node_offsets[-1])

    @property
    def max_nodes(self) -> int:
        return int(np.max(np.diff(self.node_offsets))) if len(self.node_offsets) > 1 else 0

    @property
    def words_per_row(self) -> int:
        return max(1, (self.max_nodes + 63) // 64)


def layered_dag(rng: np.random.Generator, layers: int, width: int, max_parents: int, tree: bool = False):
    """One layered DAG: layer 0 hangs off the root; a node in layer l>0 draws 1..max_parents distinct parents
    from layer l-1 (sorted).  tree=True keeps only the first (smallest-id) parent of every node, drawing the
    same random numbers, so the tree is the DAG with its extra edges removed."""
    offsets = [0]
    parents: list[int] = []
    for layer in range(layers):
        for _ in range(width):
            if layer == 0:
                ps = [-1]
            else:
                cnt = int(rng.integers(1, max_parents + 1))
                cnt = min(cnt, width)
                ps = sorted(int(x) for x in rng.choice(width, size=cnt, replace=False) + (layer - 1) * width)
                if tree:
                    ps = ps[:1]
            parents.extend(ps)
            offsets.append(len(parents))
    return np.asarray(offsets, dtype=np.int64), np.asarray(parents, dtype=np.int32)


def children_lists(n: int, offsets: np.ndarray, parents: np.ndarray):
    """children[i] = sorted nodes having i as a parent; root_children = nodes with parent -1."""
    children = [[] for _ in range(n)]
    root_children = []
    for i in range(n):
        for p in parents[offsets[i]:offsets[i + 1]]:
            if p < 0:
                root_children.append(i)
            else:
                children[int(p)].append(i)
    return children, root_children


def _draw(rng: np.random.Generator, shape, dtype: str) -> np.ndarray:
    x = rng.standard_normal(shape, dtype=np.float32)
    return x if dtype == "f32" else f32_to_bf16_bits(x)


def make_workload(cfg_id: int | VerifyConfig, seed: int | None = None, tree: bool = False,
                  with_logits: bool = True, with_qkv: bool = True) -> Workload:
    """Build the seeded workload for one of the five configs (or a custom VerifyConfig).

    Independent child streams are used for {DAG, tokens, prefix lengths, QKV, logits}, so e.g. `tree=True`
    changes the DAG's edges only and leaves tokens, Q/K/V and the raw logits noise as they were (the planted
    bumps follow the edges that remain).
    """
    if isinstance(cfg_id, VerifyConfig):
        cfg = cfg_id
        base_seed = SEED_BASE if seed is None else seed
    else:
        cfg = CONFIGS[cfg_id]
        base_seed = SEED_BASE + cfg_id if seed is None else seed
    root = np.random.default_rng(base_seed)
    r_dag, r_tok, r_len, r_qkv, r_logit, r_plant = root.spawn(6)

    B, N, V = cfg.batch, cfg.nodes, cfg.vocab
    T = B * N
    node_offsets = (np.arange(B + 1, dtype=np.int64) * N).astype(np.int32)

    parent_offsets = [np.zeros(1, dtype=np.int64)]
    parent_chunks = []
    per_seq = []
    edge_base = 0
    for _ in range(B):
        off, par = layered_dag(r_dag, cfg.layers, cfg.width, cfg.max_parents, tree=tree)
        per_seq.append((off, par))
        parent_offsets.append(off[1:] + edge_base)
        parent_chunks.append(par)
        edge_base += len(par)
    parent_offsets = np.concatenate(parent_offsets).astype(np.int32)
    parent_idx = np.concatenate(parent_chunks).astype(np.int32)

    # draft tokens: uniform over the vocab, distinct within a layer (so sibling ties are rare)
    tokens = np.empty(T, dtype=np.int32)
    for b in range(B):
        for layer in range(cfg.layers):
            lo = b * N + layer * cfg.width
            tokens[lo:lo + cfg.width] = r_tok.choice(V, size=cfg.width, replace=False)

    if cfg.prefix_min == cfg.prefix_max:
        prefix_lens = np.full(B, cfg.prefix_min, dtype=np.int32)
    else:
        prefix_lens = r_len.integers(cfg.prefix_min, cfg.prefix_max + 1, size=B).astype(np.int32)
    rows_per_seq = prefix_lens.astype(np.int64) + N
    kv_offsets = np.concatenate([[0], np.cumsum(rows_per_seq)[:-1]]).astype(np.int64)
    R = int(rows_per_seq.sum())

    if with_qkv:
        q = _draw(r_qkv, (T, cfg.num_q_heads, cfg.head_dim), cfg.dtype)
        k = _draw(r_qkv, (R, cfg.num_kv_heads, cfg.head_dim), cfg.dtype)
        v = _draw(r_qkv, (R, cfg.num_kv_heads, cfg.head_dim), cfg.dtype)
    else:
        q = k = v = np.zeros((0,), dtype=np.float32)

    # verifier logits with planted acceptance
    root_pred = np.empty(B, dtype=np.int32)
    planted_child = np.full(T, -1, dtype=np.int32)      # which child (seq-local id) got the bump, -1 = none
    for b in range(B):
        off, par = per_seq[b]
        children, root_children = children_lists(N, off, par)
        if r_plant.random() < cfg.plant_p and root_children:
            root_pred[b] = tokens[b * N + int(r_plant.choice(root_children))]
        else:
            root_pred[b] = int(r_plant.integers(0, V))
        for i in range(N):
            u = r_plant.random()
            pick = int(r_plant.integers(0, 1 << 30))
            if children[i] and u < cfg.plant_p:
                planted_child[b * N + i] = children[i][pick % len(children[i])]

    if with_logits:
        logits = np.empty((T, V), dtype=np.float32 if cfg.dtype == "f32" else np.uint16)
        chunk = max(1, min(T, (1 << 26) // V))           # <= 256 MB of fp32 noise at a time
        for lo in range(0, T, chunk):
            hi = min(T, lo + chunk)
            x = r_logit.standard_normal((hi - lo, V), dtype=np.float32)
            for t in range(lo, hi):
                c = planted_child[t]
                if c >= 0:
                    b = t // N
                    x[t - lo, tokens[b * N + c]] += np.float32(5.0)
            logits[lo:hi] = x if cfg.dtype == "f32" else f32_to_bf16_bits(x)
    else:
        logits = np.zeros((0, V), dtype=np.float32)

    return Workload(cfg=cfg, seed=base_seed, node_offsets=node_offsets, parent_offsets=parent_offsets,
                    parent_idx=parent_idx, tokens=tokens, root_pred=root_pred, prefix_lens=prefix_lens,
                    kv_offsets=kv_offsets, q=q, k=k, v=v, logits=logits,
                    softmax_scale=float(1.0 / np.sqrt(cfg.head_dim)),
                    extras={"planted_child": planted_child, "tree": tree})


def random_dag(rng: np.random.Generator, n: int, max_parents: int = 3, p_root: float = 0.25):
    """A general (not layered) DAG in topological order for property tests: node i takes the root with
    probability p_root (always for i == 0) and/or up to max_parents distinct earlier nodes."""
    offsets = [0]
    parents: list[int] = []
    for i in range(n):
        ps: list[int] = []
        if i == 0 or rng.random() < p_root:
            ps.append(-1)
        if i > 0:
            cnt = int(rng.integers(0 if ps else 1, max_parents + 1))
            cnt = min(cnt, i)
            if cnt:
                ps.extend(sorted(int(x) for x in rng.choice(i, size=cnt, replace=False)))
        parents.extend(ps)
        offsets.append(len(parents))
    return np.asarray(offsets, dtype=np.int32), np.asarray(parents, dtype=np.int32)


def merged_tree_dag(rng: np.random.Generator, n: int, max_children: int = 3, n_merges: int = 4):
    """A token graph shaped like the paper's (Section 5.3): a random token tree of n nodes (every node hangs off
    the root or an earlier node that still has fewer than max_children children, so ids are topological), in
    which n_merges leaves R are then "merged" into an earlier-explored node F: R becomes an extra parent of every
    child of F, which is the edge the paper draws from a redundant node to the first occurrence of its n-gram.
    Returns CSR (offsets, parents) with each node's parents sorted; -1 = root."""
    parent = np.full(n, -1, dtype=np.int64)
    n_children = np.zeros(n + 1, dtype=np.int64)           # slot n counts the root's children
    for i in range(n):
        while True:
            p = int(rng.integers(-1, i))
            if n_children[p] < max_children or p == -1:
                break
        parent[i] = p
        n_children[p] += 1
    children = [[] for _ in range(n)]
    for i in range(n):
        if parent[i] >= 0:
            children[int(parent[i])].append(i)
    plists = [[int(parent[i])] for i in range(n)]
    leaves = [i for i in range(n) if not children[i]]
    inner = [i for i in range(n) if children[i]]
    used = set()
    for _ in range(n_merges):
        if not inner:
            break
        f = inner[int(rng.integers(0, len(inner)))]
        cand = [r for r in leaves if r < children[f][0] and r != f and r not in used]
        if not cand:
            continue
        r = cand[int(rng.integers(0, len(cand)))]
        used.add(r)
        for c in children[f]:
            plists[c].append(r)
    offsets = [0]
    flat: list[int] = []
    for i in range(n):
        flat.extend(sorted(set(plists[i])))
        offsets.append(len(flat))
    return np.asarray(offsets, dtype=np.int32), np.asarray(flat, dtype=np.int32)
