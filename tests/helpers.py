"""Small helpers shared by the tests (plain Python/numpy re-statements used as independent pins)."""
import itertools

import numpy as np


def mask_to_bool(mask: np.ndarray, n: int) -> np.ndarray:
    """[n_rows, W] uint64 -> [n_rows, n] bool, bit j of row i (LSB first)."""
    rows = mask.shape[0]
    out = np.zeros((rows, n), dtype=bool)
    for j in range(n):
        out[:, j] = (mask[:, j // 64] >> np.uint64(j % 64)) & np.uint64(1)
    return out


def parents_of(offsets, parents, i):
    return [int(p) for p in parents[offsets[i]:offsets[i + 1]]]


def all_root_paths(n, offsets, parents):
    """Every path root -> v1 -> ... -> vm (m >= 1) of a DAG given by parent lists, as tuples of node ids."""
    children = [[] for _ in range(n)]
    roots = []
    for i in range(n):
        for p in parents_of(offsets, parents, i):
            (roots if p == -1 else children[p]).append(i)
    paths = []

    def walk(path):
        paths.append(tuple(path))
        for c in children[path[-1]]:
            walk(path + [c])

    for r in roots:
        walk([r])
    return paths


def brute_force_accept(n, offsets, parents, tokens, pred, root_pred):
    """Longest accepted root path by enumeration; ties: smallest reversed id sequence."""
    best = ()
    for path in all_root_paths(n, offsets, parents):
        ok = tokens[path[0]] == root_pred and all(tokens[path[j]] == pred[path[j - 1]] for j in range(1, len(path)))
        if not ok:
            continue
        if len(path) > len(best) or (len(path) == len(best) and tuple(reversed(path)) < tuple(reversed(best))):
            best = path
    bonus = root_pred if not best else pred[best[-1]]
    return list(best), int(bonus)


def chain_dag(n):
    offsets = np.arange(n + 1, dtype=np.int32)
    parents = np.arange(-1, n - 1, dtype=np.int32)
    return offsets, parents


def kary_tree(k, depth):
    """Complete k-ary tree below a virtual root, breadth-first ids; `depth` levels of real nodes."""
    offsets = [0]
    parents = []
    level = [-1]
    nid = 0
    for _ in range(depth):
        nxt = []
        for p in level:
            for _ in range(k):
                parents.append(p)
                offsets.append(len(parents))
                nxt.append(nid)
                nid += 1
        level = nxt
    return np.asarray(offsets, dtype=np.int32), np.asarray(parents, dtype=np.int32)


def load_hand_dag(path):
    """Parse tests/golden/hand_dag6.txt-style fixtures: 'parents i: ..', 'visible i: ..', 'name: ints'."""
    out = {"parents": {}, "visible": {}}
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            key, val = line.split(":")
            vals = [int(x) for x in val.split()]
            parts = key.split()
            if len(parts) == 2:
                out[parts[0]][int(parts[1])] = vals
            else:
                out[parts[0]] = vals
    n = len(out["parents"])
    off, par = [0], []
    for i in range(n):
        par += out["parents"][i]
        off.append(len(par))
    out["n"] = n
    out["parent_offsets"] = np.asarray(off, dtype=np.int32)
    out["parent_idx"] = np.asarray(par, dtype=np.int32)
    return out
