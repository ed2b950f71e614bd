"""Pins for the oracle's visibility mask (Section 4.1's ancestor rule on Section 5.3's DAG)."""
import numpy as np
import pytest

from paper_2407_16207_amd.workload import random_dag, layered_dag
from helpers import mask_to_bool, chain_dag, kary_tree, parents_of


def warshall_closure(n, offsets, parents):
    """Textbook reflexive-transitive closure of the parent relation (boolean Floyd-Warshall)."""
    reach = np.eye(n, dtype=bool)
    for i in range(n):
        for p in parents_of(offsets, parents, i):
            if p >= 0:
                reach[i, p] = True
    for m in range(n):
        for i in range(n):
            if reach[i, m]:
                reach[i] |= reach[m]
    return reach


@pytest.mark.parametrize("seed", range(12))
def test_closure_equals_warshall(ref, seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 90))
    off, par = random_dag(rng, n, max_parents=int(rng.integers(1, 5)))
    mask, flag = ref.build_mask([0, n], off, par)
    assert flag == 0
    assert np.array_equal(mask_to_bool(mask, n), warshall_closure(n, off, par))


def test_matrix_power_closure(ref):
    rng = np.random.default_rng(99)
    n = 40
    off, par = random_dag(rng, n, 3)
    a = np.eye(n, dtype=np.int64)
    for i in range(n):
        for p in parents_of(off, par, i):
            if p >= 0:
                a[i, p] = 1
    power = a.copy()
    for _ in range(7):                      # (I+A)^(2^7) covers any path of length < 128
        power = ((power @ power) > 0).astype(np.int64)
    mask, _ = ref.build_mask([0, n], off, par)
    assert np.array_equal(mask_to_bool(mask, n), power > 0)


def test_chain_is_lower_triangular(ref):
    n = 70
    off, par = chain_dag(n)
    mask, _ = ref.build_mask([0, n], off, par)
    assert mask.shape == (n, 2)
    assert np.array_equal(mask_to_bool(mask, n), np.tril(np.ones((n, n), dtype=bool)))


def test_tree_row_is_root_path(ref):
    off, par = kary_tree(3, 4)               # 3 + 9 + 27 + 81 nodes
    n = len(off) - 1
    assert n == (3 ** 5 - 1) // (3 - 1) - 1  # Section 4's node count, minus the virtual root
    mask, _ = ref.build_mask([0, n], off, par)
    vis = mask_to_bool(mask, n)
    for i in range(n):
        path = []
        x = i
        while x != -1:
            path.append(x)
            x = int(par[off[x]])
        expect = np.zeros(n, dtype=bool)
        expect[path] = True
        assert np.array_equal(vis[i], expect)
        assert vis[i].sum() == len(path)


def test_invariants_and_padding(ref):
    rng = np.random.default_rng(5)
    sizes = [70, 3, 129, 1]
    node_offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    offs, pars = [np.zeros(1, dtype=np.int32)], []
    e = 0
    for n in sizes:
        o, p = random_dag(rng, n, 3)
        offs.append(o[1:] + e)
        pars.append(p)
        e += len(p)
    parent_offsets = np.concatenate(offs).astype(np.int32)
    parent_idx = np.concatenate(pars)
    mask, flag = ref.build_mask(node_offsets, parent_offsets, parent_idx)
    assert flag == 0 and mask.shape == (sum(sizes), 3)
    for b, n in enumerate(sizes):
        base = node_offsets[b]
        vis = mask_to_bool(mask[base:base + n], 192)
        assert not vis[:, n:].any()                                  # bits beyond the sequence's nodes are zero
        for i in range(n):
            assert vis[i, i] and not vis[i, i + 1:].any()            # self bit, nothing later in topological order
            for p in parent_idx[parent_offsets[base + i]:parent_offsets[base + i + 1]]:
                if p >= 0:
                    assert not (vis[p] & ~vis[i]).any()              # a parent's set is contained in the child's


def test_layered_config_shape(ref):
    rng = np.random.default_rng(1)
    off, par = layered_dag(rng, 6, 8, 3)
    n = 48
    mask, _ = ref.build_mask([0, n], off.astype(np.int32), par)
    vis = mask_to_bool(mask, n)
    for i in range(n):
        layer = i // 8
        assert vis[i, :].sum() >= layer + 1                          # at least one ancestor per earlier layer
        assert not vis[i, layer * 8:(layer + 1) * 8][np.arange(8) != i % 8].any()   # no siblings


def test_bad_parent_sets_flag(ref):
    off = np.array([0, 1, 2, 3], dtype=np.int32)
    par = np.array([-1, 2, 0], dtype=np.int32)                        # node 1 names a later node
    mask, flag = ref.build_mask([0, 3], off, par)
    assert flag == 1
    assert np.array_equal(mask[:, 0], np.array([1, 2, 5], dtype=np.uint64))


def test_hand_worked_example(ref):
    """tests/golden/hand_dag6.txt: a 6-node graph whose rows were derived by hand from the ancestor rule."""
    import os
    from helpers import load_hand_dag
    g = load_hand_dag(os.path.join(os.path.dirname(__file__), "golden", "hand_dag6.txt"))
    n = g["n"]
    mask, _ = ref.build_mask([0, n], g["parent_offsets"], g["parent_idx"])
    vis = mask_to_bool(mask, n)
    for i in range(n):
        assert sorted(np.nonzero(vis[i])[0].tolist()) == g["visible"][i]
