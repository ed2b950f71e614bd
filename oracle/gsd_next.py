"""CPU oracle of the steps around the verify pass: un-merging the token graph into a token tree (Section 5.4),
committing the accepted path to the KV cache (the cache update of Section 7.1) and non-deterministic verification
(Sections 3 and 6.4).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module; the product path never
does.  Plain Python / numpy, written from the definitions; it shares nothing with the HIP path.
"""
from __future__ import annotations

import numpy as np

PATH_COUNT_CAP = 1 << 62      # reported path counts saturate here (the true count can be astronomically large)


def unmerge_to_tree(node_offsets, parent_offsets, parent_idx, max_tree_nodes):
    """Section 5.4: verification reverts the token graph to a tree by un-merging; the successors of a merged
    node are replicated once per way of reaching them.  The un-merged tree therefore has one node per ROOT PATH
    of the DAG (a path root -> v1 -> ... -> vm along parent edges); the tree parent of a path is the path without
    its last node; the tree node carries the token (and all per-node data) of the DAG node it ends at, its ORIGIN.

    Tree nodes are listed in this order (the definition of the output's numbering):
        paths are compared by the DAG id of their END node first; paths ending at the same node are compared by
        the position (slot) of their last edge in that node's stored parent list; paths that also share that
        parent are in the order of their parent paths.
    A parent path always precedes its extensions (the parent's end node has a smaller id), so the numbering is
    topological and any prefix of the list is a tree; a sequence's list is cut after `max_tree_nodes` entries.

    Returns (tree_node_offsets[B+1] int32, tree_parent[T'] int32 (sequence-local tree id, -1 = root),
             tree_origin[T'] int32 (sequence-local DAG id), path_count[B] int64 = min(#root paths, 2^62)).
    """
    node_offsets = np.asarray(node_offsets, dtype=np.int64)
    parent_offsets = np.asarray(parent_offsets, dtype=np.int64)
    parent_idx = np.asarray(parent_idx, dtype=np.int64)
    B = len(node_offsets) - 1
    offs = [0]
    all_parent, all_origin, counts = [], [], []
    for b in range(B):
        lo, hi = int(node_offsets[b]), int(node_offsets[b + 1])
        # replicas[i] = tree ids of the paths ending at DAG node i, in order (only those inside the cut are kept)
        replicas = [[] for _ in range(hi - lo)]
        n_paths = [0] * (hi - lo)                        # exact, unbounded Python integers
        tree_parent, tree_origin = [], []
        for i in range(hi - lo):
            for e in range(int(parent_offsets[lo + i]), int(parent_offsets[lo + i + 1])):
                p = int(parent_idx[e])
                if p == -1:
                    n_paths[i] += 1
                    parent_paths = [-1]
                else:
                    assert 0 <= p < i, "parents must be earlier nodes"
                    n_paths[i] += n_paths[p]
                    parent_paths = replicas[p]
                for t in parent_paths:
                    if len(tree_parent) < max_tree_nodes:
                        replicas[i].append(len(tree_parent))
                        tree_parent.append(t)
                        tree_origin.append(i)
        total = sum(n_paths)
        # a path inside the cut has its parent path inside the cut: nothing may be lost before the cut is reached
        assert len(tree_parent) == min(total, max_tree_nodes)
        counts.append(min(total, PATH_COUNT_CAP))
        all_parent.extend(tree_parent)
        all_origin.extend(tree_origin)
        offs.append(len(all_parent))
    return (np.asarray(offs, dtype=np.int32), np.asarray(all_parent, dtype=np.int32),
            np.asarray(all_origin, dtype=np.int32), np.asarray(counts, dtype=np.int64))


def commit_kv(k, v, kv_offsets, prefix_lens, accept_len, accept_path):
    """Cache update after acceptance (Section 7.1 attributes the "Others" time to it): the accepted tokens become
    part of the context, everything else drafted in this iteration is dropped.  With a sequence's rows laid out
    as [prefix rows ; draft rows], the new context of sequence b is
        old prefix rows, then the rows of accept_path[b][0 .. accept_len[b]) in path order.
    k, v: [L, R, ...] arrays (L layers, R rows, anything after); returns (new_k, new_v, new_prefix_lens) where
    rows beyond a sequence's new prefix keep their old contents (they are no longer part of anything)."""
    k = np.asarray(k)
    v = np.asarray(v)
    new_k, new_v = k.copy(), v.copy()
    new_len = np.asarray(prefix_lens, dtype=np.int32).copy()
    for b in range(len(prefix_lens)):
        base = int(kv_offsets[b]) + int(prefix_lens[b])
        for j in range(int(accept_len[b])):
            src = base + int(accept_path[b][j])
            new_k[:, base + j] = k[:, src]
            new_v[:, base + j] = v[:, src]
        new_len[b] += int(accept_len[b])
    return new_k, new_v, new_len


# ------------------------------------------------------------------------------------------ non-deterministic
def softmax_rows(logits):
    """Row-wise softmax in fp64 of stored (fp32 or bf16-bits) logits; returns (probabilities, row max, sum of exp)."""
    x = np.asarray(logits)
    if x.dtype == np.uint16:
        x = (x.astype(np.uint32) << np.uint32(16)).view(np.float32)
    x = x.astype(np.float64)
    m = x.max(axis=1, keepdims=True)
    e = np.exp(x - m)
    z = e.sum(axis=1, keepdims=True)
    return e / z, m[:, 0], z[:, 0]


def accept_stochastic(node_offsets, parent_offsets, parent_idx, tokens, p_nodes, p_root, draft_prob, accept_u,
                      q_nodes, q_root, resample_u, max_nodes=None):
    """Non-deterministic verification (Section 3; Section 6.4 gives no rule for several hypotheses, so the reading
    is stated here).  p_nodes[T, V] / p_root[B, V]: the LLM's next-token distribution after each node / after the
    context; q_nodes, q_root: the draft model's.  draft_prob[i]: the probability the draft model gave token i when
    it drafted node i; accept_u[i], resample_u[b]: uniforms in [0, 1).

      * an edge r -> i is accepted iff accept_u[i] < min(1, p_r(token_i) / draft_prob[i])   (one coin per node);
      * a root path is accepted iff all its edges are; the longest accepted root path is taken, with the
        deterministic rule's tie-breaks (smallest end node, then smallest qualifying parent);
      * the LLM then "regenerates" one token after the path's end r*: if r* has children in the graph (they were all
        rejected or not on a longer accepted path) it is drawn from the residual distribution max(p - q, 0) at r*,
        normalised (from p itself if the residual is empty), and from p if r* has no children; the draw is by
        inverse CDF: the smallest token x whose cumulative weight exceeds resample_u * total.

    Returns (accept_len[B], accept_path[B, max_nodes], bonus_token[B], edge_ok[E] bool, resid_cdf: list of [V] fp64)."""
    node_offsets = np.asarray(node_offsets, dtype=np.int64)
    parent_offsets = np.asarray(parent_offsets, dtype=np.int64)
    parent_idx = np.asarray(parent_idx, dtype=np.int64)
    B = len(node_offsets) - 1
    nmax = int(np.max(np.diff(node_offsets))) if B else 0
    max_nodes = max(1, nmax) if max_nodes is None else int(max_nodes)
    accept_len = np.zeros(B, dtype=np.int32)
    accept_path = np.full((B, max_nodes), -1, dtype=np.int32)
    bonus = np.zeros(B, dtype=np.int32)
    edge_ok = np.zeros(len(parent_idx), dtype=bool)
    cdfs = []
    for b in range(B):
        lo, hi = int(node_offsets[b]), int(node_offsets[b + 1])
        n = hi - lo
        L = [-1] * n
        back = [None] * n
        has_child = [False] * n
        root_has_child = False
        for i in range(n):
            tok = int(tokens[lo + i])
            for e in range(int(parent_offsets[lo + i]), int(parent_offsets[lo + i + 1])):
                r = int(parent_idx[e])
                if r < -1 or r >= i:
                    continue
                if r == -1:
                    root_has_child = True
                else:
                    has_child[r] = True
                p_tok = p_root[b, tok] if r == -1 else p_nodes[lo + r, tok]
                ok = accept_u[lo + i] < min(1.0, p_tok / draft_prob[lo + i])
                edge_ok[e] = ok
                lr = 0 if r == -1 else L[r]
                if ok and lr >= 0 and (lr + 1 > L[i] or (lr + 1 == L[i] and r < back[i])):
                    L[i] = lr + 1
                    back[i] = r
        best, end = 0, -1
        for i in range(n):
            if L[i] > best:
                best, end = L[i], i
        accept_len[b] = best
        v = end
        for pos in range(best - 1, -1, -1):
            accept_path[b, pos] = v
            v = back[v]
        p_end = p_root[b] if end == -1 else p_nodes[lo + end]
        q_end = q_root[b] if end == -1 else q_nodes[lo + end]
        rejected_some = root_has_child if end == -1 else has_child[end]
        w = np.maximum(p_end - q_end, 0.0) if rejected_some else p_end.copy()
        if w.sum() <= 0.0:
            w = p_end.copy()
        cdf = np.cumsum(w)
        cdfs.append(cdf)
        target = resample_u[b] * cdf[-1]
        x = int(np.searchsorted(cdf, target, side="right"))
        if x >= len(cdf):                       # target == total by rounding: the last token that carries weight
            x = int(np.flatnonzero(w > 0)[-1])
        bonus[b] = x
    return accept_len, accept_path, bonus, edge_ok, cdfs


# -------------------------------------------------------------------------------------- graph construction
def build_token_graph(node_offsets, tree_parent, tokens, draft_prob, tau, theta_prob, theta_sib):
    """Draft-side construction of the token graph (Sections 4.2, 5.2, 5.3) from what the draft model would produce:
    a token TREE per sequence (tree_parent[i] < i or -1, nodes in generation order = breadth first, so depths never
    decrease along the ids), the drafted token of every node and the probability the draft model gave it.  Nodes are
    visited in generation order:

      * a node exists in the graph only if its parent is the root or an existing node that was expanded;
      * probability pruning (Section 4.2): a node with draft_prob < theta_prob becomes a leaf;
      * sibling pruning (Section 4.2): a node with draft_prob < theta_sib * (largest draft_prob among the children of
        its parent, itself included) becomes a leaf;
      * redundancy (Section 5.2): a node of depth >= tau whose tau-gram (its token and those of its tau-1 nearest
        ancestors in the tree) equals the tau-gram of an EARLIER existing node is tau-redundant; the earliest such node
        is the first occurrence F.  The redundant node R becomes a leaf (Section 5.3);
      * merging (Section 5.3 draws an edge from R to F so that what follows F is reused below R): R becomes one more
        parent of every child of F, wherever F lies (its children may be generated later, if F is in R's own layer,
        or exist already, if F is in an earlier layer).  The one case the paper does not treat is an R that descends
        from F in the graph built so far (all parent edges, merge edges included): reusing F's children below R would
        close a cycle, so then no edge is drawn and R is only a leaf;
      * a node is expanded iff none of the three made it a leaf.

    An edge from a later layer into an earlier one breaks the generation order as a topological order, so the graph is
    renumbered: by level (0 for children of the root, else one more than the largest level among the parents), nodes
    of one level in generation order.  Without such edges this is the generation order itself.  Returns packed arrays
        (graph_node_offsets[B+1], parent_offsets[T'+1], parent_idx[E] (new sequence-local ids, ascending, -1 = root),
         origin[T'] (tree id), flags[T'] bit0 = probability-pruned, bit1 = sibling-pruned, bit2 = redundant,
         bit3 = redundant and a descendant of its first occurrence (no merge edge))."""
    node_offsets = np.asarray(node_offsets, dtype=np.int64)
    B = len(node_offsets) - 1
    g_off, p_off, p_idx, origin_all, flags_all = [0], [0], [], [], []
    for b in range(B):
        lo, hi = int(node_offsets[b]), int(node_offsets[b + 1])
        n = hi - lo
        par = [int(x) for x in tree_parent[lo:hi]]
        tok = [int(x) for x in tokens[lo:hi]]
        q = [float(x) for x in draft_prob[lo:hi]]
        exists = [False] * n
        expanded = [False] * n
        flags = [0] * n
        depth = [0] * n
        gram = [None] * n
        merged_into = {}                          # F -> [R, ...] in generation order
        # largest probability among the children of each parent (root = key -1): the children of a node exist all
        # together or not at all, so this does not depend on what is kept
        sib_max = {}
        for i in range(n):
            assert -1 <= par[i] < i
            sib_max[par[i]] = max(sib_max.get(par[i], 0.0), q[i])
            depth[i] = 1 if par[i] == -1 else depth[par[i]] + 1
            assert i == 0 or depth[i] >= depth[i - 1], "nodes must come in breadth-first order"

        def graph_parents(x):
            """Parents of existing node x in the graph built so far: its tree parent and whatever merged into it."""
            return [par[x]] + merged_into.get(par[x], [])

        def descends_from(x, f):
            seen, stack = set(), [x]
            while stack:
                for r in graph_parents(stack.pop()):
                    if r == f:
                        return True
                    if r != -1 and r not in seen:
                        seen.add(r)
                        stack.append(r)
            return False

        for i in range(n):
            p = par[i]
            if not (p == -1 or (exists[p] and expanded[p])):
                continue
            exists[i] = True
            # both thresholds are evaluated in fp32, the precision the probabilities come in
            if np.float32(q[i]) < np.float32(theta_prob):
                flags[i] |= 1
            if np.float32(q[i]) < np.float32(theta_sib) * np.float32(sib_max[p]):
                flags[i] |= 2
            if depth[i] >= tau:
                g, v = [], i
                for _ in range(tau):
                    g.append(tok[v])
                    v = par[v]
                gram[i] = tuple(g)
                for j in range(i):
                    if exists[j] and gram[j] == gram[i]:
                        flags[i] |= 4
                        if descends_from(i, j):
                            flags[i] |= 8
                        else:
                            merged_into.setdefault(j, []).append(i)
                        break
            expanded[i] = flags[i] == 0
        kept = [i for i in range(n) if exists[i]]
        level = {}
        for old in kept:                          # a parent that is a later node is a redundant leaf of a deeper layer,
            level[old] = None                     # whose own parents are earlier nodes: resolve on demand

        def level_of(x):
            if level[x] is None:
                level[x] = 0 if graph_parents(x) == [-1] else 1 + max(level_of(r) for r in graph_parents(x) if r != -1)
            return level[x]

        order = sorted(kept, key=lambda x: (level_of(x), x))
        new_id = {old: k for k, old in enumerate(order)}
        for old in order:
            ps = sorted(-1 if r == -1 else new_id[r] for r in graph_parents(old))
            assert all(r < new_id[old] for r in ps)
            p_idx.extend(ps)
            p_off.append(len(p_idx))
            origin_all.append(old)
            flags_all.append(flags[old])
        g_off.append(g_off[-1] + len(kept))
    return (np.asarray(g_off, dtype=np.int32), np.asarray(p_off, dtype=np.int32), np.asarray(p_idx, dtype=np.int32),
            np.asarray(origin_all, dtype=np.int32), np.asarray(flags_all, dtype=np.int32))
