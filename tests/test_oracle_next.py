"""Pins for the oracle's un-merge-to-tree step (Section 5.4) and KV-cache commit (Section 7.1)."""
import numpy as np
import pytest

from oracle import gsd_next
from paper_2407_16207_amd.workload import merged_tree_dag, random_dag
from helpers import all_root_paths, brute_force_accept, chain_dag, kary_tree, mask_to_bool, parents_of


def unmerge_one(off, par, cap=1 << 20):
    n = len(off) - 1
    o, tp, to, cnt = gsd_next.unmerge_to_tree([0, n], off, par, cap)
    assert o[0] == 0 and o[1] == len(tp) == len(to)
    return tp, to, int(cnt[0])


def tree_paths(tp, to):
    """Root path (as DAG ids) of every tree node, following tree parents."""
    paths = []
    for t in range(len(tp)):
        p, cur = [], t
        while cur != -1:
            p.append(int(to[cur]))
            cur = int(tp[cur])
        paths.append(tuple(reversed(p)))
    return paths


def diamond_chain(k):
    """k diamonds in a row: node 0; then for each diamond two middle nodes and a join.  2^k root paths to the end."""
    off, par = [0, 1], [-1]
    last = 0
    for _ in range(k):
        a = len(off) - 1
        par += [last]; off.append(len(par))        # a
        par += [last]; off.append(len(par))        # a + 1
        par += [a, a + 1]; off.append(len(par))    # join
        last = a + 2
    return np.asarray(off, dtype=np.int32), np.asarray(par, dtype=np.int32)


# ------------------------------------------------------------------------------------------------ un-merge
def test_hand_diamond():
    # 0 <- root; 1, 2 <- 0; 3 <- {1, 2} (merged); 4 <- 3.  Un-merging replicates 3 and its successor 4.
    off = np.array([0, 1, 2, 3, 5, 6], dtype=np.int32)
    par = np.array([-1, 0, 0, 1, 2, 3], dtype=np.int32)
    tp, to, cnt = unmerge_one(off, par)
    assert cnt == 7
    assert to.tolist() == [0, 1, 2, 3, 3, 4, 4]
    assert tp.tolist() == [-1, 0, 0, 1, 2, 3, 4]


@pytest.mark.parametrize("shape", [("chain", 9), ("tree", (3, 3)), ("tree", (2, 5))])
def test_tree_is_left_unchanged(shape):
    off, par = chain_dag(shape[1]) if shape[0] == "chain" else kary_tree(*shape[1])
    tp, to, cnt = unmerge_one(off, par)
    n = len(off) - 1
    assert cnt == n and to.tolist() == list(range(n)) and tp.tolist() == par.tolist()


@pytest.mark.parametrize("seed", range(40))
def test_one_tree_node_per_root_path_in_the_defined_order(seed):
    rng = np.random.default_rng(500 + seed)
    n = int(rng.integers(1, 13))
    off, par = random_dag(rng, n, max_parents=3, p_root=0.3) if seed % 2 else merged_tree_dag(rng, n, 3, 3)
    tp, to, cnt = unmerge_one(off, par)
    got = tree_paths(tp, to)
    want = all_root_paths(n, off, par)                      # independent enumeration (walks child lists)
    assert len(got) == len(set(got)) == len(want) == cnt and set(got) == set(want)
    # count by linear algebra: c = r + A c  (A[i, p] = 1 per edge p -> i, r[i] = 1 per root edge)
    A = np.zeros((n, n))
    r = np.zeros(n)
    for i in range(n):
        for p in parents_of(off, par, i):
            if p == -1:
                r[i] += 1
            else:
                A[i, p] += 1
    assert cnt == int(round(np.linalg.solve(np.eye(n) - A, r).sum()))

    # order: end node, then slot of the last edge, then (recursively) the parent path
    def key(path):
        k = []
        for j in range(len(path) - 1, -1, -1):
            prev = path[j - 1] if j else -1
            k += [path[j], parents_of(off, par, path[j]).index(prev)]
        return k
    assert got == sorted(want, key=key)
    # parents come first, so every prefix is a tree
    assert all(tp[t] < t for t in range(len(tp)))


@pytest.mark.parametrize("seed", range(10))
def test_cut_keeps_a_prefix_and_reports_the_full_count(seed):
    rng = np.random.default_rng(900 + seed)
    off, par = random_dag(rng, 14, max_parents=3, p_root=0.2)
    tp, to, cnt = unmerge_one(off, par)
    for cap in (1, 5, cnt // 2 + 1, cnt, cnt + 3):
        tpc, toc, cntc = unmerge_one(off, par, cap)
        k = min(cap, cnt)
        assert cntc == cnt and tpc.tolist() == tp[:k].tolist() and toc.tolist() == to[:k].tolist()


def test_count_saturates():
    off, par = diamond_chain(70)                            # 2^70 paths end at the last join alone
    tp, to, cnt = unmerge_one(off, par, cap=300)
    assert cnt == 1 << 62 and len(tp) == 300
    off, par = diamond_chain(10)
    # 1 + sum_{d=1..10} (2^(d-1) + 2^(d-1) + 2^d) = 1 + 4*(2^10 - 1)
    assert unmerge_one(off, par, cap=16)[2] == 1 + 4 * (2 ** 10 - 1)


def test_several_sequences_are_independent():
    rng = np.random.default_rng(3)
    dags = [random_dag(rng, n, 3, 0.3) for n in (5, 1, 9)]
    node_offsets, poff, pidx = [0], [0], []
    for off, par in dags:
        node_offsets.append(node_offsets[-1] + len(off) - 1)
        poff += [int(x) + len(pidx) for x in off[1:]]
        pidx += par.tolist()
    o, tp, to, cnt = gsd_next.unmerge_to_tree(node_offsets, poff, pidx, 8)
    for b, (off, par) in enumerate(dags):
        tpb, tob, cntb = unmerge_one(off, par, 8)
        assert tp[o[b]:o[b + 1]].tolist() == tpb.tolist() and to[o[b]:o[b + 1]].tolist() == tob.tolist()
        assert cnt[b] == cntb


@pytest.mark.parametrize("seed", range(30))
def test_verifying_the_tree_accepts_the_same_path(ref, seed):
    """Acceptance depends only on tokens and predictions along a path, and the tree has exactly the DAG's root
    paths: the longest accepted path of the un-merged tree, mapped back through `origin`, is the DAG's."""
    rng = np.random.default_rng(7000 + seed)
    n = int(rng.integers(1, 15))
    off, par = random_dag(rng, n, max_parents=3, p_root=0.3)
    vocab = int(rng.integers(2, 5))
    tokens = rng.integers(0, vocab, n).astype(np.int32)
    pred = rng.integers(0, vocab, n).astype(np.int32)
    root_pred = int(rng.integers(0, vocab))
    tp, to, cnt = unmerge_one(off, par)
    m = len(tp)
    ln, path, bonus = ref.accept_longest_path([0, m], np.arange(m + 1), tp, tokens[to], pred[to], [root_pred])
    tree_path = [int(to[t]) for t in path[0, :ln[0]]]
    want_path, want_bonus = brute_force_accept(n, off, par, tokens, pred, root_pred)
    assert tree_path == want_path and int(bonus[0]) == want_bonus
    dl, dpath, dbonus = ref.accept_longest_path([0, n], off, par, tokens, pred, [root_pred])
    assert dpath[0, :dl[0]].tolist() == tree_path and dbonus[0] == bonus[0]


def test_tree_mask_rows_are_single_paths(ref):
    rng = np.random.default_rng(11)
    off, par = merged_tree_dag(rng, 40, 3, 5)
    tp, to, cnt = unmerge_one(off, par)
    m = len(tp)
    assert m > 40                                            # the merges did replicate something
    mask, flag = ref.build_mask([0, m], np.arange(m + 1), tp)
    vis = mask_to_bool(mask, m)
    paths = tree_paths(tp, to)
    for t in range(m):
        assert sorted(int(to[j]) for j in np.flatnonzero(vis[t])) == sorted(paths[t])
        assert vis[t].sum() == len(paths[t])


# ------------------------------------------------------------------------------------------------ KV commit
def make_cache(rng, layers, prefix_lens, n_draft, width=6):
    rows = int(sum(p + n_draft for p in prefix_lens))
    kv_offsets = np.concatenate([[0], np.cumsum([p + n_draft for p in prefix_lens])[:-1]]).astype(np.int64)
    k = rng.integers(0, 1 << 16, size=(layers, rows, width)).astype(np.uint16)
    v = rng.integers(0, 1 << 16, size=(layers, rows, width)).astype(np.uint16)
    return k, v, kv_offsets


def test_commit_equals_appending_only_the_accepted_tokens():
    rng = np.random.default_rng(5)
    prefix_lens = np.array([7, 0, 3], dtype=np.int32)
    n_draft = 10
    k, v, kv_offsets = make_cache(rng, 3, prefix_lens, n_draft)
    accept_len = np.array([4, 0, 10], dtype=np.int32)
    accept_path = np.full((3, n_draft), -1, dtype=np.int32)
    accept_path[0, :4] = [1, 2, 3, 9]                       # row j is overwritten while row path[j'] = j is a source
    accept_path[2, :] = np.arange(10)                       # a fully accepted chain: nothing moves
    nk, nv, nl = gsd_next.commit_kv(k, v, kv_offsets, prefix_lens, accept_len, accept_path)
    assert nl.tolist() == [11, 0, 13]
    for b in range(3):
        base = int(kv_offsets[b])
        P = int(prefix_lens[b])
        for old, new in ((k, nk), (v, nv)):
            ctx = np.concatenate([old[:, base:base + P]] +
                                 [old[:, base + P + a:base + P + a + 1] for a in accept_path[b, :accept_len[b]]], axis=1)
            assert np.array_equal(new[:, base:base + nl[b]], ctx)
            # rows past the new context are untouched
            assert np.array_equal(new[:, base + nl[b]:base + P + n_draft], old[:, base + nl[b]:base + P + n_draft])
    assert np.array_equal(nk[:, kv_offsets[1]:kv_offsets[2]], k[:, kv_offsets[1]:kv_offsets[2]])
    assert np.array_equal(nk[:, kv_offsets[2]:], k[:, kv_offsets[2]:])      # identity path: no change at all


# ----------------------------------------------------------------------------------- non-deterministic verify
def tiny_problem(rng, n, vocab, peaked=False):
    off, par = random_dag(rng, n, max_parents=2, p_root=0.3)
    tokens = rng.integers(0, vocab, n).astype(np.int32)
    lp = rng.standard_normal((n + 1, vocab)) * (8.0 if peaked else 1.0)
    lq = rng.standard_normal((n + 1, vocab))
    p, _, _ = gsd_next.softmax_rows(lp.astype(np.float32))
    q, _, _ = gsd_next.softmax_rows(lq.astype(np.float32))
    return off, par, tokens, p, q


def run_stochastic(off, par, tokens, p, q, draft_prob, u, w):
    n = len(off) - 1
    return gsd_next.accept_stochastic([0, n], off, par, tokens, p[:n], p[n:], draft_prob, u, q[:n], q[n:], [w])


def test_softmax_rows_is_the_library_softmax():
    import torch
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 37)).astype(np.float32) * 3
    p, m, z = gsd_next.softmax_rows(x)
    want = torch.softmax(torch.from_numpy(x).double(), dim=1).numpy()
    assert np.abs(p - want).max() < 1e-15
    assert np.allclose(m, x.max(axis=1)) and np.allclose(np.log(z) + m, torch.logsumexp(torch.from_numpy(x).double(), 1).numpy())


@pytest.mark.parametrize("seed", range(20))
def test_limits_of_the_acceptance_test(ref, seed):
    rng = np.random.default_rng(4000 + seed)
    n, vocab = int(rng.integers(1, 14)), 5
    off, par, tokens, p, q = tiny_problem(rng, n, vocab)
    u = rng.random(n)
    # a draft that never over-estimates (draft_prob <= every p it is compared with): every edge passes, the longest
    # root path of the graph is accepted
    ln, path, _, ok, _ = run_stochastic(off, par, tokens, p, q, np.full(n, 1e-9), u, 0.5)
    assert ok[[e for i in range(n) for e in range(off[i], off[i + 1])]].all()
    depth = max(len(pth) for pth in all_root_paths(n, off, par))
    assert ln[0] == depth
    # coins at 1 - eps against a draft that is always over-confident: nothing passes
    ln, path, bonus, ok, _ = run_stochastic(off, par, tokens, p * 0.5, q, np.ones(n), np.full(n, 0.999), 0.5)
    assert ln[0] == 0 and (path == -1).all() and not ok.any()
    # a (nearly) one-hot LLM against a draft that was certain: the test degenerates to "token == the LLM's token",
    # i.e. to deterministic verification
    lp = np.full((n + 1, vocab), -60.0)
    pred = rng.integers(0, vocab, n + 1)
    lp[np.arange(n + 1), pred] = 0.0
    p1, _, _ = gsd_next.softmax_rows(lp.astype(np.float32))
    ln, path, bonus, _, _ = run_stochastic(off, par, tokens, p1, p1 * 0, np.ones(n), u * 0.999, 0.3)
    dl, dpath, dbonus = ref.accept_longest_path([0, n], off, par, tokens, pred[:n].astype(np.int32), [int(pred[n])])
    assert ln[0] == dl[0] and np.array_equal(path[0, :ln[0]], dpath[0, :dl[0]])
    assert bonus[0] == dbonus[0]            # q = 0: the residual is p itself, whose mass sits on the LLM's token


def test_hand_example_chain_of_two():
    # root -> 0 -> 1, vocabulary {0,1,2}
    off, par = chain_dag(2)
    tokens = np.array([1, 2], dtype=np.int32)
    p = np.array([[0.2, 0.3, 0.5],      # after node 0
                  [0.1, 0.1, 0.8],      # after node 1
                  [0.6, 0.3, 0.1]])     # after the context
    q = np.array([[0.1, 0.1, 0.8],
                  [0.3, 0.3, 0.4],
                  [0.2, 0.6, 0.2]])
    draft_prob = np.array([0.6, 0.8])   # q_root(1), q_0(2)
    # edge root->0: ratio 0.3/0.6 = 0.5; edge 0->1: 0.5/0.8 = 0.625
    ln, path, bonus, ok, cdfs = run_stochastic(off, par, tokens, p, q, draft_prob, np.array([0.49, 0.7]), 0.5)
    assert ok.tolist() == [True, False] and ln[0] == 1 and path[0, 0] == 0
    # rejection after node 0: residual max(p0 - q0, 0) = [0.1, 0.2, 0] -> cdf [0.1, 0.3, 0.3]; 0.5 * 0.3 = 0.15 -> token 1
    assert np.allclose(cdfs[0], [0.1, 0.3, 0.3]) and bonus[0] == 1
    ln, path, bonus, ok, cdfs = run_stochastic(off, par, tokens, p, q, draft_prob, np.array([0.51, 0.1]), 0.9)
    # first edge rejected: everything after it is discarded; residual at the root max(p - q, 0) = [0.4, 0, 0] -> token 0
    assert ln[0] == 0 and bonus[0] == 0
    ln, path, bonus, ok, cdfs = run_stochastic(off, par, tokens, p, q, draft_prob, np.array([0.1, 0.1]), 0.15)
    # both accepted; node 1 is a leaf: the next token is drawn from p_1 = [0.1, 0.1, 0.8]: 0.15 -> token 1
    assert ln[0] == 2 and path[0, :2].tolist() == [0, 1] and bonus[0] == 1


def test_first_emitted_token_is_distributed_as_the_llm_says():
    """The classic guarantee of speculative sampling (the reason for the min(1, p/q) test and the residual draw): with
    the drafted token SAMPLED from q, the token emitted at that position is distributed exactly as p."""
    rng = np.random.default_rng(12)
    vocab, trials = 4, 40000
    p = np.array([[0.1, 0.2, 0.3, 0.4], [0.25, 0.25, 0.25, 0.25]])      # row 0: after node 0 (unused), row 1: after the context
    q = np.array([[0.25, 0.25, 0.25, 0.25], [0.55, 0.05, 0.3, 0.1]])
    off, par = chain_dag(1)
    counts = np.zeros(vocab)
    for _ in range(trials):
        tok = int(rng.choice(vocab, p=q[1]))
        ln, path, bonus, _, _ = gsd_next.accept_stochastic([0, 1], off, par, np.array([tok]), p[:1], p[1:], np.array([q[1, tok]]),
                                                           rng.random(1), q[:1], q[1:], rng.random(1))
        counts[tok if ln[0] == 1 else bonus[0]] += 1
    assert np.abs(counts / trials - p[1]).max() < 4 * np.sqrt(0.25 / trials)     # four standard errors


# -------------------------------------------------------------------------------------- graph construction
def random_token_tree(rng, n, k, vocab):
    """Breadth-first token tree: every node gets up to k children while ids last; tokens from a small vocabulary so
    that n-grams do re-occur; draft probabilities decreasing among siblings."""
    par, tok, q = [], [], []
    frontier, nxt = [-1], []
    while len(par) < n:
        for p in frontier:
            kids = int(rng.integers(1, k + 1))
            probs = np.sort(rng.dirichlet(np.ones(kids + 1))[:kids])[::-1]
            for c in range(kids):
                if len(par) >= n:
                    break
                par.append(p); tok.append(int(rng.integers(0, vocab))); q.append(float(probs[c]))
                nxt.append(len(par) - 1)
        frontier, nxt = nxt, []
        if not frontier:
            break
    return np.asarray(par, dtype=np.int32), np.asarray(tok, dtype=np.int32), np.asarray(q, dtype=np.float32)


def graph_one(par, tok, q, tau, tp, ts):
    n = len(par)
    g_off, p_off, p_idx, origin, flags = gsd_next.build_token_graph([0, n], par, tok, q, tau, tp, ts)
    assert g_off.tolist() == [0, len(origin)]
    return p_off, p_idx, origin, flags


def test_graph_without_pruning_or_merging_is_the_tree():
    rng = np.random.default_rng(1)
    par, tok, q = random_token_tree(rng, 60, 3, 50)
    p_off, p_idx, origin, flags = graph_one(par, tok, q, 99, 0.0, 0.0)
    assert origin.tolist() == list(range(60)) and p_idx.tolist() == par.tolist() and not flags.any()
    assert p_off.tolist() == list(range(61))


@pytest.mark.parametrize("seed", range(15))
def test_pruning_keeps_exactly_the_nodes_below_unpruned_ancestors(seed):
    rng = np.random.default_rng(50 + seed)
    par, tok, q = random_token_tree(rng, 80, 3, 1000)
    tp, ts = 0.15, 0.5
    p_off, p_idx, origin, flags = graph_one(par, tok, q, 99, tp, ts)
    sib_max = {}
    for i, p in enumerate(par):
        sib_max[int(p)] = max(sib_max.get(int(p), 0.0), float(q[i]))
    leaf = [bool(q[i] < tp or q[i] < ts * sib_max[int(par[i])]) for i in range(len(par))]
    want = []
    for i in range(len(par)):
        v, ok = int(par[i]), True
        while v != -1:
            ok &= not leaf[v]
            v = int(par[v])
        if ok:
            want.append(i)
    assert sorted(origin.tolist()) == want
    for k, old in enumerate(origin):
        assert bool(flags[k] & 1) == bool(q[old] < tp) and bool(flags[k] & 2) == bool(q[old] < ts * sib_max[int(par[old])])
    # a tree stays a tree, parents keep their tokens' order
    new_id = {int(o): k for k, o in enumerate(origin)}
    assert all(p_idx[k] == (-1 if par[o] == -1 else new_id[int(par[o])]) for k, o in enumerate(origin))


@pytest.mark.parametrize("seed", range(25))
def test_merged_graph_spells_exactly_the_hypotheses_of_the_definition(seed):
    """Independent statement of what merging means: a hypothesis continues below a redundant node with whatever
    follows the first occurrence of its tau-gram.  The token sequences along the root paths of the built graph must be
    exactly those, and among expanded nodes no tau-gram occurs twice."""
    rng = np.random.default_rng(300 + seed)
    tau = int(rng.integers(1, 4))
    par, tok, q = random_token_tree(rng, int(rng.integers(5, 40)), 3, int(rng.integers(2, 6)))
    n = len(par)
    p_off, p_idx, origin, flags = graph_one(par, tok, q, tau, 0.0, 0.0)
    m = len(origin)
    # hypotheses spelled by the graph: un-merge it and read the tokens along every tree path
    o, tpar, torg, cnt = gsd_next.unmerge_to_tree([0, m], p_off, p_idx, 200000)
    assert cnt[0] < 200000
    spelled = set()
    for t in range(len(tpar)):
        seq, v = [], t
        while v != -1:
            seq.append(int(tok[origin[torg[v]]]))
            v = int(tpar[v])
        spelled.add(tuple(reversed(seq)))
    # the same from the definition, on the tree: replay the construction with plain sets
    kids = {}
    for i, p in enumerate(par):
        kids.setdefault(int(p), []).append(i)
    first_seen, exists, follows = {}, set(), {}

    def continuations(v):                                  # the nodes a hypothesis can go to after v, so far
        src = follows.get(v)
        return [] if src is None else [c for c in kids.get(src, []) if c in exists]

    def hypothesis_passes(f, r):                           # some hypothesis built so far visits f and later r
        seen, todo = {f}, [f]
        while todo:
            for c in continuations(todo.pop()):
                if c == r:
                    return True
                if c not in seen:
                    seen.add(c)
                    todo.append(c)
        return False

    for i in range(n):
        p = int(par[i])
        if p != -1 and (p not in exists or follows[p] != p):
            continue                                      # parent missing or a leaf
        exists.add(i)
        g, v = [], i
        while v != -1 and len(g) < tau:
            g.append(int(tok[v])); v = int(par[v])
        follows[i] = i                                     # continues with its own children
        if len(g) == tau:
            key = tuple(g)
            if key in first_seen:
                f = first_seen[key]
                # Section 5.3: a leaf that continues with whatever follows the first occurrence f, wherever f lies;
                # unless the hypotheses through f already run into i (then reuse would loop: a leaf only)
                follows[i] = None
                if not hypothesis_passes(f, i):
                    follows[i] = f
            else:
                first_seen[key] = i
    want = set()

    def walk(v, prefix):
        prefix = prefix + (int(tok[v]),)
        want.add(prefix)
        src = follows[v]
        if src is None:
            return
        for c in kids.get(src, []):
            if c in exists:
                walk(c, prefix)
    for r in kids.get(-1, []):
        walk(r, ())
    assert spelled == want
    grams = {}
    for k, old in enumerate(origin):
        if flags[k] == 0:
            g, v = [], int(old)
            while v != -1 and len(g) < tau:
                g.append(int(tok[v])); v = int(par[v])
            if len(g) == tau:
                assert tuple(g) not in grams
                grams[tuple(g)] = old
    # numbering: parents first; by level (longest distance from the root), nodes of one level in generation order
    level = []
    for k in range(m):
        ps = [int(r) for r in p_idx[p_off[k]:p_off[k + 1]]]
        assert all(r < k for r in ps) and ps == sorted(ps)
        level.append(0 if ps == [-1] else 1 + max(level[r] for r in ps if r != -1))
    keys = [(level[k], int(origin[k])) for k in range(m)]
    assert keys == sorted(keys)
    # a redundant node is a leaf; bit 3 marks exactly those whose first occurrence leads to them
    for k, old in enumerate(origin):
        if flags[k] & 4:
            assert follows[int(old)] != int(old)
            assert bool(flags[k] & 8) == (follows[int(old)] is None)


def test_sibling_pruning_and_merge_hand_example():
    # root -> 0 (A, .6), 1 (B, .3), 2 (C, .05);  0 -> 3 (X, .9);  1 -> 4 (X, .8);  3 -> 5 (Y, .7);  4 -> 6 (Y, .6)
    par = np.array([-1, -1, -1, 0, 1, 3, 4], dtype=np.int32)
    tok = np.array([10, 11, 12, 20, 20, 30, 30], dtype=np.int32)
    q = np.array([.6, .3, .05, .9, .8, .7, .6], dtype=np.float32)
    p_off, p_idx, origin, flags = graph_one(par, tok, q, 1, 0.1, 0.4)
    # node 2: below theta_prob (0.05 < 0.1) and below 0.4 * 0.6 -> both pruning flags; node 1: 0.3 >= 0.24 stays
    # tau = 1: node 4 repeats token X (first at 3) -> redundant leaf merged into 3; its child 6 is never generated;
    # node 5 (child of 3) gets 4 as second parent and therefore moves behind it
    assert origin.tolist() == [0, 1, 2, 3, 4, 5]
    assert flags.tolist() == [0, 0, 3, 0, 4, 0]
    assert p_off.tolist() == [0, 1, 2, 3, 4, 5, 7] and p_idx.tolist() == [-1, -1, -1, 0, 1, 3, 4]


def test_cross_depth_merge_hand_example():
    """tests/golden/hand_merge8.txt: a same-layer merge, a refused (cyclic) one and a merge into an earlier layer that
    forces the renumbering; worked out by hand from Section 5.3."""
    import os
    from helpers import load_hand_dag
    h = load_hand_dag(os.path.join(os.path.dirname(__file__), "golden", "hand_merge8.txt"))
    par = np.asarray(h["tree_parent"], dtype=np.int32)
    tok = np.asarray(h["tokens"], dtype=np.int32)
    q = np.full(len(par), 0.5, dtype=np.float32)
    p_off, p_idx, origin, flags = graph_one(par, tok, q, h["tau"][0], 0.0, 0.0)
    assert origin.tolist() == h["origin"]
    assert flags.tolist() == h["flags"]
    assert p_off.tolist() == h["parent_offsets"].tolist() and p_idx.tolist() == h["parent_idx"].tolist()
    # and the hypotheses listed in the fixture's last line
    o, tpar, torg, cnt = gsd_next.unmerge_to_tree([0, len(origin)], p_off, p_idx, 1000)
    spelled = set()
    for t in range(len(tpar)):
        seq, v = "", t
        while v != -1:
            seq = chr(int(tok[origin[torg[v]]])) + seq
            v = int(tpar[v])
        spelled.add(seq)
    assert spelled == set("A B AB AC BA BD ABA ABD ACE BDC ABDC BDCE ABDCE".split())


def test_pruning_thresholds_are_strict_and_compared_in_fp32():
    """The library takes its thresholds as fp32 and the probabilities come as fp32: a probability exactly at the
    (fp32) threshold stays, the next fp32 number below it is pruned; likewise for the sibling rule, whose threshold is
    the fp32 product theta_sib * max."""
    theta_p, theta_s = 0.2, 0.3
    at_p = np.float32(theta_p)
    below_p = np.nextafter(at_p, np.float32(0))
    big = np.float32(0.9)
    at_s = np.float32(theta_s) * big
    below_s = np.nextafter(at_s, np.float32(0))
    assert float(at_p) > theta_p and float(at_s) != theta_s * float(big)      # fp64 would decide differently somewhere
    # root -> 0 (big), 1 (exactly theta_s*big), 2 (just below it), 3 (exactly theta_p: but below the sibling bar)
    par = np.array([-1, -1, -1, -1], dtype=np.int32)
    tok = np.array([1, 2, 3, 4], dtype=np.int32)
    q = np.array([big, at_s, below_s, at_p], dtype=np.float32)
    _, _, _, flags = graph_one(par, tok, q, 9, theta_p, theta_s)
    assert flags.tolist() == [0, 0, 2, 2]
    q = np.array([at_p, below_p, at_p, at_p], dtype=np.float32)                # sibling bar 0.3 * ~0.2: nobody below it
    _, _, _, flags = graph_one(par, tok, q, 9, theta_p, theta_s)
    assert flags.tolist() == [0, 1, 0, 0]
