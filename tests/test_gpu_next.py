"""GPU parity for the steps around the verify pass: un-merge-to-tree (Section 5.4) and the KV-cache commit
(Section 7.1), through the C ABI, bit-exact against the CPU oracle; and the tree variant of the whole verify
pass against the oracle run on the oracle's tree."""
import numpy as np
import pytest
import torch

from oracle import gsd_next
from paper_2407_16207_amd.workload import make_workload, merged_tree_dag, random_dag, VerifyConfig

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import gpu_util
    return gpu_util


def pack(dags):
    node_offsets, poff, pidx = [0], [0], []
    for off, par in dags:
        node_offsets.append(node_offsets[-1] + len(off) - 1)
        poff += [int(x) + len(pidx) for x in off[1:]]
        pidx += par.tolist()
    return (np.asarray(node_offsets, dtype=np.int32), np.asarray(poff, dtype=np.int32),
            np.asarray(pidx if pidx else [0], dtype=np.int32))


def run_unmerge(gpu, gsd, node_offsets, poff, pidx, max_nodes, cap):
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    o, tp, tpo, to, cnt = gsd.gsd_unmerge_to_tree(gpu.to_dev(node_offsets), gpu.to_dev(poff), gpu.to_dev(pidx),
                                                  max_nodes, cap, dag_error_flag=flag)
    torch.cuda.synchronize()
    o = o.cpu().numpy()
    total = int(o[-1])
    return o, tp.cpu().numpy()[:total], tpo.cpu().numpy()[:total + 1], to.cpu().numpy()[:total], \
        cnt.cpu().numpy(), int(flag.item())


def diamond_chain(k):
    off, par, last = [0, 1], [-1], 0
    for _ in range(k):
        a = len(off) - 1
        par += [last]; off.append(len(par))
        par += [last]; off.append(len(par))
        par += [a, a + 1]; off.append(len(par))
        last = a + 2
    return np.asarray(off, dtype=np.int32), np.asarray(par, dtype=np.int32)


@pytest.mark.parametrize("cap", [1, 7, 64, 512, 4096])
def test_unmerge_matches_oracle(gpu, cap):
    import paper_2407_16207_amd as gsd
    rng = np.random.default_rng(77)
    dags = [merged_tree_dag(rng, 64, 3, 6), random_dag(rng, 17, 3, 0.3), merged_tree_dag(rng, 1, 3, 0),
            random_dag(rng, 300, 2, 0.05), diamond_chain(70), merged_tree_dag(rng, 512, 4, 40),
            (np.array([0, 1, 1, 2], dtype=np.int32), np.array([-1, 0], dtype=np.int32))]   # node 1 has no parent
    node_offsets, poff, pidx = pack(dags)
    o, tp, tpo, to, cnt, flag = run_unmerge(gpu, gsd, node_offsets, poff, pidx, 512, cap)
    ro, rtp, rto, rcnt = gsd_next.unmerge_to_tree(node_offsets, poff, pidx, cap)
    assert flag == 0
    assert np.array_equal(o, ro) and np.array_equal(cnt, rcnt)
    assert np.array_equal(tp, rtp) and np.array_equal(to, rto)
    assert np.array_equal(tpo, np.arange(len(tp) + 1))
    assert cnt[4] == 1 << 62                                     # the diamond chain saturates the count


def test_unmerge_config_workloads_and_bad_edges(gpu):
    import paper_2407_16207_amd as gsd
    for cfg in (1, 3, 5):
        w = make_workload(cfg, with_logits=False, with_qkv=False)
        o, tp, tpo, to, cnt, flag = run_unmerge(gpu, gsd, w.node_offsets, w.parent_offsets, w.parent_idx,
                                                w.max_nodes, 512)
        ro, rtp, rto, rcnt = gsd_next.unmerge_to_tree(w.node_offsets, w.parent_offsets, w.parent_idx, 512)
        assert flag == 0 and np.array_equal(o, ro) and np.array_equal(cnt, rcnt)
        assert np.array_equal(tp, rtp) and np.array_equal(to, rto)
    # a forward edge and an out-of-range id are ignored and flagged; the rest is as if they were absent
    off = np.array([0, 1, 3, 5], dtype=np.int32)
    par = np.array([-1, 0, 2, 1, -7], dtype=np.int32)
    o, tp, tpo, to, cnt, flag = run_unmerge(gpu, gsd, np.array([0, 3], dtype=np.int32), off, par, 3, 64)
    assert flag == 1 and to.tolist() == [0, 1, 2] and tp.tolist() == [-1, 0, 1] and cnt.tolist() == [3]


def test_gather_rows(gpu):
    import paper_2407_16207_amd as gsd
    rng = np.random.default_rng(5)
    idx = rng.integers(0, 1000, 3001).astype(np.int32)
    for shape, dtype in (((1000, 8, 128), np.int16), ((1000,), np.int32), ((1000, 3), np.float32),
                         ((1000, 6), np.int16)):
        src = rng.integers(-30000, 30000, size=shape).astype(dtype)
        out = gsd.gsd_gather_rows(torch.from_numpy(src).cuda(), torch.from_numpy(idx).cuda())
        assert np.array_equal(out.cpu().numpy(), src[idx])
    # strided source rows (a column slice), and indices out of range leave their rows alone
    src = rng.integers(0, 100, size=(50, 16)).astype(np.int32)
    view = torch.from_numpy(src).cuda()[:, 4:12]
    out = torch.full((6, 8), -5, dtype=torch.int32, device="cuda")
    gsd.gsd_gather_rows(view, torch.tensor([3, -1, 49, 50, 0, 7], dtype=torch.int32, device="cuda"), out=out)
    want = np.full((6, 8), -5, dtype=np.int32)
    for r, s in enumerate([3, -1, 49, 50, 0, 7]):
        if 0 <= s < 50:
            want[r] = src[s, 4:12]
    assert np.array_equal(out.cpu().numpy(), want)


@pytest.mark.parametrize("layers,row_elems", [(1, 8), (3, 1024), (5, 8 * 128)])
def test_commit_kv_matches_oracle(gpu, layers, row_elems):
    import paper_2407_16207_amd as gsd
    rng = np.random.default_rng(layers * 1000 + row_elems)
    B, N = 6, 40
    prefix_lens = np.array([5, 0, 33, 7, 64, 1], dtype=np.int32)
    rows = int((prefix_lens + N).sum())
    kv_offsets = np.concatenate([[0], np.cumsum(prefix_lens + N)[:-1]]).astype(np.int64)
    k = rng.integers(0, 1 << 16, size=(layers, rows, 1, row_elems)).astype(np.uint16)
    v = rng.integers(0, 1 << 16, size=(layers, rows, 1, row_elems)).astype(np.uint16)
    accept_len = np.array([12, 0, 40, 1, 23, 9], dtype=np.int32)
    accept_path = np.full((B, N), -1, dtype=np.int32)
    for b in range(B):
        if b == 2:
            accept_path[b] = np.arange(N)                          # fully accepted chain: nothing moves
        else:
            accept_path[b, :accept_len[b]] = np.sort(rng.choice(N, size=accept_len[b], replace=False))
    accept_path[5, :9] = np.arange(1, 10)                          # every destination is the next row's source
    nk, nv, nl = gsd_next.commit_kv(k, v, kv_offsets, prefix_lens, accept_len, accept_path)
    dk = torch.from_numpy(k.view(np.int16)).cuda()
    dv = torch.from_numpy(v.view(np.int16)).cuda()
    got_len = gsd.gsd_commit_kv(dk, dv, gpu.to_dev(kv_offsets), gpu.to_dev(prefix_lens), gpu.to_dev(accept_len),
                                gpu.to_dev(accept_path))
    torch.cuda.synchronize()
    assert np.array_equal(got_len.cpu().numpy(), nl)
    assert np.array_equal(dk.cpu().numpy().view(np.uint16), nk)
    assert np.array_equal(dv.cpu().numpy().view(np.uint16), nv)


def test_tree_verification_end_to_end(gpu):
    """The paper's exact variant: un-merge, carry per-node data to the replicas, then the same mask / attention /
    acceptance calls on the tree.  Checked against the oracle applied to the oracle's tree; the accepted path,
    mapped back through `origin`, is the one found on the graph directly."""
    import paper_2407_16207_amd as gsd
    from oracle import gsd_ref
    rng = np.random.default_rng(2024)
    B, N, Hq, Hkv, D, P, V = 3, 96, 8, 2, 128, 200, 211
    cfg = VerifyConfig("tree-e2e", B, Hq, Hkv, D, P, P, 1, N, 2, V, 0.8, "bf16")
    w = make_workload(cfg, seed=99)
    dags = [merged_tree_dag(rng, N, 3, 8) for _ in range(B)]
    node_offsets, poff, pidx = pack(dags)
    tokens = rng.integers(0, 5, B * N).astype(np.int32)
    pred = rng.integers(0, 5, B * N).astype(np.int32)
    root_pred = rng.integers(0, 5, B).astype(np.int32)
    cap = 512
    d_no, d_po, d_pi = gpu.to_dev(node_offsets), gpu.to_dev(poff), gpu.to_dev(pidx)
    t_no, t_par, t_po, t_org, cnt = gsd.gsd_unmerge_to_tree(d_no, d_po, d_pi, N, cap)
    ro, rtp, rto, rcnt = gsd_next.unmerge_to_tree(node_offsets, poff, pidx, cap)
    o = t_no.cpu().numpy()
    Tt = int(o[-1])
    assert np.array_equal(o, ro) and Tt > B * N and (rcnt <= cap).all()
    sizes = np.diff(o)
    n_max = int(sizes.max())
    # packed source rows of every replica (setup arithmetic on indices, not part of the method)
    seq_of = np.repeat(np.arange(B), sizes)
    src_node = torch.from_numpy((node_offsets[seq_of] + rto).astype(np.int32)).cuda()
    q_t = gsd.gsd_gather_rows(gpu.to_dev(w.q), src_node)
    tok_t = gsd.gsd_gather_rows(gpu.to_dev(tokens), src_node)
    pred_t = gsd.gsd_gather_rows(gpu.to_dev(pred), src_node)
    # K/V of the tree pass: each sequence's prefix rows, then its replicas' rows
    kv_rows = w.prefix_lens.astype(np.int64) + sizes
    t_kv_offsets = np.concatenate([[0], np.cumsum(kv_rows)[:-1]]).astype(np.int64)
    src_kv = np.concatenate([np.concatenate([w.kv_offsets[b] + np.arange(P),
                                             w.kv_offsets[b] + P + rto[o[b]:o[b + 1]]]) for b in range(B)])
    src_kv_t = torch.from_numpy(src_kv.astype(np.int32)).cuda()
    k_t = gsd.gsd_gather_rows(gpu.to_dev(w.k), src_kv_t)
    v_t = gsd.gsd_gather_rows(gpu.to_dev(w.v), src_kv_t)
    t_par, t_po = t_par[:Tt].contiguous(), t_po[:Tt + 1].contiguous()
    mask = gsd.gsd_build_mask(t_no, t_po, t_par, n_max)
    out = gsd.gsd_dag_attention(q_t, k_t, v_t, gpu.to_dev(t_kv_offsets), gpu.to_dev(w.prefix_lens), t_no, mask,
                                n_max, P, w.softmax_scale)
    ln, path, bonus, _ = gsd.gsd_accept_longest_path(t_no, t_po, t_par, tok_t, gpu.to_dev(root_pred), n_max,
                                                     pred=pred_t)
    torch.cuda.synchronize()
    # oracle on the oracle's tree
    rmask, _ = gsd_ref.build_mask(ro, np.arange(Tt + 1), rtp)
    assert np.array_equal(gpu.mask_to_numpy(mask), rmask)
    ref_out = gsd_ref.dag_attention(w.q[src_node.cpu().numpy()], w.k[src_kv], w.v[src_kv], t_kv_offsets,
                                    w.prefix_lens, ro, rmask, w.softmax_scale)
    assert np.abs(gpu.out_to_f64(out) - ref_out).max() <= 2e-2
    rl, rpath, rbonus = gsd_ref.accept_longest_path(ro, np.arange(Tt + 1), rtp, tokens[src_node.cpu().numpy()],
                                                    pred[src_node.cpu().numpy()], root_pred, max_nodes=n_max)
    assert np.array_equal(ln.cpu().numpy(), rl) and np.array_equal(path.cpu().numpy(), rpath)
    assert np.array_equal(bonus.cpu().numpy(), rbonus)
    # mapped back to graph ids it is the graph's own longest accepted path
    dl, dpath, dbonus = gsd_ref.accept_longest_path(node_offsets, poff, pidx, tokens, pred, root_pred)
    for b in range(B):
        tree_ids = rpath[b, :rl[b]]
        assert rto[o[b] + tree_ids].tolist() == dpath[b, :dl[b]].tolist()
    assert np.array_equal(dbonus, rbonus) and (rl > 0).any()


# ---------------------------------------------------------------------------------- non-deterministic verify
def stochastic_problem(rng, sizes, vocab, dtype, max_parents=3, peaked=2.0):
    from paper_2407_16207_amd.workload import f32_to_bf16_bits
    dags = [random_dag(rng, n, max_parents, 0.2) for n in sizes]
    node_offsets, poff, pidx = pack(dags)
    T, B = int(node_offsets[-1]), len(sizes)

    def logits(rows):
        x = (rng.standard_normal((rows, vocab)) * peaked).astype(np.float32)
        return x if dtype == "f32" else f32_to_bf16_bits(x)
    lp, lp_root, lq, lq_root = logits(T), logits(B), logits(T), logits(B)
    p, _, _ = gsd_next.softmax_rows(lp)
    p_root, _, _ = gsd_next.softmax_rows(lp_root)
    q, _, _ = gsd_next.softmax_rows(lq)
    q_root, _, _ = gsd_next.softmax_rows(lq_root)
    # drafted tokens: mostly the draft model's likely ones, so that p/q is of order one
    tokens = np.empty(T, dtype=np.int32)
    draft_prob = np.empty(T, dtype=np.float32)
    for b in range(B):
        lo = int(node_offsets[b])
        for i in range(sizes[b]):
            e = int(poff[lo + i])
            r = int(pidx[e]) if poff[lo + i + 1] > e else -1
            qr = q_root[b] if r < 0 or r >= i else q[lo + r]
            tok = int(rng.choice(vocab, p=qr))
            tokens[lo + i] = tok
            draft_prob[lo + i] = max(float(qr[tok]), 1e-6)
    accept_u = rng.random(T).astype(np.float32)
    resample_u = rng.random(B).astype(np.float32)
    # keep every coin clear of its threshold (the GPU evaluates p in fp32): pull a close call well inside "accept"
    for b in range(B):
        lo = int(node_offsets[b])
        for i in range(sizes[b]):
            for e in range(int(poff[lo + i]), int(poff[lo + i + 1])):
                r = int(pidx[e])
                if r < -1 or r >= i:
                    continue
                pt = p_root[b, tokens[lo + i]] if r == -1 else p[lo + r, tokens[lo + i]]
                thr = min(1.0, pt / draft_prob[lo + i])
                if abs(accept_u[lo + i] - thr) < 1e-3 * max(thr, 1e-9) + 1e-7:
                    accept_u[lo + i] = np.float32(0.5 * thr)
    return dict(node_offsets=node_offsets, poff=poff, pidx=pidx, tokens=tokens, lp=lp, lp_root=lp_root, lq=lq,
                lq_root=lq_root, p=p, p_root=p_root, q=q, q_root=q_root, draft_prob=draft_prob, accept_u=accept_u,
                resample_u=resample_u, max_nodes=max(sizes))


@pytest.mark.parametrize("dtype,vocab,sizes", [("f32", 1003, [60, 1, 200, 17, 512, 33]),
                                               ("bf16", 1003, [60, 1, 200, 17, 512, 33]),
                                               # 8192: the draw kernel's slices are whole 16-byte runs (its vector path)
                                               ("f32", 8192, [60, 40, 150, 17, 90, 33]), ("bf16", 8192, [60, 40, 150, 17, 90, 33]),
                                               # 32000: a full register slice (32 values) per thread of the draw kernel
                                               ("f32", 32000, [30, 12, 25, 7, 40, 18, 33]), ("bf16", 32000, [30, 12, 25, 7, 40, 18, 33])])
def test_softmax_stats_and_stochastic_acceptance(gpu, dtype, vocab, sizes):
    import paper_2407_16207_amd as gsd
    rng = np.random.default_rng((31 if dtype == "f32" else 32) + vocab)
    pr = stochastic_problem(rng, sizes, vocab, dtype)
    d = {k: gpu.to_dev(v) for k, v in pr.items() if isinstance(v, np.ndarray) and k not in ("p", "p_root", "q", "q_root")}
    ln, path, end, bonus, row_max, row_sum = gsd.gsd_accept_stochastic(
        d["node_offsets"], d["poff"], d["pidx"], d["tokens"], d["lp"], d["lp_root"], d["lq"], d["lq_root"],
        d["draft_prob"], d["accept_u"], d["resample_u"], pr["max_nodes"])
    torch.cuda.synchronize()
    # normalisers against the fp64 softmax
    _, m_ref, z_ref = gsd_next.softmax_rows(np.concatenate([pr["lp"], pr["lp_root"]]))
    assert np.array_equal(row_max.cpu().numpy().astype(np.float64), m_ref)
    assert np.abs(row_sum.cpu().numpy() / z_ref - 1).max() < 2e-6
    m2, s2 = gsd.gsd_softmax_stats(d["lq"][:, 3:-2])            # misaligned rows, odd length
    _, m_ref2, z_ref2 = gsd_next.softmax_rows(pr["lq"][:, 3:-2])
    assert np.array_equal(m2.cpu().numpy().astype(np.float64), m_ref2) and np.abs(s2.cpu().numpy() / z_ref2 - 1).max() < 2e-6
    # accepted paths: exact
    rl, rpath, rbonus, _, cdfs = gsd_next.accept_stochastic(pr["node_offsets"], pr["poff"], pr["pidx"], pr["tokens"], pr["p"],
                                                            pr["p_root"], pr["draft_prob"], pr["accept_u"], pr["q"],
                                                            pr["q_root"], pr["resample_u"])
    assert np.array_equal(ln.cpu().numpy(), rl) and np.array_equal(path.cpu().numpy(), rpath)
    assert (rl > 0).sum() >= 3                   # the case is not trivial
    ends = end.cpu().numpy()
    for b in range(len(rl)):
        assert ends[b] == (rpath[b, rl[b] - 1] if rl[b] else -1)
    # regenerated token: the GPU sums in fp32 in its own order, so its draw is checked against the oracle's CDF: the
    # target must fall into the drawn token's interval, up to the rounding of the partial sums
    got = bonus.cpu().numpy()
    exact = 0
    for b, cdf in enumerate(cdfs):
        x = int(got[b])
        target = float(pr["resample_u"][b]) * cdf[-1]
        lo_edge = cdf[x - 1] if x else 0.0
        tol = 2e-5 * cdf[-1]
        assert cdf[x] > lo_edge                      # a token that carries weight
        assert lo_edge - tol <= target <= cdf[x] + tol, (b, x, rbonus[b])
        exact += int(x == rbonus[b])
    assert exact >= len(cdfs) - 1


def test_stochastic_acceptance_many_parents(gpu):
    """Nodes with more parents than the kernel keeps in registers (4): accepted paths stay exact."""
    import paper_2407_16207_amd as gsd
    rng = np.random.default_rng(77)
    pr = stochastic_problem(rng, [90, 300, 512], 257, "f32", max_parents=9)
    assert np.diff(pr["poff"]).max() > 4
    d = {k: gpu.to_dev(v) for k, v in pr.items() if isinstance(v, np.ndarray) and k not in ("p", "p_root", "q", "q_root")}
    ln, path, end, bonus, _, _ = gsd.gsd_accept_stochastic(
        d["node_offsets"], d["poff"], d["pidx"], d["tokens"], d["lp"], d["lp_root"], d["lq"], d["lq_root"],
        d["draft_prob"], d["accept_u"], d["resample_u"], pr["max_nodes"])
    torch.cuda.synchronize()
    rl, rpath, _, _, _ = gsd_next.accept_stochastic(pr["node_offsets"], pr["poff"], pr["pidx"], pr["tokens"], pr["p"],
                                                    pr["p_root"], pr["draft_prob"], pr["accept_u"], pr["q"],
                                                    pr["q_root"], pr["resample_u"])
    assert np.array_equal(ln.cpu().numpy(), rl) and np.array_equal(path.cpu().numpy(), rpath)
    assert rl.max() > 2


def test_stochastic_limits_on_gpu(gpu, ref):
    """Coins at zero accept every edge with positive probability (the graph's deepest path); a one-hot LLM with a
    certain draft reduces to deterministic verification."""
    import paper_2407_16207_amd as gsd
    rng = np.random.default_rng(77)
    pr = stochastic_problem(rng, [90, 40], 257, "f32")
    T, B, V = len(pr["tokens"]), 2, 257
    d = {k: gpu.to_dev(v) for k, v in pr.items() if isinstance(v, np.ndarray) and k not in ("p", "p_root", "q", "q_root")}
    zeros = torch.zeros(T, dtype=torch.float32, device="cuda")
    ln, path, end, bonus, _, _ = gsd.gsd_accept_stochastic(d["node_offsets"], d["poff"], d["pidx"], d["tokens"], d["lp"],
                                                          d["lp_root"], d["lq"], d["lq_root"], d["draft_prob"], zeros,
                                                          d["resample_u"], pr["max_nodes"])
    rl, rpath, _, _, _ = gsd_next.accept_stochastic(pr["node_offsets"], pr["poff"], pr["pidx"], pr["tokens"], pr["p"],
                                                    pr["p_root"], pr["draft_prob"], np.zeros(T), pr["q"], pr["q_root"],
                                                    pr["resample_u"])
    assert np.array_equal(ln.cpu().numpy(), rl) and np.array_equal(path.cpu().numpy(), rpath) and (rl >= 3).all()
    # one-hot LLM
    pred = rng.integers(0, V, T + B)
    lp = np.full((T + B, V), -80.0, dtype=np.float32)
    lp[np.arange(T + B), pred] = 0.0
    tokens = pr["tokens"].copy()
    hit = rng.random(T) < 0.7                            # plant matches along first parents
    for b in range(B):
        lo = int(pr["node_offsets"][b])
        for i in range(int(pr["node_offsets"][b + 1]) - lo):
            r = int(pr["pidx"][pr["poff"][lo + i]])
            if hit[lo + i]:
                tokens[lo + i] = pred[T + b] if r < 0 else pred[lo + r]
    ones = torch.ones(T, dtype=torch.float32, device="cuda")
    u = torch.full((T,), 0.9, dtype=torch.float32, device="cuda")
    ln, path, end, bonus, _, _ = gsd.gsd_accept_stochastic(d["node_offsets"], d["poff"], d["pidx"], gpu.to_dev(tokens),
                                                          gpu.to_dev(lp[:T]), gpu.to_dev(lp[T:]), d["lq"], d["lq_root"], ones, u,
                                                          d["resample_u"], pr["max_nodes"])
    dl, dpath, dbonus = ref.accept_longest_path(pr["node_offsets"], pr["poff"], pr["pidx"], tokens, pred[:T].astype(np.int32),
                                                pred[T:].astype(np.int32))
    assert np.array_equal(ln.cpu().numpy(), dl) and np.array_equal(path.cpu().numpy(), dpath) and (dl > 0).any()


def test_many_sequences_unmerge_mask_and_acceptance(gpu, ref):
    """650 small graphs in one call: more sequences than a work-group has threads (the packed position of a
    sequence's tree is a sum over all sequences before it), one work-group per sequence everywhere else."""
    import paper_2407_16207_amd as gsd
    from paper_2407_16207_amd.workload import random_dag, merged_tree_dag
    rng = np.random.default_rng(123)
    dags = [(merged_tree_dag(rng, int(n), 3, int(rng.integers(0, 4))) if rng.random() < 0.5
             else random_dag(rng, int(n), 3, 0.2)) for n in rng.integers(1, 30, 650)]
    no, poff, pidx = pack(dags)
    o, tpar, tpo, to, cnt, fl = run_unmerge(gpu, gsd, no, poff, pidx, 32, 64)
    ro, rtp, rto, rcnt = gsd_next.unmerge_to_tree(no, poff, pidx, 64)
    assert fl == 0 and np.array_equal(o, ro) and np.array_equal(cnt, rcnt)
    assert np.array_equal(tpar, rtp) and np.array_equal(to, rto)
    n_max = int(np.diff(no).max())
    mask = gsd.gsd_build_mask(gpu.to_dev(no), gpu.to_dev(poff), gpu.to_dev(pidx), n_max)
    rmask, _ = ref.build_mask(no, poff, pidx)
    assert np.array_equal(gpu.mask_to_numpy(mask), rmask)
    T, B = int(no[-1]), len(no) - 1
    tokens, pred = rng.integers(0, 3, T).astype(np.int32), rng.integers(0, 3, T).astype(np.int32)
    rootp = rng.integers(0, 3, B).astype(np.int32)
    ln, path, bonus, _ = gsd.gsd_accept_longest_path(gpu.to_dev(no), gpu.to_dev(poff), gpu.to_dev(pidx),
                                                     gpu.to_dev(tokens), gpu.to_dev(rootp), n_max, pred=gpu.to_dev(pred))
    wl, wp, wb = ref.accept_longest_path(no, poff, pidx, tokens, pred, rootp)
    assert np.array_equal(ln.cpu().numpy(), wl) and np.array_equal(path.cpu().numpy(), wp)
    assert np.array_equal(bonus.cpu().numpy(), wb) and (wl > 0).sum() > 100


# -------------------------------------------------------------------------------------- graph construction
def token_trees(rng, sizes, k, vocab):
    from test_oracle_next import random_token_tree
    node_offsets, par, tok, q = [0], [], [], []
    for n in sizes:
        p, t, pr = random_token_tree(rng, n, k, vocab)
        node_offsets.append(node_offsets[-1] + len(p))
        par.append(p); tok.append(t); q.append(pr)
    return (np.asarray(node_offsets, dtype=np.int32), np.concatenate(par).astype(np.int32),
            np.concatenate(tok).astype(np.int32), np.concatenate(q).astype(np.float32))


@pytest.mark.parametrize("tau,theta_prob,theta_sib", [(1, 0.0, 0.0), (2, 0.0, 0.0), (3, 0.1, 0.3), (2, 0.2, 0.3),
                                                     (8, 0.05, 0.0), (100, 0.0, 0.6)])
def test_build_token_graph_matches_oracle(gpu, tau, theta_prob, theta_sib):
    import paper_2407_16207_amd as gsd
    rng = np.random.default_rng(1000 + tau)
    node_offsets, par, tok, q = token_trees(rng, [300, 1, 512, 40, 7, 511], 4, 6 if tau < 8 else 2)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    g_off, p_off, p_idx, origin, flags, counts = gsd.gsd_build_token_graph(
        gpu.to_dev(node_offsets), gpu.to_dev(par), gpu.to_dev(tok), gpu.to_dev(q), 512, tau, theta_prob, theta_sib,
        error_flag=flag)
    torch.cuda.synchronize()
    r_goff, r_poff, r_pidx, r_origin, r_flags = gsd_next.build_token_graph(node_offsets, par, tok, q, tau, theta_prob, theta_sib)
    assert flag.item() == 0
    g_off = g_off.cpu().numpy()
    Tn = int(g_off[-1])
    assert np.array_equal(g_off, r_goff)
    p_off = p_off.cpu().numpy()[:Tn + 1]
    assert np.array_equal(p_off, r_poff)
    assert np.array_equal(p_idx.cpu().numpy()[:p_off[-1]], r_pidx)
    assert np.array_equal(origin.cpu().numpy()[:Tn], r_origin) and np.array_equal(flags.cpu().numpy()[:Tn], r_flags)
    cn = counts.cpu().numpy()
    assert np.array_equal(cn[:, 0], np.diff(r_goff))
    assert cn[:, 1].sum() == len(r_pidx)
    if tau <= 3:
        assert (r_flags & 4).any() and len(r_pidx) > Tn          # something was merged: the case is not trivial
    # the result feeds the verify path as it is: visibility mask of the graph against the oracle's
    from oracle import gsd_ref
    n_max = int(np.diff(g_off).max())
    mask = gsd.gsd_build_mask(gpu.to_dev(g_off), gpu.to_dev(p_off), gpu.to_dev(r_pidx), n_max)
    rmask, rflag = gsd_ref.build_mask(r_goff, r_poff, r_pidx)
    assert rflag == 0 and np.array_equal(gpu.mask_to_numpy(mask), rmask)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_argmax_and_softmax_normalisers_in_one_pass(gpu, ref, dtype):
    """gsd_node_argmax_stats: the argmax bit-exact against the oracle, the normalisers against the fp64 softmax, on
    aligned and misaligned rows, ties, -inf rows and the full config-4 logits (the launch the benchmark times)."""
    import paper_2407_16207_amd as gsd
    from paper_2407_16207_amd.workload import f32_to_bf16_bits, bf16_bits_to_f32, make_workload
    rng = np.random.default_rng(77)
    for vocab in (1, 7, 1000, 32003):
        x = (rng.standard_normal((9, vocab)) * 3).astype(np.float32)
        x[0, :] = 0.5
        x[1, vocab - 1] = 9.0
        x[2, 0] = 9.0
        x[3, :] = -np.inf
        if vocab > 10:
            x[6, [vocab - 2, 5, vocab // 2]] = 7.0
        stored = x if dtype == "f32" else f32_to_bf16_bits(x)
        vals = x if dtype == "f32" else bf16_bits_to_f32(stored)
        t = gpu.to_dev(stored)
        for view, np_view in ((t, vals), (t[:, 1:], vals[:, 1:])) if vocab > 1 else ((t, vals),):
            pred, m, s_ = gsd.gsd_node_argmax_stats(view)
            torch.cuda.synchronize()
            assert np.array_equal(pred.cpu().numpy(), ref.node_argmax(np.ascontiguousarray(np_view)))
            _, m_ref, z_ref = gsd_next.softmax_rows(np_view.astype(np.float64))
            assert np.array_equal(m.cpu().numpy().astype(np.float64), m_ref)
            got = s_.cpu().numpy().astype(np.float64)
            ok = z_ref > 0
            assert np.abs(got[ok] / z_ref[ok] - 1).max() < 2e-6 and np.all(got[~ok] == 0)
    if dtype == "bf16":
        w = make_workload(4, with_qkv=False)
        logits = gpu.to_dev(w.logits)
        pred, m, s_ = gsd.gsd_node_argmax_stats(logits)
        torch.cuda.synchronize()
        assert np.array_equal(pred.cpu().numpy(), ref.node_argmax(w.logits))
        assert torch.equal(pred, gsd.gsd_node_argmax(logits))
        m2, s2 = gsd.gsd_softmax_stats(logits)
        assert torch.equal(m, m2) and (s_ / s2 - 1).abs().max().item() < 2e-6


def compare_graph_with_oracle(gpu, node_offsets, par, tok, q, tau, theta_prob, theta_sib, max_nodes=512):
    import paper_2407_16207_amd as gsd
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    r = gsd_next.build_token_graph(node_offsets, par, tok, q, tau, theta_prob, theta_sib)
    g_off, p_off, p_idx, origin, flags, counts = gsd.gsd_build_token_graph(
        gpu.to_dev(node_offsets), gpu.to_dev(par), gpu.to_dev(tok), gpu.to_dev(q), max_nodes, tau, theta_prob, theta_sib,
        edge_capacity=max(16, len(r[2])), error_flag=flag)
    torch.cuda.synchronize()
    assert flag.item() == 0
    g_off = g_off.cpu().numpy()
    Tn = int(g_off[-1])
    assert np.array_equal(g_off, r[0])
    assert np.array_equal(p_off.cpu().numpy()[:Tn + 1], r[1])
    assert np.array_equal(p_idx.cpu().numpy()[:len(r[2])], r[2])
    assert np.array_equal(origin.cpu().numpy()[:Tn], r[3]) and np.array_equal(flags.cpu().numpy()[:Tn], r[4])
    return r


def test_build_token_graph_hand_example_with_a_merge_into_an_earlier_layer(gpu):
    """tests/golden/hand_merge8.txt (worked out by hand from Section 5.3) through the kernel."""
    import os
    from helpers import load_hand_dag
    h = load_hand_dag(os.path.join(os.path.dirname(__file__), "golden", "hand_merge8.txt"))
    par, tok = np.asarray(h["tree_parent"], dtype=np.int32), np.asarray(h["tokens"], dtype=np.int32)
    r = compare_graph_with_oracle(gpu, np.array([0, len(par)], dtype=np.int32), par, tok,
                                  np.full(len(par), 0.5, dtype=np.float32), h["tau"][0], 0.0, 0.0, max_nodes=8)
    assert r[3].tolist() == h["origin"] and r[4].tolist() == h["flags"] and r[2].tolist() == h["parent_idx"].tolist()


@pytest.mark.parametrize("seed", range(12))
def test_build_token_graph_random_trees(gpu, seed):
    """Trees of many shapes and alphabets: merges within a layer, into earlier layers, refused (cyclic) ones, graphs
    that have to be renumbered, first occurrences with dozens of merged nodes."""
    rng = np.random.default_rng(7000 + seed)
    sizes = [int(x) for x in rng.integers(1, 513, 5)] + [512]
    k, vocab, tau = int(rng.integers(2, 5)), int(rng.integers(2, 30)), int(rng.integers(1, 4))
    node_offsets, par, tok, q = token_trees(rng, sizes, k, vocab)
    tp, ts = (0.0, 0.0) if seed % 3 else (0.05, 0.2)
    r = compare_graph_with_oracle(gpu, node_offsets, par, tok, q, tau, tp, ts)
    print(f"[graph] seed {seed}: k {k} vocab {vocab} tau {tau}: {int(r[0][-1])} nodes, {len(r[2])} edges, "
          f"{int(((r[4] & 4) != 0).sum())} redundant, {int(((r[4] & 8) != 0).sum())} of them cyclic", flush=True)


@pytest.mark.parametrize("k,vocab,tau,seed,at_least", [(8, 3, 2, 5, 33), (6, 4, 3, 8, 65), (12, 4, 2, 3, 129),
                                                       (10, 6, 3, 9, 129), (16, 6, 2, 1, 257), (30, 8, 2, 4, 257)])
def test_build_token_graph_many_redundant_nodes(gpu, k, vocab, tau, seed, at_least):
    """Wide trees over tiny alphabets: one sequence with more than 32, 64, 128 and 256 redundant nodes (the merge
    decisions are taken in groups of 64), refused (cyclic) merges among them, next to a small and an empty-ish one."""
    from test_oracle_next import random_token_tree
    rng = np.random.default_rng(seed)
    p, t, q = random_token_tree(rng, 512, k, vocab)
    p2, t2, q2 = random_token_tree(rng, 37, 3, vocab)
    node_offsets = np.array([0, len(p), len(p) + len(p2), len(p) + len(p2) + 1], dtype=np.int32)
    par = np.concatenate([p, p2, [-1]]).astype(np.int32)
    # token ids at the ends of the int32 range: a token is only ever compared for equality
    ids = np.array([-1, -2**31, 2**31 - 1, 0, 1, -2, 65536, 12345678], dtype=np.int64)
    tok = ids[np.concatenate([t, t2, [0]]).astype(np.int64)].astype(np.int32)
    prob = np.concatenate([q, q2, [1.0]]).astype(np.float32)
    r = compare_graph_with_oracle(gpu, node_offsets, par, tok, prob, tau, 0.0, 0.0)
    first = r[4][:int(r[0][1])]
    assert int(((first & 4) != 0).sum()) >= at_least, int(((first & 4) != 0).sum())


def test_build_token_graph_many_sequences(gpu):
    """More sequences than a work-group has threads: every work-group adds up the counts of all sequences before it."""
    rng = np.random.default_rng(99)
    sizes = [int(x) for x in rng.integers(1, 40, 700)] + [512, 300]
    node_offsets, par, tok, q = token_trees(rng, sizes, 3, 5)
    r = compare_graph_with_oracle(gpu, node_offsets, par, tok, q, 2, 0.0, 0.0)
    assert len(r[0]) == len(sizes) + 1 and int(((r[4] & 4) != 0).sum()) > 1000


def test_build_token_graph_flags_bad_input_and_small_capacity(gpu):
    import paper_2407_16207_amd as gsd
    par = np.array([-1, 0, 3, 0, -5, 1], dtype=np.int32)          # node 2 points forward, node 4 below -1
    tok = np.array([1, 2, 3, 4, 5, 6], dtype=np.int32)
    q = np.ones(6, dtype=np.float32)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    g_off, p_off, p_idx, origin, flags, counts = gsd.gsd_build_token_graph(
        gpu.to_dev(np.array([0, 6], dtype=np.int32)), gpu.to_dev(par), gpu.to_dev(tok), gpu.to_dev(q), 6, 5, 0.0, 0.0,
        error_flag=flag)
    torch.cuda.synchronize()
    assert flag.item() & 1
    assert origin.cpu().numpy()[:int(g_off[-1])].tolist() == [0, 1, 3, 5]      # the malformed nodes are dropped
    # capacity: a merged graph needs more edge slots than nodes
    rng = np.random.default_rng(9)
    node_offsets, par, tok, q = token_trees(rng, [200], 4, 3)
    flag.zero_()
    out = gsd.gsd_build_token_graph(gpu.to_dev(node_offsets), gpu.to_dev(par), gpu.to_dev(tok), gpu.to_dev(q), 512, 1,
                                    0.0, 0.0, edge_capacity=3, error_flag=flag)
    torch.cuda.synchronize()
    assert flag.item() & 2


def test_measurement_aid_counts_what_it_says(gpu):
    """The benchmark's bare matrix-instruction loop really issues iters*16 instructions per lane: with all-ones operands
    every instruction adds 16 to each of a lane's 64 accumulator elements, four instructions per accumulator block and
    trip."""
    import bench
    ones = torch.ones(4096, dtype=torch.bfloat16, device="cuda")
    for wgs, iters in ((3, 1), (5, 7)):
        sink = bench.mfma_loop(ones, wgs, iters)
        torch.cuda.synchronize()
        assert sink.numel() == wgs * 512
        assert torch.all(sink == 64.0 * 16.0 * 4 * iters)
