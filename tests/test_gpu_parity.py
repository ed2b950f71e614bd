"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.
Bit-exact for masks, argmax ids and accepted paths; attention within max-abs 1e-4 (fp32) / 2e-2 (bf16)."""
import numpy as np
import pytest
import torch

from paper_2407_16207_amd.workload import (VerifyConfig, Workload, make_workload, random_dag, f32_to_bf16_bits)

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import gpu_util
    return gpu_util


_cache = {}


def workload(cfg_id, **kw):
    key = (cfg_id, tuple(sorted(kw.items())))
    if key not in _cache:
        if len(_cache) > 1:          # keep at most two big workloads alive on the host
            _cache.pop(next(iter(_cache)))
        print(f"[gen] config {cfg_id} {kw}", flush=True)
        _cache[key] = make_workload(cfg_id, **kw)
    return _cache[key]


def custom_workload(rng, sizes, prefixes, Hq, Hkv, D, dtype, vocab=97, max_parents=3):
    """Several sequences with general (non-layered) DAGs of different sizes and prefix lengths."""
    B = len(sizes)
    node_offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    offs, pars, e = [np.zeros(1, dtype=np.int32)], [], 0
    for n in sizes:
        o, p = random_dag(rng, n, max_parents)
        offs.append(o[1:] + e)
        pars.append(p)
        e += len(p)
    T = int(node_offsets[-1])
    prefix_lens = np.asarray(prefixes, dtype=np.int32)
    rows = prefix_lens.astype(np.int64) + np.asarray(sizes)
    kv_offsets = np.concatenate([[0], np.cumsum(rows)[:-1]]).astype(np.int64)
    R = int(rows.sum())

    def draw(shape):
        x = rng.standard_normal(shape, dtype=np.float32)
        return x if dtype == "f32" else f32_to_bf16_bits(x)

    cfg = VerifyConfig("custom", B, Hq, Hkv, D, int(min(prefixes)), int(max(prefixes)), 1, max(sizes), max_parents,
                       vocab, 0.5, dtype)
    tokens = rng.integers(0, 6, T).astype(np.int32)                  # tiny token alphabet: ties and long paths
    logits = rng.standard_normal((T, vocab), dtype=np.float32)
    logits[np.arange(T), rng.integers(0, 6, T)] += 6.0
    return Workload(cfg=cfg, seed=0, node_offsets=node_offsets, parent_offsets=np.concatenate(offs).astype(np.int32),
                    parent_idx=np.concatenate(pars).astype(np.int32), tokens=tokens,
                    root_pred=rng.integers(0, 6, B).astype(np.int32), prefix_lens=prefix_lens, kv_offsets=kv_offsets,
                    q=draw((T, Hq, D)), k=draw((R, Hkv, D)), v=draw((R, Hkv, D)),
                    logits=logits if dtype == "f32" else f32_to_bf16_bits(logits),
                    softmax_scale=float(1.0 / np.sqrt(D)))


# ------------------------------------------------------------------------------------------------- mask
@pytest.mark.parametrize("cfg_id", [1, 2, 3, 4, 5])
def test_mask_configs(gpu, ref, cfg_id):
    w = workload(cfg_id, with_qkv=False, with_logits=False)
    d = gpu.DeviceWorkload(w)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    got = gpu.mask_to_numpy(d.build_mask(flag=flag))
    want, _ = ref.build_mask(w.node_offsets, w.parent_offsets, w.parent_idx)
    assert np.array_equal(got, want)
    assert int(flag.item()) == 0
    if cfg_id == 5:                                   # the same-size tree-shaped comparison mask
        wt = workload(5, with_qkv=False, with_logits=False, tree=True)
        got = gpu.mask_to_numpy(gpu.DeviceWorkload(wt).build_mask())
        assert np.array_equal(got, ref.build_mask(wt.node_offsets, wt.parent_offsets, wt.parent_idx)[0])


def test_mask_general_dags_and_edges(gpu, ref):
    rng = np.random.default_rng(77)
    w = custom_workload(rng, [1, 70, 512, 3, 129, 64, 65], [0] * 7, 1, 1, 64, "f32")
    d = gpu.DeviceWorkload(w)
    got = gpu.mask_to_numpy(d.build_mask())
    assert np.array_equal(got, ref.build_mask(w.node_offsets, w.parent_offsets, w.parent_idx)[0])
    # wider rows than needed: the extra words are zero
    got = gpu.mask_to_numpy(d.build_mask(words_per_row=8))
    want = ref.build_mask(w.node_offsets, w.parent_offsets, w.parent_idx, words_per_row=8)[0]
    assert np.array_equal(got, want)
    # a deep chain: the longest dependency run the relaxation can meet
    n = 512
    w2 = custom_workload(rng, [n], [0], 1, 1, 64, "f32")
    w2.parent_offsets = np.arange(n + 1, dtype=np.int32)
    w2.parent_idx = np.arange(-1, n - 1, dtype=np.int32)
    got = gpu.mask_to_numpy(gpu.DeviceWorkload(w2).build_mask())
    assert np.array_equal(got, ref.build_mask(w2.node_offsets, w2.parent_offsets, w2.parent_idx)[0])


def test_mask_and_accept_dense_dags(gpu, ref):
    """Nodes with more parents than the kernels keep in registers (4), and a sequence whose parent lists (more than
    6144 entries) do not fit the kernels' LDS copy and are read from memory."""
    for seed, sizes, max_parents in ((5, [40, 200, 512], 9), (6, [512, 300], 40)):
        rng = np.random.default_rng(seed)
        w = custom_workload(rng, sizes, [0] * len(sizes), 1, 1, 64, "f32", vocab=6, max_parents=max_parents)
        per_seq_edges = np.diff(w.parent_offsets[w.node_offsets])
        assert np.diff(w.parent_offsets).max() > 4
        if max_parents == 40:
            assert per_seq_edges.max() > 6144
        d = gpu.DeviceWorkload(w)
        got = gpu.mask_to_numpy(d.build_mask())
        assert np.array_equal(got, ref.build_mask(w.node_offsets, w.parent_offsets, w.parent_idx)[0])
        pred = rng.integers(0, 6, w.total_nodes).astype(np.int32)
        ln, path, bonus, _ = d.accept(logits=False, pred=torch.from_numpy(pred).cuda())
        wl, wp, wb = ref.accept_longest_path(w.node_offsets, w.parent_offsets, w.parent_idx, w.tokens, pred,
                                             w.root_pred)
        assert np.array_equal(ln.cpu().numpy(), wl) and np.array_equal(path.cpu().numpy(), wp)
        assert np.array_equal(bonus.cpu().numpy(), wb)


def test_mask_bad_parent_sets_flag(gpu, ref):
    rng = np.random.default_rng(3)
    w = custom_workload(rng, [6], [0], 1, 1, 64, "f32")
    w.parent_offsets = np.array([0, 1, 2, 3, 4, 5, 6], dtype=np.int32)
    w.parent_idx = np.array([-1, 0, 4, 1, 2, -7], dtype=np.int32)     # node 2 names a later node, node 5 garbage
    d = gpu.DeviceWorkload(w)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    got = gpu.mask_to_numpy(d.build_mask(flag=flag))
    want, want_flag = ref.build_mask(w.node_offsets, w.parent_offsets, w.parent_idx)
    assert int(flag.item()) == 1 == want_flag
    assert np.array_equal(got, want)


# -------------------------------------------------------------------------------------------- attention
def check_attention(gpu, ref, w, d=None, rows=None, **kw):
    d = d or gpu.DeviceWorkload(w)
    mask_ref, _ = ref.build_mask(w.node_offsets, w.parent_offsets, w.parent_idx)
    mask = d.build_mask()
    assert np.array_equal(gpu.mask_to_numpy(mask), mask_ref)
    out, lse = d.attention(mask, return_lse=True, **kw)
    torch.cuda.synchronize()
    got, got_lse = gpu.out_to_f64(out), lse.cpu().numpy().astype(np.float64)
    tol = TOL[w.cfg.dtype]
    if rows is None:
        want, want_lse = ref.dag_attention(w.q, w.k, w.v, w.kv_offsets, w.prefix_lens, w.node_offsets, mask_ref,
                                           w.softmax_scale, return_lse=True)
    else:
        rb, ri, rh = rows
        want, want_lse = ref.dag_attention(w.q, w.k, w.v, w.kv_offsets, w.prefix_lens, w.node_offsets, mask_ref,
                                           w.softmax_scale, rows=rows, return_lse=True)
        t = w.node_offsets[rb] + ri
        got, got_lse = got[t, rh], got_lse[t, rh]
    err = np.abs(got - want).max()
    lse_err = np.abs(got_lse - want_lse).max()
    print(f"[attn] {w.cfg.name} {kw} max-abs err {err:.3e} lse err {lse_err:.3e}", flush=True)
    assert np.isfinite(got).all()
    assert err <= tol, err
    # the bf16 path folds scale*log2(e) into Q (one more bf16 rounding of Q: relative 2^-9 per element, so a few
    # 1e-3 on a score) and sums bf16-rounded probabilities; its log-sum-exp is an auxiliary output
    assert lse_err <= (1e-4 if w.cfg.dtype == "f32" else 1e-2), lse_err
    return out


def test_attention_config1_fp32(gpu, ref):
    check_attention(gpu, ref, workload(1))


@pytest.mark.parametrize("D", [64, 128])
def test_attention_fp32_general(gpu, ref, D):
    rng = np.random.default_rng(10 + D)
    w = custom_workload(rng, [5, 130, 1, 64], [0, 77, 300, 64], 6, 2, D, "f32")
    check_attention(gpu, ref, w)


@pytest.mark.parametrize("waves", [4, 8, 64])
@pytest.mark.parametrize("splits", [1, 2, 3, 7])
@pytest.mark.parametrize("D", [128, 64])
def test_attention_bf16_small_all_rows(gpu, ref, D, splits, waves):
    """Several row tiles and KV tiles, ragged tails on both axes, GQA, an empty prefix, forced KV splits, both
    work-group shapes (128- and 256-row tiles)."""
    rng = np.random.default_rng(100 + D + splits)
    w = custom_workload(rng, [200, 1, 65, 37], [333, 0, 64, 130], 8, 2, D, "bf16")
    check_attention(gpu, ref, w, num_splits=splits, wg_waves=waves)


def test_attention_bf16_mha_and_odd_group(gpu, ref):
    rng = np.random.default_rng(5)
    check_attention(gpu, ref, custom_workload(rng, [70, 3], [129, 5], 3, 3, 128, "bf16"))     # MHA
    check_attention(gpu, ref, custom_workload(rng, [90, 130], [200, 63], 6, 2, 128, "bf16"))  # group of 3
    check_attention(gpu, ref, custom_workload(rng, [512], [100], 8, 1, 128, "bf16"))          # 4096 rows, 8 words
    check_attention(gpu, ref, custom_workload(rng, [300, 40], [70, 1000], 4, 4, 128, "bf16"), wg_waves=8)


def test_attention_strided_layouts_and_wide_mask_rows(gpu, ref):
    """K/V stored head-major ([Hkv, R, D]) and Q/O with padded rows, reached through the descriptor's strides; mask rows
    wider than the graph needs.  Same numbers as the packed layout, bit for bit."""
    import paper_2407_16207_amd as gsd
    rng = np.random.default_rng(31)
    w = custom_workload(rng, [150, 33], [260, 70], 8, 2, 128, "bf16")
    d = gpu.DeviceWorkload(w)
    mask = d.build_mask(words_per_row=5)
    want = ref.dag_attention(w.q, w.k, w.v, w.kv_offsets, w.prefix_lens, w.node_offsets,
                             ref.build_mask(w.node_offsets, w.parent_offsets, w.parent_idx)[0], w.softmax_scale)
    base = d.attention(mask)
    assert np.abs(gpu.out_to_f64(base) - want).max() <= 2e-2
    k_hm = d.k.permute(1, 0, 2).contiguous().permute(1, 0, 2)          # same values, head-major storage
    v_hm = d.v.permute(1, 0, 2).contiguous().permute(1, 0, 2)
    assert k_hm.stride(1) > k_hm.stride(0)
    q_pad = torch.zeros((d.q.shape[0], d.q.shape[1], 160), dtype=d.q.dtype, device="cuda")[:, :, :128]
    q_pad.copy_(d.q)
    o_pad = torch.zeros_like(q_pad)
    out = gsd.gsd_dag_attention(q_pad, k_hm, v_hm, d.kv_offsets, d.prefix_lens, d.node_offsets, mask, d.max_nodes,
                                d.max_prefix, w.softmax_scale, out=o_pad)
    assert torch.equal(out.contiguous().view(torch.int16), base.view(torch.int16))


def test_attention_chain_equals_causal_sdpa(gpu):
    """A chain-shaped graph is plain causal attention: checked against torch's own SDPA on the GPU in fp32."""
    rng = np.random.default_rng(9)
    n, P, H, D = 150, 100, 4, 128
    w = custom_workload(rng, [n], [P], H, H, D, "bf16")
    w.parent_offsets = np.arange(n + 1, dtype=np.int32)
    w.parent_idx = np.arange(-1, n - 1, dtype=np.int32)
    d = gpu.DeviceWorkload(w)
    out = d.attention(d.build_mask()).float()
    qf = torch.zeros(H, P + n, D, device="cuda")
    qf[:, P:] = d.q.float().permute(1, 0, 2)
    o = torch.nn.functional.scaled_dot_product_attention(qf[None], d.k.float().permute(1, 0, 2)[None],
                                                         d.v.float().permute(1, 0, 2)[None], is_causal=True)[0]
    assert (out - o[:, P:].permute(1, 0, 2)).abs().max().item() <= 2e-2


def sample_rows(w, rng, count, full_seq=None):
    B, N, H = w.cfg.batch, w.cfg.nodes, w.cfg.num_q_heads
    rb, ri, rh = rng.integers(0, B, count), rng.integers(0, N, count), rng.integers(0, H, count)
    if full_seq is not None:
        ii, hh = np.meshgrid(np.arange(N), np.arange(H), indexing="ij")
        rb = np.concatenate([rb, np.full(N * H, full_seq)])
        ri = np.concatenate([ri, ii.ravel()])
        rh = np.concatenate([rh, hh.ravel()])
    return rb.astype(np.int32), ri.astype(np.int32), rh.astype(np.int32)


@pytest.mark.parametrize("cfg_id", [2, 3])
def test_attention_configs_all_rows(gpu, ref, cfg_id):
    check_attention(gpu, ref, workload(cfg_id, with_logits=False))


def test_attention_config4_all_rows(gpu, ref):
    """The headline configuration, in the launch shape the benchmark times: every one of its 2048 x 64 rows against
    the oracle; the same launch again is bit-identical."""
    w = workload(4, with_logits=False)
    d = gpu.DeviceWorkload(w)
    out = check_attention(gpu, ref, w, d=d)
    out2 = d.attention(d.build_mask())
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))


def test_attention_config5_full_size_sampled(gpu, ref):
    """Full-size launch as the benchmark times it; the oracle checks 4096 random (sequence, node, head) rows plus
    every row of one whole sequence (the one with the shortest prefix); then the same-size tree-shaped graph."""
    w = workload(5, with_logits=False)
    rng = np.random.default_rng(5)
    rows = sample_rows(w, rng, 4096, full_seq=int(np.argmin(w.prefix_lens)))
    d = gpu.DeviceWorkload(w)
    out = check_attention(gpu, ref, w, d=d, rows=rows)
    out2 = d.attention(d.build_mask())
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))
    wt = workload(5, with_logits=False, tree=True)
    wt.q, wt.k, wt.v = w.q, w.k, w.v
    check_attention(gpu, ref, wt, rows=sample_rows(wt, rng, 2048))


# ------------------------------------------------------------------------------------- argmax + acceptance
@pytest.mark.parametrize("cfg_id", [1, 2, 3, 4, 5])
def test_argmax_and_accept_configs(gpu, ref, cfg_id):
    w = workload(cfg_id, with_qkv=False)
    d = gpu.DeviceWorkload(w)
    ln, path, bonus, pred = d.accept()
    torch.cuda.synchronize()
    want_pred = ref.node_argmax(w.logits)
    assert np.array_equal(pred.cpu().numpy(), want_pred)
    wl, wp, wb = ref.accept_longest_path(w.node_offsets, w.parent_offsets, w.parent_idx, w.tokens, want_pred,
                                         w.root_pred)
    assert np.array_equal(ln.cpu().numpy(), wl)
    assert np.array_equal(path.cpu().numpy(), wp)
    assert np.array_equal(bonus.cpu().numpy(), wb)
    print(f"[accept] config {cfg_id} accepted lengths {wl.tolist()[:8]}", flush=True)


def test_argmax_edge_rows(gpu, ref):
    import paper_2407_16207_amd as gsd
    rng = np.random.default_rng(1)
    for vocab in (1, 7, 1000, 32000, 32003):
        x = rng.standard_normal((9, vocab)).astype(np.float32)
        x[0, :] = 0.5                              # a whole row of ties
        x[1, vocab - 1] = 9.0
        x[2, 0] = 9.0
        x[3, :] = -np.inf
        x[4, :] = np.nan
        x[5, ::3] = np.nan
        if vocab > 10:
            x[6, [vocab - 2, 5, vocab // 2]] = 7.0
        got = gsd.gsd_node_argmax(torch.from_numpy(x).cuda()).cpu().numpy()
        assert np.array_equal(got, ref.node_argmax(x)), vocab
        xb = f32_to_bf16_bits(x)                   # NaN and -inf survive the rounding
        got = gsd.gsd_node_argmax(gpu.to_dev(xb)).cpu().numpy()
        assert np.array_equal(got, ref.node_argmax(xb)), vocab
    # rows that start off the 16-byte grid (odd row stride)
    big = torch.from_numpy(rng.standard_normal((5, 1003)).astype(np.float32)).cuda()
    view = big[:, 1:1000]
    got = gsd.gsd_node_argmax(view).cpu().numpy()
    assert np.array_equal(got, np.argmax(view.cpu().numpy(), axis=1))


def test_accept_general_dags_with_ties(gpu, ref):
    rng = np.random.default_rng(2024)
    for trial in range(6):
        sizes = [int(x) for x in rng.integers(1, 200, 5)] + [512, 1]
        w = custom_workload(rng, sizes, [0] * len(sizes), 1, 1, 64, "f32", vocab=6, max_parents=4)
        d = gpu.DeviceWorkload(w)
        pred = rng.integers(0, 6, w.total_nodes).astype(np.int32)
        ln, path, bonus, _ = d.accept(logits=False, pred=torch.from_numpy(pred).cuda())
        wl, wp, wb = ref.accept_longest_path(w.node_offsets, w.parent_offsets, w.parent_idx, w.tokens, pred,
                                             w.root_pred)
        assert np.array_equal(ln.cpu().numpy(), wl) and np.array_equal(path.cpu().numpy(), wp)
        assert np.array_equal(bonus.cpu().numpy(), wb)
        assert wl.max() > 1


def test_end_to_end_verify_step_config2(gpu, ref):
    """All three ABI calls back to back on one stream, as one verify step."""
    w = workload(2)
    d = gpu.DeviceWorkload(w)
    mask = d.build_mask()
    out = d.attention(mask)
    ln, path, bonus, pred = d.accept()
    torch.cuda.synchronize()
    mask_ref, _ = ref.build_mask(w.node_offsets, w.parent_offsets, w.parent_idx)
    want = ref.dag_attention(w.q, w.k, w.v, w.kv_offsets, w.prefix_lens, w.node_offsets, mask_ref, w.softmax_scale)
    assert np.abs(gpu.out_to_f64(out) - want).max() <= 2e-2
    wl, wp, wb = ref.accept_longest_path(w.node_offsets, w.parent_offsets, w.parent_idx, w.tokens,
                                         ref.node_argmax(w.logits), w.root_pred)
    assert np.array_equal(ln.cpu().numpy(), wl) and np.array_equal(path.cpu().numpy(), wp)
    assert np.array_equal(bonus.cpu().numpy(), wb)
