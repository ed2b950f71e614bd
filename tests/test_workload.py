"""The seeded input generators: determinism, shapes and the structure the configs call for."""
import numpy as np

from paper_2407_16207_amd.workload import (CONFIGS, make_workload, f32_to_bf16_bits, bf16_bits_to_f32)


def test_bf16_rounding_is_nearest_even():
    import torch
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 37.0
    ours = f32_to_bf16_bits(x)
    theirs = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, theirs)
    assert np.array_equal(bf16_bits_to_f32(ours), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_config_shapes_and_structure():
    for cid in (1, 2, 3):
        cfg = CONFIGS[cid]
        w = make_workload(cid)
        w2 = make_workload(cid)
        T = cfg.batch * cfg.nodes
        assert w.q.shape == (T, cfg.num_q_heads, cfg.head_dim)
        assert w.k.shape == (int(w.prefix_lens.sum()) + T, cfg.num_kv_heads, cfg.head_dim) == w.v.shape
        assert w.logits.shape == (T, cfg.vocab)
        assert w.q.dtype == (np.float32 if cfg.dtype == "f32" else np.uint16)
        for a, b in ((w.q, w2.q), (w.k, w2.k), (w.logits, w2.logits), (w.parent_idx, w2.parent_idx), (w.tokens, w2.tokens)):
            assert np.array_equal(a, b)
        for t in range(T):
            i = t % cfg.nodes
            ps = w.parent_idx[w.parent_offsets[t]:w.parent_offsets[t + 1]]
            layer = i // cfg.width
            if layer == 0:
                assert ps.tolist() == [-1]
            else:
                assert 1 <= len(ps) <= cfg.max_parents and len(set(ps.tolist())) == len(ps)
                assert all((layer - 1) * cfg.width <= p < layer * cfg.width for p in ps)
        for b in range(cfg.batch):
            for layer in range(cfg.layers):
                lo = b * cfg.nodes + layer * cfg.width
                assert len(set(w.tokens[lo:lo + cfg.width].tolist())) == cfg.width


def test_tree_variant_keeps_first_parent_only():
    w = make_workload(3, with_logits=False, with_qkv=False)
    t = make_workload(3, tree=True, with_logits=False, with_qkv=False)
    assert np.array_equal(w.tokens, t.tokens)
    assert np.all(np.diff(t.parent_offsets) == 1)
    firsts = w.parent_idx[w.parent_offsets[:-1]]
    assert np.array_equal(t.parent_idx, firsts)


def test_ragged_prefix_lengths_config5_shape_only():
    cfg = CONFIGS[5]
    w = make_workload(5, with_logits=False, with_qkv=False)
    assert w.prefix_lens.min() >= 1024 and w.prefix_lens.max() <= 8192 and len(set(w.prefix_lens.tolist())) > 16
    assert w.kv_offsets[1] == w.prefix_lens[0] + cfg.nodes
