"""The allocation-free attention entry point (gsd_dag_attention_static: split-KV partials in the library's static
device array) against gsd_dag_attention on the same inputs, through the C ABI: bit-identical outputs, on two calls in
a row of which the second is smaller (the array keeps the first call's contents), and a descriptor whose partials
exceed the array is refused before anything is launched."""
import numpy as np
import pytest
import torch

import paper_2407_16207_amd as gsd
from paper_2407_16207_amd.workload import VerifyConfig, make_workload

pytestmark = pytest.mark.gpu


def run_both(cfg, seed, num_splits):
    import gpu_util
    w = make_workload(cfg, seed=seed, with_logits=False)
    d = gpu_util.DeviceWorkload(w)
    mask = d.build_mask()
    outs = []
    for static in (False, True):
        out = torch.full_like(d.q, float("nan"))
        lse = torch.full((d.q.shape[0], d.q.shape[1]), float("nan"), dtype=torch.float32, device="cuda")
        desc = gsd.make_attn_desc(d.q, d.k, d.v, d.kv_offsets, d.prefix_lens, d.node_offsets, mask, d.max_nodes,
                                  d.max_prefix, w.softmax_scale, out=out, lse=lse, num_splits=num_splits)
        assert gsd.gsd_dag_attention_splits(desc) == num_splits
        need = gsd.gsd_dag_attention_workspace(desc)
        assert 0 < need <= gsd.GSD_STATIC_SCRATCH_BYTES
        if static:
            gsd.gsd_dag_attention_static(desc)          # no workspace in the descriptor
        else:
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            desc.workspace, desc.workspace_bytes = ws.data_ptr(), need
            gsd.gsd_dag_attention_desc(desc)
        torch.cuda.synchronize()
        outs.append((out, lse))
    (o0, l0), (o1, l1) = outs
    assert torch.isfinite(o1.float()).all() and torch.isfinite(l1).all()
    assert torch.equal(o0.view(torch.int16), o1.view(torch.int16))
    assert torch.equal(l0, l1)
    return w, d, mask, o1


def test_static_scratch_matches_workspace_entry_point(ref):
    big = VerifyConfig("no-alloc-a", 2, 8, 2, 128, 700, 900, 10, 8, 3, 8, 0.5, "bf16")
    small = VerifyConfig("no-alloc-b", 1, 4, 4, 128, 200, 200, 3, 8, 2, 8, 0.5, "bf16")
    w, d, mask, out = run_both(big, 11, 4)
    # and against the oracle, once
    mask_ref, _ = ref.build_mask(w.node_offsets, w.parent_offsets, w.parent_idx)
    want = ref.dag_attention(w.q, w.k, w.v, w.kv_offsets, w.prefix_lens, w.node_offsets, mask_ref, w.softmax_scale)
    assert np.abs(out.float().cpu().numpy().astype(np.float64) - want).max() <= 2e-2
    run_both(small, 12, 3)                              # second call, smaller, same array


def test_static_scratch_refuses_what_does_not_fit():
    import gpu_util
    cfg = VerifyConfig("no-alloc-c", 4, 32, 32, 128, 600, 600, 16, 8, 2, 8, 0.5, "bf16")
    w = make_workload(cfg, seed=13, with_logits=False)
    d = gpu_util.DeviceWorkload(w)
    mask = d.build_mask()
    out = torch.zeros_like(d.q)
    desc = gsd.make_attn_desc(d.q, d.k, d.v, d.kv_offsets, d.prefix_lens, d.node_offsets, mask, d.max_nodes,
                              d.max_prefix, w.softmax_scale, out=out, num_splits=10)
    assert gsd.gsd_dag_attention_workspace(desc) > gsd.GSD_STATIC_SCRATCH_BYTES
    with pytest.raises(gsd.GsdError) as e:
        gsd.gsd_dag_attention_static(desc)
    assert e.value.status == gsd.GSD_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert not out.any()                                # nothing ran
