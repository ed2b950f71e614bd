"""Helpers for the GPU parity tests: move a seeded workload to the device and run the library on it."""
import numpy as np
import torch

import paper_2407_16207_amd as gsd


def to_dev(a: np.ndarray):
    if a.dtype == np.uint16:                       # bf16 bit patterns
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


class DeviceWorkload:
    def __init__(self, w):
        self.w = w
        self.node_offsets = to_dev(w.node_offsets)
        self.parent_offsets = to_dev(w.parent_offsets)
        self.parent_idx = to_dev(w.parent_idx if len(w.parent_idx) else np.zeros(1, dtype=np.int32))
        self.tokens = to_dev(w.tokens)
        self.root_pred = to_dev(w.root_pred)
        self.prefix_lens = to_dev(w.prefix_lens)
        self.kv_offsets = to_dev(w.kv_offsets)
        self.q = to_dev(w.q) if w.q.size else None
        self.k = to_dev(w.k) if w.k.size else None
        self.v = to_dev(w.v) if w.v.size else None
        self.logits = to_dev(w.logits) if w.logits.size else None
        self.max_nodes = w.max_nodes
        self.max_prefix = int(w.prefix_lens.max())

    def build_mask(self, words_per_row=None, flag=None):
        return gsd.gsd_build_mask(self.node_offsets, self.parent_offsets, self.parent_idx, self.max_nodes,
                                  words_per_row=words_per_row, dag_error_flag=flag)

    def attention(self, mask, **kw):
        return gsd.gsd_dag_attention(self.q, self.k, self.v, self.kv_offsets, self.prefix_lens, self.node_offsets,
                                     mask, self.max_nodes, self.max_prefix, self.w.softmax_scale, **kw)

    def accept(self, logits=True, pred=None):
        return gsd.gsd_accept_longest_path(self.node_offsets, self.parent_offsets, self.parent_idx, self.tokens,
                                           self.root_pred, self.max_nodes,
                                           logits=self.logits if logits else None, pred=pred)


def mask_to_numpy(mask_t) -> np.ndarray:
    return mask_t.cpu().numpy().view(np.uint64)


def out_to_f64(o) -> np.ndarray:
    return o.float().cpu().numpy().astype(np.float64)
