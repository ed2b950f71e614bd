"""Host-side pieces of bench.py that need no GPU: the one-GPU contract, the algorithmic flop count behind
`roofline.achieved` (Section 4.1: a node attends to the context and to its ancestors, so the work is 4 * head_dim flops
per (query row, visible key) pair), the peaks the fractions are priced against, and the committed traffic figure."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from paper_2407_16207_amd.workload import make_workload  # noqa: E402
from oracle import gsd_ref  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)


def test_peaks_are_the_published_ones():
    assert bench.MFMA_BF16_PEAK_TFLOPS == 2500.0 and bench.HBM_PEAK_GBS == 8000.0


def test_popcount_rows_counts_visible_draft_nodes():
    rng = np.random.default_rng(3)
    words = rng.integers(0, 2**63, size=(37, 5), dtype=np.int64).astype(np.uint64)
    words[0] = 0
    words[1] = np.uint64(2**64 - 1)
    want = [sum(bin(int(x)).count("1") for x in row) for row in words]
    assert bench.popcount_rows(words).tolist() == want


def test_algorithmic_flops_of_config_1_by_direct_count():
    """The bench's formula, 4 D Hq sum(P_b + visible draft nodes), against a count of the (query row, key) pairs that
    the oracle's mask lets through on the small config."""
    w = make_workload(1)
    cfg = w.cfg
    mask, _ = gsd_ref.build_mask(w.node_offsets, w.parent_offsets, w.parent_idx)
    vis = bench.popcount_rows(np.ascontiguousarray(mask).view(np.uint64))
    per_node_keys = np.repeat(w.prefix_lens.astype(np.int64), np.diff(w.node_offsets)) + vis
    flops = 4.0 * cfg.head_dim * cfg.num_q_heads * float(per_node_keys.sum())
    pairs = 0
    for b in range(cfg.batch):
        lo, hi = int(w.node_offsets[b]), int(w.node_offsets[b + 1])
        for i in range(lo, hi):
            row = mask[i]
            visible = sum(1 for j in range(hi - lo) if (int(row[j // 64]) >> (j % 64)) & 1)
            pairs += cfg.num_q_heads * (int(w.prefix_lens[b]) + visible)
    assert flops == 4.0 * cfg.head_dim * pairs


def test_committed_traffic_figure_is_read_and_plausible():
    """roofline.traffic comes from the committed counter summary; it has to be there and close to the algorithmic
    bytes of config 4 (Q + O + K + V + mask, every byte once)."""
    t = bench.measured_traffic("cfg4-llama2-70b-shaped-gqa")
    assert t is not None
    T, Hq, Hkv, D, P, N, B, W = 2048, 64, 8, 128, 4096, 256, 8, 4
    algorithmic = 2 * T * Hq * D * 2 + 2 * B * (P + N) * Hkv * D * 2 + T * W * 8
    assert 0.95 * algorithmic <= t <= 1.10 * algorithmic, (t, algorithmic)
