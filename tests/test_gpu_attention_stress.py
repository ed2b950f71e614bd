"""GPU parity of the bf16 attention kernel on peaked inputs: score distributions under which the row offset of the
kernel's softmax has to move (large sums raise it) or cannot follow (the row is computed again by the kernel's exact
path).  Every row of every case is compared with the fp64 oracle, max-abs <= 2e-2, over the three work-group shapes and
with and without KV splits.  A small numpy model of the kernel's documented offset policy (first tile's max, then
the per-lane tile sums against 2^14 / 2^64 / 2^-64) only asserts that each input really reaches the path it is meant
for; it takes no part in the comparison.

Values of V are clipped to [-3, 3] here: with one dominant key the output is that key's V row, and bf16 rounding of
the probability and of the output (2^-9 relative each) alone approaches the absolute tolerance beyond |v| ~ 5."""
import numpy as np
import pytest
import torch

from paper_2407_16207_amd.workload import VerifyConfig, Workload, bf16_bits_to_f32, f32_to_bf16_bits, random_dag

pytestmark = pytest.mark.gpu

LOG2E = 1.4426950408889634


@pytest.fixture(scope="module")
def gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import gpu_util
    return gpu_util


def base_workload(rng, sizes, prefixes, Hq, Hkv, D, scale_mult=1.0, roots_only=False):
    B = len(sizes)
    node_offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    offs, pars, e = [np.zeros(1, dtype=np.int32)], [], 0
    for n in sizes:
        if roots_only:                      # every node hangs off the root: a row sees the prefix and itself only
            o, p = np.arange(n + 1, dtype=np.int32), np.full(n, -1, dtype=np.int32)
        else:
            o, p = random_dag(rng, n, 3)
        offs.append(o[1:] + e)
        pars.append(p)
        e += len(p)
    T = int(node_offsets[-1])
    prefix_lens = np.asarray(prefixes, dtype=np.int32)
    rows = prefix_lens.astype(np.int64) + np.asarray(sizes)
    kv_offsets = np.concatenate([[0], np.cumsum(rows)[:-1]]).astype(np.int64)
    R = int(rows.sum())
    cfg = VerifyConfig("stress", B, Hq, Hkv, D, int(min(prefixes)), int(max(prefixes)), 1, max(sizes), 3, 8, 0.5, "bf16")
    q = rng.standard_normal((T, Hq, D), dtype=np.float32)
    k = rng.standard_normal((R, Hkv, D), dtype=np.float32)
    v = np.clip(rng.standard_normal((R, Hkv, D), dtype=np.float32), -3.0, 3.0)
    return Workload(cfg=cfg, seed=0, node_offsets=node_offsets, parent_offsets=np.concatenate(offs).astype(np.int32),
                    parent_idx=np.concatenate(pars).astype(np.int32), tokens=np.zeros(T, dtype=np.int32),
                    root_pred=np.zeros(B, dtype=np.int32), prefix_lens=prefix_lens, kv_offsets=kv_offsets,
                    q=q, k=k, v=v, logits=np.zeros((0, 8), dtype=np.float32),
                    softmax_scale=float(scale_mult / np.sqrt(D)))


def finish(w):
    """Round Q, K, V to bf16 bit patterns (what both sides read)."""
    w.q, w.k, w.v = f32_to_bf16_bits(w.q), f32_to_bf16_bits(w.k), f32_to_bf16_bits(w.v)
    return w


def policy_events(w, mask_bool_rows):
    """Which rows of an unsplit launch raise their offset at least once, and which are handed to the exact path,
    under the kernel's documented policy (prefix >= 1 assumed, so that tile 0 sets every row's offset)."""
    q, k = bf16_bits_to_f32(w.q).astype(np.float64), bf16_bits_to_f32(w.k).astype(np.float64)
    G = w.cfg.num_q_heads // w.cfg.num_kv_heads
    raised = exact = rows = 0
    for b in range(w.cfg.batch):
        P, n0, n1 = int(w.prefix_lens[b]), int(w.node_offsets[b]), int(w.node_offsets[b + 1])
        kb = k[w.kv_offsets[b]:w.kv_offsets[b] + P + (n1 - n0)]
        for h in range(w.cfg.num_q_heads):
            s = q[n0:n1, h] @ kb[:, h // G].T * (w.softmax_scale * LOG2E)          # [n, P + n] in the exponent's units
            s[:, P:][~mask_bool_rows[n0:n1, :n1 - n0]] = -np.inf
            pad_p, pad_d = (-P) % 64, (-(n1 - n0)) % 64
            s = np.concatenate([s[:, :P], np.full((s.shape[0], pad_p), -np.inf), s[:, P:],
                                np.full((s.shape[0], pad_d), -np.inf)], axis=1)
            tiles = s.reshape(s.shape[0], -1, 2, 2, 2, 8)                          # key = 32a + 16b + 8*half + c
            offset = tiles[:, 0].max(axis=(1, 2, 3, 4))
            was_raised = np.zeros(s.shape[0], dtype=bool)
            flagged = np.zeros(s.shape[0], dtype=bool)
            total = np.zeros(s.shape[0])
            with np.errstate(over="ignore", invalid="ignore"):
                for ti in range(tiles.shape[1]):
                    per_lane = np.exp2(tiles[:, ti] - offset[:, None, None, None, None]).sum(axis=(1, 2, 4))   # [n, half]
                    bad = ~(per_lane < 2.0 ** 64)
                    flagged |= bad.any(axis=1)
                    big = np.where(bad, 0.0, per_lane).max(axis=1)
                    delta = np.where(big >= 2.0 ** 14, np.frexp(big)[1], 0)
                    total = (total + np.where(bad, 0.0, per_lane).sum(axis=1)) * np.exp2(-delta.astype(np.float64))
                    offset = offset + delta
                    was_raised |= delta > 0
            flagged |= ~(total >= 2.0 ** -64)
            raised += int((was_raised & ~flagged).sum())
            exact += int(flagged.sum())
            rows += s.shape[0]
    return raised, exact, rows


def run_case(gpu, ref, w, expect_raised=None, expect_exact=None, shapes=(0, 4, 8, 64), splits=(1, 3)):
    from helpers import mask_to_bool
    d = gpu.DeviceWorkload(w)
    mask_ref, _ = ref.build_mask(w.node_offsets, w.parent_offsets, w.parent_idx)
    if expect_raised is not None or expect_exact is not None:
        raised, exact, rows = policy_events(w, mask_to_bool(mask_ref, w.max_nodes))
        print(f"[stress] {rows} rows: {raised} raise their offset, {exact} take the exact path", flush=True)
        if expect_raised is not None:
            assert (raised > 0) == expect_raised, (raised, rows)
        if expect_exact is not None:
            assert (exact > 0) == expect_exact, (exact, rows)
    want, want_lse = ref.dag_attention(w.q, w.k, w.v, w.kv_offsets, w.prefix_lens, w.node_offsets, mask_ref,
                                       w.softmax_scale, return_lse=True)
    mask = d.build_mask()
    for waves in shapes:
        for ns in splits:
            out, lse = d.attention(mask, return_lse=True, wg_waves=waves, num_splits=ns)
            torch.cuda.synchronize()
            got = gpu.out_to_f64(out)
            assert np.isfinite(got).all(), (waves, ns)
            err = np.abs(got - want).max()
            lse_err = np.abs(lse.cpu().numpy().astype(np.float64) - want_lse).max()
            print(f"[stress] wg_waves {waves} splits {ns}: max-abs err {err:.3e}, lse err {lse_err:.3e}", flush=True)
            assert err <= 2e-2, (waves, ns, err)
            assert lse_err <= 1e-2, (waves, ns, lse_err)


SIZES, PREFIXES = [200, 70, 130], [1100, 300, 650]


def test_row_max_climbs_along_the_prefix(gpu, ref):
    """K rows grow along the sequence, so every row's max climbs by more than 8 (log2) every few tiles."""
    rng = np.random.default_rng(41)
    w = base_workload(rng, SIZES, PREFIXES, 8, 2, 128)
    for b in range(w.cfg.batch):
        lo, n_rows = int(w.kv_offsets[b]), int(w.prefix_lens[b]) + SIZES[b]
        w.k[lo:lo + n_rows] *= (1.0 + 9.0 * np.arange(n_rows, dtype=np.float32) / n_rows)[:, None, None]
    run_case(gpu, ref, finish(w), expect_raised=True, expect_exact=False)


def test_softmax_scale_eight_times_larger(gpu, ref):
    rng = np.random.default_rng(42)
    w = base_workload(rng, SIZES, PREFIXES, 8, 2, 128, scale_mult=8.0)
    run_case(gpu, ref, finish(w), expect_raised=True, expect_exact=False)


def test_late_outlier_keys_in_prefix_and_draft(gpu, ref):
    """One key late in the prefix and one draft key (visible to its descendants only, i.e. to some rows of a wave
    and not to others) line up with particular queries: a jump of ~30 (log2) for those rows, none for the rest."""
    rng = np.random.default_rng(43)
    w = base_workload(rng, SIZES, PREFIXES, 8, 2, 128)
    for b in range(w.cfg.batch):
        lo, P, n0 = int(w.kv_offsets[b]), int(w.prefix_lens[b]), int(w.node_offsets[b])
        w.k[lo + P - 70, 0] = 2.0 * w.q[n0 + 5, 1]                 # late prefix key, aimed at (node 5, head 1)
        w.k[lo + P - 3, 1] = 2.0 * w.q[n0 + 9, 6]
        w.k[lo + P + 40, 0] = 2.0 * w.q[n0 + SIZES[b] - 1, 2]      # draft node 40's key, aimed at the last node
        w.k[lo + P + 66 % SIZES[b], 1] = 2.5 * w.q[n0 + SIZES[b] - 2, 5]
    run_case(gpu, ref, finish(w), expect_raised=True, expect_exact=False)


def test_scores_span_more_than_100_log2_gradually(gpu, ref):
    """The max climbs by well over 100 (log2) across the prefix in steps the offset can follow: early keys end up
    far below anything fp32 can hold next to the late ones."""
    rng = np.random.default_rng(44)
    w = base_workload(rng, SIZES, PREFIXES, 4, 1, 128, scale_mult=4.0)
    for b in range(w.cfg.batch):
        lo, n_rows = int(w.kv_offsets[b]), int(w.prefix_lens[b]) + SIZES[b]
        w.k[lo:lo + n_rows] *= (0.25 + 8.0 * np.arange(n_rows, dtype=np.float32) / n_rows)[:, None, None]
    run_case(gpu, ref, finish(w), expect_raised=True)      # (a few rows jump too far in one tile and go the exact way)


def test_jump_beyond_what_the_offset_can_follow_takes_the_exact_path(gpu, ref):
    """A late key scores ~130 (log2) above everything before it for a few rows: those rows are computed again by the
    kernel's exact path; their neighbours in the same wave are not disturbed."""
    rng = np.random.default_rng(45)
    w = base_workload(rng, SIZES, PREFIXES, 8, 2, 128)
    for b in range(w.cfg.batch):
        lo, P, n0 = int(w.kv_offsets[b]), int(w.prefix_lens[b]), int(w.node_offsets[b])
        w.k[lo + P - 100, 0] = 8.0 * w.q[n0 + 3, 0]
        w.k[lo + P + 10, 1] = 8.0 * w.q[n0 + SIZES[b] - 1, 7]      # in a draft tile
    run_case(gpu, ref, finish(w), expect_exact=True)


def test_scores_far_below_the_first_guess(gpu, ref):
    """No prefix and every node a child of the root: a row sees its own key only, which for most rows is not in the
    first tile its work-group walks, and scores ~ -100 (log2): far below the offset guessed without it.  Then the same
    with a prefix whose keys all score below -128 (log2) while the first tile sets the offset."""
    rng = np.random.default_rng(46)
    w = base_workload(rng, [300, 64, 65], [0, 0, 0], 2, 2, 128, roots_only=True)
    for b in range(w.cfg.batch):
        lo, n0, n = int(w.kv_offsets[b]), int(w.node_offsets[b]), int(w.node_offsets[b + 1] - w.node_offsets[b])
        w.k[lo:lo + n] = -6.0 * w.q[n0:n0 + n]
    run_case(gpu, ref, finish(w))
    w = base_workload(rng, [100, 40], [200, 64], 4, 2, 128)
    base = rng.standard_normal(128).astype(np.float32)
    w.q[:] = 4.0 * base + 0.1 * w.q
    w.k[:] = -4.0 * base + 0.1 * w.k           # every score ~ -4*4*128/sqrt(128)*log2(e) ~ -260
    run_case(gpu, ref, finish(w), expect_exact=False)


def test_head_dim_64_climb_and_jump(gpu, ref):
    rng = np.random.default_rng(47)
    w = base_workload(rng, [150, 40], [500, 129], 4, 2, 64, scale_mult=3.0)
    for b in range(w.cfg.batch):
        lo, P, n0 = int(w.kv_offsets[b]), int(w.prefix_lens[b]), int(w.node_offsets[b])
        n_rows = P + int(w.node_offsets[b + 1]) - n0
        w.k[lo:lo + n_rows] *= (0.5 + 5.0 * np.arange(n_rows, dtype=np.float32) / n_rows)[:, None, None]
        w.k[lo + P - 20, 0] = 12.0 * w.q[n0 + 7, 1]
    run_case(gpu, ref, finish(w), expect_raised=True, expect_exact=True)
