"""The C ABI without a GPU: the library loads, exports every declared symbol, and rejects bad arguments on the
host before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2407_16207_amd as gsd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(gsd.LIB_PATH):
        from paper_2407_16207_amd.build import build_library
        build_library()
    return gsd.load_library()


def declared_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):      # gsd.h and the measurement aids beside it
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(gsd_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(gsd.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None
    assert lib.gsd_version().decode().startswith("gsd-gfx950")
    assert lib.gsd_status_string(0) == b"ok" and lib.gsd_status_string(4) == b"workspace too small"


def good_desc():
    d = gsd.AttnDesc()
    d.batch, d.total_nodes, d.max_nodes, d.max_prefix = 2, 128, 64, 1024
    d.num_q_heads, d.num_kv_heads, d.head_dim, d.dtype = 8, 2, 128, gsd.GSD_BF16
    d.words_per_row, d.num_splits, d.softmax_scale = 1, 0, 0.088
    for f in ("q", "o", "k", "v", "kv_offsets", "prefix_lens", "node_offsets", "mask"):
        setattr(d, f, 0x10000)
    d.q_token_stride = d.o_token_stride = 8 * 128
    d.kv_token_stride = 2 * 128
    d.q_head_stride = d.o_head_stride = d.kv_head_stride = 128
    return d


def test_attention_descriptor_validation(lib):
    null = ctypes.c_void_p(0)
    d = good_desc()
    assert lib.gsd_dag_attention_splits(ctypes.byref(d)) >= 1
    need = lib.gsd_dag_attention_workspace(ctypes.byref(d))
    splits = lib.gsd_dag_attention_splits(ctypes.byref(d))
    assert need == (0 if splits == 1 else splits * 128 * 8 * (128 + 2) * 4)
    # a split run without workspace is refused on the host
    d.num_splits = 4
    assert lib.gsd_dag_attention_workspace(ctypes.byref(d)) == 4 * 128 * 8 * 130 * 4
    assert lib.gsd_dag_attention(ctypes.byref(d), null) == gsd.GSD_ERR_WORKSPACE
    assert b"workspace" in lib.gsd_last_error()
    cases = [("num_kv_heads", 3, gsd.GSD_ERR_INVALID_ARG), ("head_dim", 96, gsd.GSD_ERR_UNSUPPORTED),
             ("dtype", 7, gsd.GSD_ERR_UNSUPPORTED), ("batch", 0, gsd.GSD_ERR_INVALID_ARG),
             ("words_per_row", 0, gsd.GSD_ERR_INVALID_ARG), ("max_nodes", 100000, gsd.GSD_ERR_UNSUPPORTED),
             ("q", None, gsd.GSD_ERR_INVALID_ARG), ("mask", None, gsd.GSD_ERR_INVALID_ARG),
             ("k", 0x10002, gsd.GSD_ERR_INVALID_ARG), ("kv_token_stride", 100, gsd.GSD_ERR_INVALID_ARG),
             ("softmax_scale", 0.0, gsd.GSD_ERR_INVALID_ARG), ("num_splits", -1, gsd.GSD_ERR_INVALID_ARG)]
    for field, value, code in cases:
        d = good_desc()
        setattr(d, field, value)
        assert lib.gsd_dag_attention(ctypes.byref(d), null) == code, field
        assert lib.gsd_last_error() != b""
    assert lib.gsd_dag_attention(None, null) == gsd.GSD_ERR_INVALID_ARG
    d = good_desc()
    d.head_dim = 96
    assert lib.gsd_dag_attention_workspace(ctypes.byref(d)) == ctypes.c_size_t(-1).value
    assert lib.gsd_dag_attention_splits(ctypes.byref(d)) == -1


def test_other_entry_points_validate(lib):
    p = ctypes.c_void_p(0x10000)
    null = ctypes.c_void_p(0)
    assert lib.gsd_build_mask(0, 16, 1, p, p, p, p, null, null) == gsd.GSD_ERR_INVALID_ARG
    assert lib.gsd_build_mask(1, 65, 1, p, p, p, p, null, null) == gsd.GSD_ERR_INVALID_ARG      # words too few
    assert lib.gsd_build_mask(1, 513, 9, p, p, p, p, null, null) == gsd.GSD_ERR_UNSUPPORTED
    assert lib.gsd_build_mask(1, 16, 1, p, null, p, p, null, null) == gsd.GSD_ERR_INVALID_ARG
    assert lib.gsd_node_argmax(0, 10, 0, p, 10, p, null) == gsd.GSD_ERR_INVALID_ARG
    assert lib.gsd_node_argmax(4, 10, 0, p, 9, p, null) == gsd.GSD_ERR_INVALID_ARG               # stride < vocab
    assert lib.gsd_node_argmax(4, 10, 5, p, 10, p, null) == gsd.GSD_ERR_UNSUPPORTED
    assert lib.gsd_node_argmax(4, 10, 0, null, 10, p, null) == gsd.GSD_ERR_INVALID_ARG
    args = [1, 16, 16, p, p, p, p, null, 0, 0, 0, p, p, p, p, p, null]
    bad = list(args)
    bad[11] = null                                                                               # pred missing
    assert lib.gsd_accept_longest_path(*bad) == gsd.GSD_ERR_INVALID_ARG
    bad = list(args)
    bad[2] = 4096
    assert lib.gsd_accept_longest_path(*bad) == gsd.GSD_ERR_UNSUPPORTED
    bad = list(args)
    bad[7], bad[8], bad[9], bad[10] = p, 0, 0, 0                                                 # logits with vocab 0
    assert lib.gsd_accept_longest_path(*bad) == gsd.GSD_ERR_INVALID_ARG


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(gsd, "_lib", None)
    monkeypatch.setattr(gsd, "LIB_PATH", "/nonexistent/libgsd.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        gsd.load_library()


def test_unmerge_gather_commit_validate(lib):
    p = ctypes.c_void_p(0x10000)
    q = ctypes.c_void_p(0x20000)
    null = ctypes.c_void_p(0)
    good = [2, 64, 128, p, p, p, p, p, null, p, p, null, null]
    for pos, value, code in ((0, 0, gsd.GSD_ERR_INVALID_ARG), (1, 513, gsd.GSD_ERR_UNSUPPORTED),
                             (2, 0, gsd.GSD_ERR_INVALID_ARG), (2, 1 << 30, gsd.GSD_ERR_UNSUPPORTED),
                             (6, null, gsd.GSD_ERR_INVALID_ARG), (10, null, gsd.GSD_ERR_INVALID_ARG)):
        bad = list(good)
        bad[pos] = value
        assert lib.gsd_unmerge_to_tree(*bad) == code, pos
    good = [10, 64, p, 100, 64, p, q, 64, null]
    for pos, value in ((0, 0), (1, 6), (1, 2), (4, 60), (7, 32), (2, null), (5, null), (6, ctypes.c_void_p(0x20002))):
        bad = list(good)
        bad[pos] = value
        assert lib.gsd_gather_rows(*bad) == gsd.GSD_ERR_INVALID_ARG, pos
    good = [2, 64, 4, 2048, p, q, 2048, 1 << 20, p, p, p, p, q, null]
    for pos, value, code in ((0, 0, gsd.GSD_ERR_INVALID_ARG), (2, 0, gsd.GSD_ERR_INVALID_ARG),
                             (1, 513, gsd.GSD_ERR_UNSUPPORTED),
                             (2, 70000, gsd.GSD_ERR_UNSUPPORTED), (3, 2040, gsd.GSD_ERR_INVALID_ARG),
                             (6, 1024, gsd.GSD_ERR_INVALID_ARG), (7, 1000, gsd.GSD_ERR_INVALID_ARG),
                             (4, ctypes.c_void_p(0x10008), gsd.GSD_ERR_INVALID_ARG), (12, p, gsd.GSD_ERR_INVALID_ARG),
                             (11, null, gsd.GSD_ERR_INVALID_ARG)):
        bad = list(good)
        bad[pos] = value
        assert lib.gsd_commit_kv(*bad) == code, pos


def test_stochastic_entry_points_validate(lib):
    p = ctypes.c_void_p(0x10000)
    null = ctypes.c_void_p(0)
    assert lib.gsd_softmax_stats(0, 10, 0, p, 10, p, p, null) == gsd.GSD_ERR_INVALID_ARG
    assert lib.gsd_node_argmax_stats(0, 10, 0, p, 10, p, p, p, null) == gsd.GSD_ERR_INVALID_ARG
    assert lib.gsd_node_argmax_stats(4, 10, 0, p, 10, p, null, p, null) == gsd.GSD_ERR_INVALID_ARG
    assert lib.gsd_node_argmax_stats(4, 10, 7, p, 10, p, p, p, null) == gsd.GSD_ERR_UNSUPPORTED
    assert lib.gsd_node_argmax_stats(4, 10, 1, p, 9, p, p, p, null) == gsd.GSD_ERR_INVALID_ARG
    assert lib.gsd_softmax_stats(4, 10, 0, p, 9, p, p, null) == gsd.GSD_ERR_INVALID_ARG
    assert lib.gsd_softmax_stats(4, 10, 3, p, 10, p, p, null) == gsd.GSD_ERR_UNSUPPORTED
    assert lib.gsd_softmax_stats(4, 10, 0, p, 10, null, p, null) == gsd.GSD_ERR_INVALID_ARG
    assert lib.gsd_accept_stochastic(None, null) == gsd.GSD_ERR_INVALID_ARG

    def good():
        d = gsd.StochasticDesc()
        d.batch, d.total_nodes, d.max_nodes, d.vocab, d.dtype, d.row_stride = 2, 64, 32, 1000, gsd.GSD_BF16, 1000
        for name, _ in gsd.StochasticDesc._fields_:
            if getattr(d, name) is None:
                setattr(d, name, 0x10000)
        return d
    for field, value, code in (("batch", 0, gsd.GSD_ERR_INVALID_ARG), ("max_nodes", 1000, gsd.GSD_ERR_UNSUPPORTED),
                               ("dtype", 9, gsd.GSD_ERR_UNSUPPORTED), ("row_stride", 999, gsd.GSD_ERR_INVALID_ARG),
                               ("end_node", None, gsd.GSD_ERR_INVALID_ARG), ("draft_logits", None, gsd.GSD_ERR_INVALID_ARG),
                               ("logits", 0x10001, gsd.GSD_ERR_INVALID_ARG)):
        d = good()
        setattr(d, field, value)
        assert lib.gsd_accept_stochastic(ctypes.byref(d), null) == code, field
