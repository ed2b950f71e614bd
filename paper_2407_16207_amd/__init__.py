"""Thin Python binding of libgsd (include/gsd.h): the MI355X verification hot path of Graph-structured
Speculative Decoding.  Argument marshalling only: torch supplies device memory and the stream, every step of
the path runs in the library's HIP kernels.  There is no CPU fallback; a missing library raises.

    gsd_build_mask, gsd_dag_attention, gsd_node_argmax, gsd_accept_longest_path,
    gsd_unmerge_to_tree, gsd_gather_rows, gsd_commit_kv, gsd_softmax_stats, gsd_accept_stochastic,
    gsd_build_token_graph

mirror the C entry points of the same names.
"""
from __future__ import annotations

import ctypes
import os

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libgsd.so")

GSD_OK = 0
GSD_ERR_INVALID_ARG, GSD_ERR_UNSUPPORTED, GSD_ERR_WORKSPACE, GSD_ERR_HIP = 1, 3, 4, 5
GSD_F32, GSD_BF16 = 0, 1
GSD_MAX_NODES_PER_SEQ = 512
GSD_STATIC_SCRATCH_BYTES = 32 << 20

EXPORTS = ("gsd_status_string", "gsd_last_error", "gsd_version", "gsd_build_mask", "gsd_dag_attention_workspace",
           "gsd_dag_attention_splits", "gsd_dag_attention", "gsd_dag_attention_static", "gsd_node_argmax", "gsd_node_argmax_stats", "gsd_accept_longest_path",
           "gsd_unmerge_to_tree", "gsd_gather_rows", "gsd_commit_kv", "gsd_softmax_stats", "gsd_accept_stochastic",
           "gsd_build_token_graph")


class GsdError(RuntimeError):
    def __init__(self, status: int, detail: str):
        super().__init__(f"libgsd status {status}: {detail}")
        self.status = status


class AttnDesc(ctypes.Structure):
    """Mirror of struct gsd_attn_desc."""
    _fields_ = [
        ("batch", ctypes.c_int32), ("total_nodes", ctypes.c_int32), ("max_nodes", ctypes.c_int32),
        ("max_prefix", ctypes.c_int32), ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32), ("words_per_row", ctypes.c_int32),
        ("num_splits", ctypes.c_int32), ("softmax_scale", ctypes.c_float), ("wg_waves", ctypes.c_int32),
        ("q", ctypes.c_void_p), ("o", ctypes.c_void_p), ("lse", ctypes.c_void_p), ("k", ctypes.c_void_p),
        ("v", ctypes.c_void_p), ("kv_offsets", ctypes.c_void_p), ("prefix_lens", ctypes.c_void_p),
        ("node_offsets", ctypes.c_void_p), ("mask", ctypes.c_void_p),
        ("q_token_stride", ctypes.c_int64), ("q_head_stride", ctypes.c_int64),
        ("o_token_stride", ctypes.c_int64), ("o_head_stride", ctypes.c_int64),
        ("kv_token_stride", ctypes.c_int64), ("kv_head_stride", ctypes.c_int64),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
    ]


class StochasticDesc(ctypes.Structure):
    """Mirror of struct gsd_stochastic_desc."""
    _fields_ = [
        ("batch", ctypes.c_int32), ("total_nodes", ctypes.c_int32), ("max_nodes", ctypes.c_int32),
        ("vocab", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("node_offsets", ctypes.c_void_p), ("parent_offsets", ctypes.c_void_p), ("parent_idx", ctypes.c_void_p),
        ("tokens", ctypes.c_void_p), ("logits", ctypes.c_void_p), ("root_logits", ctypes.c_void_p),
        ("draft_logits", ctypes.c_void_p), ("root_draft_logits", ctypes.c_void_p), ("row_stride", ctypes.c_int64),
        ("draft_prob", ctypes.c_void_p), ("accept_u", ctypes.c_void_p), ("resample_u", ctypes.c_void_p),
        ("row_max", ctypes.c_void_p), ("row_sumexp", ctypes.c_void_p), ("accept_len", ctypes.c_void_p),
        ("accept_path", ctypes.c_void_p), ("end_node", ctypes.c_void_p), ("bonus_token", ctypes.c_void_p),
    ]


_lib = None


def _load_hip_runtime():
    """libgsd.so is linked without a HIP runtime of its own: it must run on the runtime that owns torch's
    device memory and streams.  Make that runtime's symbols globally visible before libgsd is loaded."""
    import torch
    candidates = [os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so"),
                  "/opt/rocm/lib/libamdhip64.so"]
    for path in candidates:
        if os.path.exists(path):
            ctypes.CDLL(path, mode=ctypes.RTLD_GLOBAL)
            return path
    raise RuntimeError("no HIP runtime (libamdhip64.so) found next to torch or under /opt/rocm")


def load_library() -> ctypes.CDLL:
    """Load libgsd.so (built in-tree by paper_2407_16207_amd.build); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2407_16207_amd.build` "
                               "(there is no fallback path)")
        _load_hip_runtime()
        lib = ctypes.CDLL(LIB_PATH)
        for name in ("gsd_status_string", "gsd_last_error", "gsd_version"):
            getattr(lib, name).restype = ctypes.c_char_p
        lib.gsd_dag_attention_workspace.restype = ctypes.c_size_t
        lib.gsd_dag_attention_workspace.argtypes = [ctypes.POINTER(AttnDesc)]
        lib.gsd_dag_attention_splits.argtypes = [ctypes.POINTER(AttnDesc)]
        lib.gsd_dag_attention.argtypes = [ctypes.POINTER(AttnDesc), ctypes.c_void_p]
        lib.gsd_dag_attention_static.argtypes = [ctypes.POINTER(AttnDesc), ctypes.c_void_p]
        i32, i64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        lib.gsd_build_mask.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp]
        lib.gsd_node_argmax.argtypes = [i32, i32, ctypes.c_int, vp, i64, vp, vp]
        lib.gsd_node_argmax_stats.argtypes = [i32, i32, ctypes.c_int, vp, i64, vp, vp, vp, vp]
        lib.gsd_accept_longest_path.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, ctypes.c_int, i32, i64, vp, vp,
                                                vp, vp, vp, vp]
        lib.gsd_unmerge_to_tree.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.gsd_gather_rows.argtypes = [i64, i64, vp, i64, i64, vp, vp, i64, vp]
        lib.gsd_commit_kv.argtypes = [i32, i32, i32, i64, vp, vp, i64, i64, vp, vp, vp, vp, vp, vp]
        lib.gsd_softmax_stats.argtypes = [i64, i32, ctypes.c_int, vp, i64, vp, vp, vp]
        lib.gsd_accept_stochastic.argtypes = [ctypes.POINTER(StochasticDesc), vp]
        lib.gsd_build_token_graph.argtypes = [i32, i32, i32, ctypes.c_float, ctypes.c_float, vp, vp, vp, vp, vp, vp, vp,
                                              vp, i64, vp, vp, vp, vp]
        _lib = lib
    return _lib


def _check(status: int):
    if status != GSD_OK:
        lib = load_library()
        detail = lib.gsd_last_error().decode() or lib.gsd_status_string(status).decode()
        raise GsdError(status, detail)


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return GSD_F32
    if t.dtype == torch.bfloat16:
        return GSD_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _require(t, dtype, name):
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")


def gsd_build_mask(node_offsets, parent_offsets, parent_idx, max_nodes: int, words_per_row: int | None = None,
                   mask=None, dag_error_flag=None, stream=None):
    """mask[T, W] (int64 storage of the uint64 words) from the packed token graph.  See gsd_build_mask in gsd.h."""
    import torch
    for t, name in ((node_offsets, "node_offsets"), (parent_offsets, "parent_offsets"), (parent_idx, "parent_idx")):
        _require(t, torch.int32, name)
    batch = node_offsets.numel() - 1
    total = parent_offsets.numel() - 1
    W = (max_nodes + 63) // 64 if words_per_row is None else int(words_per_row)
    if mask is None:
        mask = torch.empty((total, W), dtype=torch.int64, device=node_offsets.device)
    else:
        _require(mask, torch.int64, "mask")
        if mask.numel() != total * W:
            raise ValueError("mask has the wrong size")
    if dag_error_flag is not None:
        _require(dag_error_flag, torch.int32, "dag_error_flag")
    _check(load_library().gsd_build_mask(batch, max_nodes, W, _ptr(node_offsets), _ptr(parent_offsets),
                                         _ptr(parent_idx), _ptr(mask), _ptr(dag_error_flag), _stream_ptr(stream)))
    return mask


def make_attn_desc(q, k, v, kv_offsets, prefix_lens, node_offsets, mask, max_nodes: int, max_prefix: int,
                   softmax_scale: float, out=None, lse=None, num_splits: int = 0, workspace=None,
                   wg_waves: int = 0) -> AttnDesc:
    import torch
    code = _dtype_code(q)
    for t, name in ((q, "q"), (k, "k"), (v, "v")):
        if not t.is_cuda or t.dim() != 3 or t.stride(2) != 1 or _dtype_code(t) != code:
            raise ValueError(f"{name} must be a GPU tensor [rows, heads, head_dim] with a contiguous last dim")
    if k.stride() != v.stride() or k.shape != v.shape:
        raise ValueError("k and v must share shape and strides")
    _require(kv_offsets, torch.int64, "kv_offsets")
    _require(prefix_lens, torch.int32, "prefix_lens")
    _require(node_offsets, torch.int32, "node_offsets")
    _require(mask, torch.int64, "mask")
    d = AttnDesc()
    d.batch = prefix_lens.numel()
    d.total_nodes, d.num_q_heads, d.head_dim = q.shape
    d.num_kv_heads = k.shape[1]
    d.max_nodes, d.max_prefix = int(max_nodes), int(max_prefix)
    d.dtype = code
    d.words_per_row = mask.shape[1]
    d.num_splits = int(num_splits)
    d.wg_waves = int(wg_waves)
    d.softmax_scale = float(softmax_scale)
    d.q, d.k, d.v = q.data_ptr(), k.data_ptr(), v.data_ptr()
    d.o = out.data_ptr() if out is not None else None
    d.lse = lse.data_ptr() if lse is not None else None
    d.kv_offsets, d.prefix_lens, d.node_offsets, d.mask = (kv_offsets.data_ptr(), prefix_lens.data_ptr(),
                                                           node_offsets.data_ptr(), mask.data_ptr())
    d.q_token_stride, d.q_head_stride = q.stride(0), q.stride(1)
    if out is not None:
        d.o_token_stride, d.o_head_stride = out.stride(0), out.stride(1)
    d.kv_token_stride, d.kv_head_stride = k.stride(0), k.stride(1)
    if workspace is not None:
        d.workspace, d.workspace_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    return d


def gsd_dag_attention_workspace(desc: AttnDesc) -> int:
    n = load_library().gsd_dag_attention_workspace(ctypes.byref(desc))
    if n == ctypes.c_size_t(-1).value:
        _check(GSD_ERR_INVALID_ARG)
    return n


def gsd_dag_attention_splits(desc: AttnDesc) -> int:
    return load_library().gsd_dag_attention_splits(ctypes.byref(desc))


def gsd_dag_attention(q, k, v, kv_offsets, prefix_lens, node_offsets, mask, max_nodes: int, max_prefix: int,
                      softmax_scale: float, out=None, lse=None, num_splits: int = 0, workspace=None, stream=None,
                      return_lse: bool = False, wg_waves: int = 0):
    """DAG-masked attention of every packed node; returns out (same dtype/shape as q).  See gsd.h."""
    import torch
    if out is None:
        out = torch.empty_like(q, memory_format=torch.contiguous_format)
    if return_lse and lse is None:
        lse = torch.empty((q.shape[0], q.shape[1]), dtype=torch.float32, device=q.device)
    if lse is not None:
        _require(lse, torch.float32, "lse")
    desc = make_attn_desc(q, k, v, kv_offsets, prefix_lens, node_offsets, mask, max_nodes, max_prefix, softmax_scale,
                          out=out, lse=lse, num_splits=num_splits, workspace=workspace, wg_waves=wg_waves)
    if workspace is None:
        need = gsd_dag_attention_workspace(desc)
        if need:
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
            desc.workspace, desc.workspace_bytes = workspace.data_ptr(), need
    _check(load_library().gsd_dag_attention(ctypes.byref(desc), _stream_ptr(stream)))
    return (out, lse) if return_lse else out


def gsd_dag_attention_desc(desc: AttnDesc, stream=None):
    """Launch from a prepared descriptor (no allocation, for timing loops)."""
    _check(load_library().gsd_dag_attention(ctypes.byref(desc), _stream_ptr(stream)))


def gsd_dag_attention_static(desc: AttnDesc, stream=None):
    """gsd_dag_attention_static of gsd.h: launch from a prepared descriptor, split partials in the library's static
    scratch array (the descriptor's workspace fields are ignored).  Allocates nothing."""
    _check(load_library().gsd_dag_attention_static(ctypes.byref(desc), _stream_ptr(stream)))


def gsd_node_argmax(logits, pred=None, stream=None):
    """pred[r] = lowest index of the row maximum of logits[r].  See gsd_node_argmax in gsd.h."""
    import torch
    if not logits.is_cuda or logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be a GPU tensor [rows, vocab] with a contiguous last dim")
    rows, vocab = logits.shape
    if pred is None:
        pred = torch.empty(rows, dtype=torch.int32, device=logits.device)
    _require(pred, torch.int32, "pred")
    _check(load_library().gsd_node_argmax(rows, vocab, _dtype_code(logits), _ptr(logits), logits.stride(0),
                                          _ptr(pred), _stream_ptr(stream)))
    return pred


def gsd_node_argmax_stats(logits, pred=None, row_max=None, row_sumexp=None, stream=None):
    """One pass over the logits: (pred, row_max, row_sumexp) as gsd_node_argmax and gsd_softmax_stats give them.
    See gsd_node_argmax_stats in gsd.h."""
    import torch
    if not logits.is_cuda or logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be a GPU tensor [rows, vocab] with a contiguous last dim")
    rows, vocab = logits.shape
    pred = torch.empty(rows, dtype=torch.int32, device=logits.device) if pred is None else pred
    row_max = torch.empty(rows, dtype=torch.float32, device=logits.device) if row_max is None else row_max
    row_sumexp = torch.empty(rows, dtype=torch.float32, device=logits.device) if row_sumexp is None else row_sumexp
    _require(pred, torch.int32, "pred")
    _require(row_max, torch.float32, "row_max")
    _require(row_sumexp, torch.float32, "row_sumexp")
    _check(load_library().gsd_node_argmax_stats(rows, vocab, _dtype_code(logits), _ptr(logits), logits.stride(0),
                                                _ptr(pred), _ptr(row_max), _ptr(row_sumexp), _stream_ptr(stream)))
    return pred, row_max, row_sumexp


def gsd_accept_longest_path(node_offsets, parent_offsets, parent_idx, tokens, root_pred, max_nodes: int,
                            logits=None, pred=None, accept_len=None, accept_path=None, bonus_token=None,
                            stream=None):
    """Longest accepted root path per sequence; returns (accept_len[B], accept_path[B, max_nodes], bonus[B], pred).
    With `logits` the per-node argmax runs first on the same stream.  See gsd_accept_longest_path in gsd.h."""
    import torch
    for t, name in ((node_offsets, "node_offsets"), (parent_offsets, "parent_offsets"), (parent_idx, "parent_idx"),
                    (tokens, "tokens"), (root_pred, "root_pred")):
        _require(t, torch.int32, name)
    batch = node_offsets.numel() - 1
    total = tokens.numel()
    dev = tokens.device
    if pred is None:
        if logits is None:
            raise ValueError("give logits or pred")
        pred = torch.empty(total, dtype=torch.int32, device=dev)
    _require(pred, torch.int32, "pred")
    accept_len = torch.empty(batch, dtype=torch.int32, device=dev) if accept_len is None else accept_len
    accept_path = torch.empty((batch, max_nodes), dtype=torch.int32, device=dev) if accept_path is None else accept_path
    bonus_token = torch.empty(batch, dtype=torch.int32, device=dev) if bonus_token is None else bonus_token
    for t, name in ((accept_len, "accept_len"), (accept_path, "accept_path"), (bonus_token, "bonus_token")):
        _require(t, torch.int32, name)
    if logits is not None:
        if not logits.is_cuda or logits.dim() != 2 or logits.stride(1) != 1 or logits.shape[0] != total:
            raise ValueError("logits must be a GPU tensor [T, vocab] with a contiguous last dim")
        dtype, vocab, stride = _dtype_code(logits), logits.shape[1], logits.stride(0)
    else:
        dtype, vocab, stride = GSD_F32, 0, 0
    _check(load_library().gsd_accept_longest_path(batch, total, max_nodes, _ptr(node_offsets), _ptr(parent_offsets),
                                                  _ptr(parent_idx), _ptr(tokens), _ptr(logits), dtype, vocab, stride,
                                                  _ptr(pred), _ptr(root_pred), _ptr(accept_len), _ptr(accept_path),
                                                  _ptr(bonus_token), _stream_ptr(stream)))
    return accept_len, accept_path, bonus_token, pred


def gsd_unmerge_to_tree(node_offsets, parent_offsets, parent_idx, max_nodes: int, max_tree_nodes: int,
                        dag_error_flag=None, stream=None):
    """Token graph -> token tree with replicated successors.  Returns (tree_node_offsets[B+1], tree_parent,
    tree_parent_offsets, tree_origin, path_count[B]); the three per-node arrays are allocated at their bound
    B*max_tree_nodes (+1) and only their first tree_node_offsets[B] (+1) entries are written.  See gsd.h."""
    import torch
    for t, name in ((node_offsets, "node_offsets"), (parent_offsets, "parent_offsets"), (parent_idx, "parent_idx")):
        _require(t, torch.int32, name)
    batch = node_offsets.numel() - 1
    dev = node_offsets.device
    bound = batch * int(max_tree_nodes)
    tree_node_offsets = torch.empty(batch + 1, dtype=torch.int32, device=dev)
    tree_parent = torch.empty(bound, dtype=torch.int32, device=dev)
    tree_parent_offsets = torch.empty(bound + 1, dtype=torch.int32, device=dev)
    tree_origin = torch.empty(bound, dtype=torch.int32, device=dev)
    path_count = torch.empty(batch, dtype=torch.int64, device=dev)
    if dag_error_flag is not None:
        _require(dag_error_flag, torch.int32, "dag_error_flag")
    _check(load_library().gsd_unmerge_to_tree(batch, max_nodes, max_tree_nodes, _ptr(node_offsets),
                                              _ptr(parent_offsets), _ptr(parent_idx), _ptr(tree_node_offsets),
                                              _ptr(tree_parent), _ptr(tree_parent_offsets), _ptr(tree_origin),
                                              _ptr(path_count), _ptr(dag_error_flag), _stream_ptr(stream)))
    return tree_node_offsets, tree_parent, tree_parent_offsets, tree_origin, path_count


def gsd_gather_rows(src, index, out=None, rows: int | None = None, stream=None):
    """out[r] = src[index[r]] along dim 0 (rows of any trailing shape, contiguous within a row).  See gsd.h."""
    import torch
    _require(index, torch.int32, "index")
    if not src.is_cuda or src.dim() < 1 or not src[0].is_contiguous():
        raise ValueError("src must be a GPU tensor whose rows (dim 0 slices) are contiguous")
    rows = index.numel() if rows is None else int(rows)
    if out is None:
        out = torch.empty((rows,) + tuple(src.shape[1:]), dtype=src.dtype, device=src.device)
    elif out.dtype != src.dtype or tuple(out.shape[1:]) != tuple(src.shape[1:]) or out.shape[0] < rows or \
            not out[0].is_contiguous():
        raise ValueError("out must match src's dtype and row shape and hold `rows` rows")
    if rows == 0:
        return out
    es = src.element_size()
    row_elems = 1
    for d in src.shape[1:]:
        row_elems *= d
    src_stride = src.stride(0) if src.shape[0] > 1 else row_elems
    out_stride = out.stride(0) if out.shape[0] > 1 else row_elems
    _check(load_library().gsd_gather_rows(rows, row_elems * es, _ptr(src), src.shape[0], src_stride * es, _ptr(index),
                                          _ptr(out), out_stride * es, _stream_ptr(stream)))
    return out


def gsd_commit_kv(k, v, kv_offsets, prefix_lens, accept_len, accept_path, new_prefix_lens=None, stream=None):
    """In-place KV-cache commit of the accepted path.  k, v: [L, R, Hkv, D] (or [R, Hkv, D] for one layer) with
    contiguous rows; returns new_prefix_lens[B].  See gsd_commit_kv in gsd.h."""
    import torch
    if k.dim() == 3:
        k, v = k.unsqueeze(0), v.unsqueeze(0)
    if k.dim() != 4 or k.shape != v.shape or k.stride() != v.stride() or not k.is_cuda or not k[0, 0].is_contiguous():
        raise ValueError("k and v must be GPU tensors [layers, rows, kv_heads, head_dim] with contiguous rows")
    _require(kv_offsets, torch.int64, "kv_offsets")
    for t, name in ((prefix_lens, "prefix_lens"), (accept_len, "accept_len"), (accept_path, "accept_path")):
        _require(t, torch.int32, name)
    batch = prefix_lens.numel()
    max_nodes = accept_path.shape[1]
    if new_prefix_lens is None:
        new_prefix_lens = torch.empty(batch, dtype=torch.int32, device=k.device)
    _require(new_prefix_lens, torch.int32, "new_prefix_lens")
    es = k.element_size()
    _check(load_library().gsd_commit_kv(batch, max_nodes, k.shape[0], k.shape[2] * k.shape[3] * es, _ptr(k), _ptr(v),
                                        k.stride(1) * es, k.stride(0) * es, _ptr(kv_offsets), _ptr(prefix_lens),
                                        _ptr(accept_len), _ptr(accept_path), _ptr(new_prefix_lens),
                                        _stream_ptr(stream)))
    return new_prefix_lens


def gsd_softmax_stats(logits, row_max=None, row_sumexp=None, stream=None):
    """(row_max[r], row_sumexp[r]) of every logits row.  See gsd_softmax_stats in gsd.h."""
    import torch
    if not logits.is_cuda or logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be a GPU tensor [rows, vocab] with a contiguous last dim")
    rows, vocab = logits.shape
    row_max = torch.empty(rows, dtype=torch.float32, device=logits.device) if row_max is None else row_max
    row_sumexp = torch.empty(rows, dtype=torch.float32, device=logits.device) if row_sumexp is None else row_sumexp
    _require(row_max, torch.float32, "row_max")
    _require(row_sumexp, torch.float32, "row_sumexp")
    _check(load_library().gsd_softmax_stats(rows, vocab, _dtype_code(logits), _ptr(logits), logits.stride(0),
                                            _ptr(row_max), _ptr(row_sumexp), _stream_ptr(stream)))
    return row_max, row_sumexp


def gsd_accept_stochastic(node_offsets, parent_offsets, parent_idx, tokens, logits, root_logits, draft_logits,
                          root_draft_logits, draft_prob, accept_u, resample_u, max_nodes: int, stream=None):
    """Non-deterministic verification; returns (accept_len[B], accept_path[B, max_nodes], end_node[B], bonus_token[B],
    row_max[T+B], row_sumexp[T+B]).  See gsd_accept_stochastic in gsd.h."""
    import torch
    for t, name in ((node_offsets, "node_offsets"), (parent_offsets, "parent_offsets"), (parent_idx, "parent_idx"),
                    (tokens, "tokens")):
        _require(t, torch.int32, name)
    for t, name in ((draft_prob, "draft_prob"), (accept_u, "accept_u"), (resample_u, "resample_u")):
        _require(t, torch.float32, name)
    code = _dtype_code(logits)
    T, V = logits.shape
    B = node_offsets.numel() - 1
    for t, name, rows in ((logits, "logits", T), (root_logits, "root_logits", B), (draft_logits, "draft_logits", T),
                          (root_draft_logits, "root_draft_logits", B)):
        if not t.is_cuda or t.dim() != 2 or t.shape != (rows, V) or t.stride(1) != 1 or _dtype_code(t) != code or \
                (rows > 1 and t.stride(0) != logits.stride(0)):
            raise ValueError(f"{name} must be a GPU tensor [{rows}, {V}] of the same dtype and row stride as logits")
    dev = logits.device
    d = StochasticDesc()
    d.batch, d.total_nodes, d.max_nodes, d.vocab, d.dtype = B, T, int(max_nodes), V, code
    d.row_stride = logits.stride(0)
    out = {"row_max": torch.empty(T + B, dtype=torch.float32, device=dev),
           "row_sumexp": torch.empty(T + B, dtype=torch.float32, device=dev),
           "accept_len": torch.empty(B, dtype=torch.int32, device=dev),
           "accept_path": torch.empty((B, max_nodes), dtype=torch.int32, device=dev),
           "end_node": torch.empty(B, dtype=torch.int32, device=dev),
           "bonus_token": torch.empty(B, dtype=torch.int32, device=dev)}
    for name, t in (("node_offsets", node_offsets), ("parent_offsets", parent_offsets), ("parent_idx", parent_idx),
                    ("tokens", tokens), ("logits", logits), ("root_logits", root_logits),
                    ("draft_logits", draft_logits), ("root_draft_logits", root_draft_logits),
                    ("draft_prob", draft_prob), ("accept_u", accept_u), ("resample_u", resample_u), *out.items()):
        setattr(d, name, t.data_ptr())
    _check(load_library().gsd_accept_stochastic(ctypes.byref(d), _stream_ptr(stream)))
    return (out["accept_len"], out["accept_path"], out["end_node"], out["bonus_token"], out["row_max"],
            out["row_sumexp"])


def gsd_build_token_graph(node_offsets, tree_parent, tokens, draft_prob, max_nodes: int, tau: int, theta_prob: float,
                          theta_sib: float, edge_capacity: int | None = None, error_flag=None, stream=None):
    """Drafted token trees -> pruned, merged token graphs.  Returns (graph_node_offsets[B+1], parent_offsets[T+1],
    parent_idx[edge_capacity], origin[T], flags[T], counts[B, 2]); only the first T' (+1) / E entries are written.
    See gsd_build_token_graph in gsd.h."""
    import torch
    for t, name in ((node_offsets, "node_offsets"), (tree_parent, "tree_parent"), (tokens, "tokens")):
        _require(t, torch.int32, name)
    _require(draft_prob, torch.float32, "draft_prob")
    B, T = node_offsets.numel() - 1, tokens.numel()
    dev = tokens.device
    cap = int(edge_capacity) if edge_capacity is not None else 8 * T
    counts = torch.empty((B, 2), dtype=torch.int32, device=dev)
    g_off = torch.empty(B + 1, dtype=torch.int32, device=dev)
    p_off = torch.empty(T + 1, dtype=torch.int32, device=dev)
    p_idx = torch.empty(cap, dtype=torch.int32, device=dev)
    origin = torch.empty(T, dtype=torch.int32, device=dev)
    flags = torch.empty(T, dtype=torch.int32, device=dev)
    if error_flag is not None:
        _require(error_flag, torch.int32, "error_flag")
    _check(load_library().gsd_build_token_graph(B, max_nodes, tau, theta_prob, theta_sib, _ptr(node_offsets),
                                                _ptr(tree_parent), _ptr(tokens), _ptr(draft_prob), _ptr(counts),
                                                _ptr(g_off), _ptr(p_off), _ptr(p_idx), cap, _ptr(origin), _ptr(flags),
                                                _ptr(error_flag), _stream_ptr(stream)))
    return g_off, p_off, p_idx, origin, flags, counts
