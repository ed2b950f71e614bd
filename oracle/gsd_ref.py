"""ctypes front-end of the CPU oracle (oracle/gsd_ref.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module; the product path
never does.  It marshals numpy arrays into the C oracle and holds no arithmetic of its own.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gsd_ref.c")
_LIB = os.path.join(_HERE, "libgsd_ref.so")
_lib = None

F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over rows; no BLAS, no hand vectorisation)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def num_threads() -> int:
    """Threads the oracle's row loops run on (OpenMP's current maximum)."""
    return int(_load().gsd_ref_num_threads())


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"oracle takes float32 or bf16-as-uint16 arrays, got {a.dtype}")


def build_mask(node_offsets, parent_offsets, parent_idx, words_per_row=None):
    """Returns (mask[T, W] uint64, dag_error_flag)."""
    node_offsets, parent_offsets, parent_idx = _i32(node_offsets), _i32(parent_offsets), _i32(parent_idx)
    B = len(node_offsets) - 1
    T = int(node_offsets[-1])
    nmax = int(np.max(np.diff(node_offsets))) if B else 0
    W = max(1, (nmax + 63) // 64) if words_per_row is None else int(words_per_row)
    mask = np.zeros((T, W), dtype=np.uint64)
    flag = np.zeros(1, dtype=np.int32)
    if len(parent_idx) == 0:
        parent_idx = np.zeros(1, dtype=np.int32)
    rc = _load().gsd_ref_build_mask(ctypes.c_int32(B), ctypes.c_int32(W), _p(node_offsets), _p(parent_offsets),
                                    _p(parent_idx), _p(mask), _p(flag))
    if rc != 0:
        raise ValueError("gsd_ref_build_mask: words_per_row too small")
    return mask, int(flag[0])


def _attn_common(q, k, v, num_kv_heads):
    code = _dtype_code(q)
    assert _dtype_code(k) == code and _dtype_code(v) == code
    q = np.ascontiguousarray(q)
    k = np.ascontiguousarray(k)
    v = np.ascontiguousarray(v)
    T, Hq, D = q.shape
    assert k.shape[1] == num_kv_heads and k.shape[2] == D and v.shape == k.shape
    return code, q, k, v, T, Hq, D


def dag_attention(q, k, v, kv_offsets, prefix_lens, node_offsets, mask, scale, rows=None, return_lse=False):
    """q [T,Hq,D], k/v [R,Hkv,D] (float32 or bf16 bits).  Returns fp64 out [T,Hq,D] (or [n_rows,D] when
    `rows` = (row_b, row_i, row_h) selects a subset) and optionally the log-sum-exp of the scaled scores."""
    Hkv = k.shape[1]
    code, q, k, v, T, Hq, D = _attn_common(q, k, v, Hkv)
    kv_offsets = np.ascontiguousarray(kv_offsets, dtype=np.int64)
    prefix_lens, node_offsets = _i32(prefix_lens), _i32(node_offsets)
    mask = np.ascontiguousarray(mask, dtype=np.uint64)
    B = len(prefix_lens)
    W = mask.shape[1]
    lib = _load()
    head = (ctypes.c_int32(B), ctypes.c_int32(Hq), ctypes.c_int32(Hkv), ctypes.c_int32(D), ctypes.c_int32(code),
            ctypes.c_double(scale), _p(q), ctypes.c_int64(Hq * D), ctypes.c_int64(D), _p(k), _p(v),
            ctypes.c_int64(Hkv * D), ctypes.c_int64(D), _p(kv_offsets), _p(prefix_lens), _p(node_offsets),
            _p(mask), ctypes.c_int32(W))
    if rows is None:
        out = np.zeros((T, Hq, D), dtype=np.float64)
        lse = np.zeros((T, Hq), dtype=np.float64)
        rc = lib.gsd_ref_dag_attention(*head, _p(out), _p(lse))
    else:
        rb, ri, rh = (_i32(x) for x in rows)
        n = len(rb)
        out = np.zeros((n, D), dtype=np.float64)
        lse = np.zeros((n,), dtype=np.float64)
        rc = lib.gsd_ref_dag_attention_rows(*head, ctypes.c_int64(n), _p(rb), _p(ri), _p(rh), _p(out), _p(lse))
    if rc != 0:
        raise ValueError("gsd_ref_dag_attention: bad arguments")
    return (out, lse) if return_lse else out


def node_argmax(logits):
    logits = np.ascontiguousarray(logits)
    code = _dtype_code(logits)
    rows, vocab = logits.shape
    pred = np.zeros(rows, dtype=np.int32)
    _load().gsd_ref_node_argmax(ctypes.c_int64(rows), ctypes.c_int32(vocab), ctypes.c_int32(code), _p(logits),
                                ctypes.c_int64(vocab), _p(pred))
    return pred


def accept_longest_path(node_offsets, parent_offsets, parent_idx, tokens, pred, root_pred, max_nodes=None):
    """Returns (accept_len[B], accept_path[B, max_nodes], bonus_token[B])."""
    node_offsets, parent_offsets, parent_idx = _i32(node_offsets), _i32(parent_offsets), _i32(parent_idx)
    tokens, pred, root_pred = _i32(tokens), _i32(pred), _i32(root_pred)
    B = len(node_offsets) - 1
    nmax = int(np.max(np.diff(node_offsets))) if B else 0
    max_nodes = max(1, nmax) if max_nodes is None else int(max_nodes)
    if len(parent_idx) == 0:
        parent_idx = np.zeros(1, dtype=np.int32)
    accept_len = np.zeros(B, dtype=np.int32)
    accept_path = np.zeros((B, max_nodes), dtype=np.int32)
    bonus = np.zeros(B, dtype=np.int32)
    rc = _load().gsd_ref_accept_longest_path(ctypes.c_int32(B), ctypes.c_int32(max_nodes), _p(node_offsets),
                                             _p(parent_offsets), _p(parent_idx), _p(tokens), _p(pred),
                                             _p(root_pred), _p(accept_len), _p(accept_path), _p(bonus))
    if rc != 0:
        raise ValueError("gsd_ref_accept_longest_path: max_nodes too small")
    return accept_len, accept_path, bonus
