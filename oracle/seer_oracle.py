"""ctypes front end of the C oracle (oracle/seer_oracle.c).

TEST INFRASTRUCTURE ONLY.  Arrays in, arrays out, all numpy on the host; bf16
tensors travel as uint16 bit patterns.  The arithmetic lives in the C file; this
module only marshals arguments and builds the shared object with gcc.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "seer_oracle.c")
_LIB = os.path.join(_HERE, "libseer_oracle.so")
_lib = None

_ERR = {-1: "bad shape or null pointer", -2: "ctx_len < T or more pages than the table holds",
        -3: "block-table entry outside the pool", -4: "tree_parent not in [-2, t)", -5: "out of memory"}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_argmax.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p]
        _lib.oracle_verify_attention.argtypes = [ctypes.c_void_p] * 7 + [ctypes.c_int] * 9 + [ctypes.c_double]
        _lib.oracle_verify_attention_rows.argtypes = ([ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
                                                      + [ctypes.c_void_p] * 6 + [ctypes.c_int] * 9
                                                      + [ctypes.c_double])
        _lib.oracle_accept.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int] * 2 + [ctypes.c_void_p] * 3
    return _lib


def _check(rc: int) -> None:
    if rc != 0:
        raise ValueError("oracle: %s (%d)" % (_ERR.get(rc, "error"), rc))


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _attn_args(q, k_pages, v_pages, block_table, ctx_len, tree_mask):
    q = _c(q, np.uint16)
    k_pages = _c(k_pages, np.uint16)
    v_pages = _c(v_pages, np.uint16)
    block_table = _c(block_table, np.int32)
    ctx_len = _c(ctx_len, np.int32)
    tree_mask = _c(tree_mask, np.uint64)
    B, T, Hq, Dqk = q.shape
    num_pages, Hkv, P, dk = k_pages.shape
    assert dk == Dqk and block_table.shape[0] == B and ctx_len.shape == (B,)
    if tree_mask is not None:
        assert tree_mask.shape == (B, T)
    return q, k_pages, v_pages, block_table, ctx_len, tree_mask, (B, T, Hq, Hkv, Dqk, P, num_pages)


def verify_attention(q, k_pages, v_pages, block_table, ctx_len, tree_mask, scale: float,
                     Dv: Optional[int] = None) -> np.ndarray:
    """out[B,T,Hq,Dv] float64.  v_pages None = shared latent: V is the first Dv components of K."""
    q, k_pages, v_pages, block_table, ctx_len, tree_mask, dims = _attn_args(
        q, k_pages, v_pages, block_table, ctx_len, tree_mask)
    B, T, Hq, Hkv, Dqk, P, num_pages = dims
    if v_pages is not None:
        Dv = v_pages.shape[3]
    assert Dv is not None
    out = np.empty((B, T, Hq, Dv), dtype=np.float64)
    _check(_load().oracle_verify_attention(_p(out), _p(q), _p(k_pages), _p(v_pages), _p(block_table),
                                           _p(ctx_len), _p(tree_mask), B, T, Hq, Hkv, Dqk, Dv, P, num_pages,
                                           block_table.shape[1], float(scale)))
    return out


def verify_attention_rows(rows, q, k_pages, v_pages, block_table, ctx_len, tree_mask, scale: float,
                          Dv: Optional[int] = None) -> np.ndarray:
    """out[len(rows), Dv] float64 for rows[i] = (b, t, h)."""
    q, k_pages, v_pages, block_table, ctx_len, tree_mask, dims = _attn_args(
        q, k_pages, v_pages, block_table, ctx_len, tree_mask)
    B, T, Hq, Hkv, Dqk, P, num_pages = dims
    if v_pages is not None:
        Dv = v_pages.shape[3]
    assert Dv is not None
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
    out = np.empty((rows.shape[0], Dv), dtype=np.float64)
    _check(_load().oracle_verify_attention_rows(_p(out), _p(rows), rows.shape[0], _p(q), _p(k_pages),
                                                _p(v_pages), _p(block_table), _p(ctx_len), _p(tree_mask),
                                                B, T, Hq, Hkv, Dqk, Dv, P, num_pages, block_table.shape[1],
                                                float(scale)))
    return out


def argmax(logits) -> np.ndarray:
    """target[...] int32 over the last axis of float32 logits (lowest index on ties)."""
    logits = _c(logits, np.float32)
    V = logits.shape[-1]
    out = np.empty(logits.shape[:-1], dtype=np.int32)
    _check(_load().oracle_argmax(_p(logits), int(np.prod(logits.shape[:-1], dtype=np.int64)), V, _p(out)))
    return out


def accept(target, draft_tokens, tree_parent):
    """(accepted_len[B], accepted_path[B,T], bonus[B]) from per-slot target tokens."""
    target = _c(target, np.int32)
    draft_tokens = _c(draft_tokens, np.int32)
    tree_parent = _c(tree_parent, np.int32)
    B, T = target.shape
    assert draft_tokens.shape == (B, T)
    alen = np.empty(B, dtype=np.int32)
    path = np.empty((B, T), dtype=np.int32)
    bonus = np.empty(B, dtype=np.int32)
    _check(_load().oracle_accept(_p(target), _p(draft_tokens), _p(tree_parent), B, T, _p(alen), _p(path),
                                 _p(bonus)))
    return alen, path, bonus


def verify_accept(logits, draft_tokens, tree_parent):
    """argmax then acceptance: (accepted_len, accepted_path, bonus, target)."""
    tgt = argmax(logits)
    alen, path, bonus = accept(tgt, draft_tokens, tree_parent)
    return alen, path, bonus, tgt
