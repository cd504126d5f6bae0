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
_SRC_NEXT = os.path.join(_HERE, "seer_oracle_next.c")      # commit of the accepted path, sampled verification
# SEER_ORACLE_SANITIZE=1: the same sources under gcc's address and undefined-behaviour sanitizers (run the tests with
# LD_PRELOAD=$(gcc -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0 so that the runtime comes first)
_SANITIZE = os.environ.get("SEER_ORACLE_SANITIZE", "") not in ("", "0")
_LIB = os.path.join(_HERE, "libseer_oracle_san.so" if _SANITIZE else "libseer_oracle.so")
_lib = None

_ERR = {-1: "bad shape or null pointer", -2: "ctx_len < T or more pages than the table holds",
        -3: "block-table entry outside the pool", -4: "tree_parent not in [-2, t)", -5: "out of memory"}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_NEXT))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        tmp = _LIB + ".tmp%d" % os.getpid()
        common = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-Wall", "-Wextra"]
        if _SANITIZE:
            common = ["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fPIC", "-Wall", "-Wextra", "-fno-omit-frame-pointer",
                      "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
        objs = []
        # the second file decides an argmax in fp32: no contraction of a*b+c beyond the fmaf calls it writes
        for src, extra in ((_SRC, []), (_SRC_NEXT, ["-ffp-contract=off"])):
            obj = "%s.%d.o" % (os.path.splitext(src)[0], os.getpid())
            subprocess.check_call(common + extra + ["-c", "-o", obj, src])
            objs.append(obj)
        try:
            subprocess.check_call(common + ["-shared", "-o", tmp] + objs + ["-lm"])
        finally:
            for obj in objs:
                os.remove(obj)
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
        _lib.oracle_kv_commit.argtypes = [ctypes.c_void_p] * 6 + [ctypes.c_int] * 8 + [ctypes.c_void_p]
        _lib.oracle_emitted_tokens.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int] * 2 + [ctypes.c_void_p] * 2
        _lib.oracle_philox4x32_10.argtypes = [ctypes.c_void_p] * 3
        _lib.oracle_philox4x32_10.restype = None
        _lib.oracle_log2_det.argtypes = [ctypes.c_float]
        _lib.oracle_log2_det.restype = ctypes.c_float
        _lib.oracle_gumbel.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32]
        _lib.oracle_gumbel.restype = ctypes.c_float
        _lib.oracle_gumbel_of_words.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
        _lib.oracle_gumbel_of_words.restype = None
        _lib.oracle_argmax_sampled.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float,
                                               ctypes.c_uint64, ctypes.c_void_p]
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


def kv_commit(k_pages, v_pages, block_table, ctx_len, accepted_len, accepted_path):
    """Compacts the accepted path's key/value rows behind the root (oracle_kv_commit).

    Returns (k_pages, v_pages, ctx_len) after the step; the inputs are not modified.  Pools are uint16
    bit patterns [num_pages, Hkv, P, D]; v_pages None = shared latent.
    """
    k = np.array(k_pages, dtype=np.uint16, order="C", copy=True)
    v = None if v_pages is None else np.array(v_pages, dtype=np.uint16, order="C", copy=True)
    bt, cl = _c(block_table, np.int32), _c(ctx_len, np.int32)
    al, ap = _c(accepted_len, np.int32), _c(accepted_path, np.int32)
    num_pages, Hkv, P, Dqk = k.shape
    B, T = ap.shape
    Dv = v.shape[3] if v is not None else 0
    out_len = np.empty(B, np.int32)
    _check(_load().oracle_kv_commit(_p(k), _p(v), _p(bt), _p(cl), _p(al), _p(ap), B, T, Hkv, Dqk, Dv, P, num_pages,
                                    bt.shape[1], _p(out_len)))
    return k, v, out_len


def emitted_tokens(draft_tokens, accepted_len, accepted_path, bonus_token):
    """(emitted [B,T] padded with -1, n_emitted [B]): accepted draft tokens in path order, then the bonus."""
    d, al, ap, bo = (_c(x, np.int32) for x in (draft_tokens, accepted_len, accepted_path, bonus_token))
    B, T = d.shape
    em, n = np.empty((B, T), np.int32), np.empty(B, np.int32)
    _check(_load().oracle_emitted_tokens(_p(d), _p(al), _p(ap), _p(bo), B, T, _p(em), _p(n)))
    return em, n


def philox4x32_10(counter, key) -> np.ndarray:
    c, k = np.asarray(counter, np.uint32).copy(), np.asarray(key, np.uint32).copy()
    out = np.empty(4, np.uint32)
    _load().oracle_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def log2_det(x: float) -> float:
    return float(_load().oracle_log2_det(float(x)))


def gumbel(seed: int, row: int, v: int) -> float:
    return float(_load().oracle_gumbel(seed, row, v))


def gumbel_of_words(words) -> np.ndarray:
    """The Gumbel deviates that the given 32-bit generator words turn into (same arithmetic as `gumbel`)."""
    w = _c(words, np.uint32)
    out = np.empty(w.shape, dtype=np.float32)
    _load().oracle_gumbel_of_words(_p(w), w.size, _p(out))
    return out


def argmax_sampled(logits, temperature: float, seed: int) -> np.ndarray:
    """Token drawn from softmax(logits / temperature) per row, by the reproducible Gumbel-max rule."""
    lg = _c(logits, np.float32)
    V = lg.shape[-1]
    rows = lg.size // V
    out = np.empty(rows, np.int32)
    _check(_load().oracle_argmax_sampled(_p(lg), rows, V, temperature, seed, _p(out)))
    return out.reshape(lg.shape[:-1])
