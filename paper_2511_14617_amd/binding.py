"""Thin Python binding of libseer_verify.so (include/seer_verify.h, include/seer_verify_diag.h).

Argument marshalling only: tensors are torch CUDA(HIP) tensors whose device
pointers are handed to the C ABI; every step of the path runs in the library's
kernels.  There is no fallback: if the shared object is missing the import of
the functions fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libseer_verify.so")

SEER_OK, SEER_EINVAL, SEER_ESHAPE, SEER_EUNSUPPORTED, SEER_EWORKSPACE, SEER_EALIGN, SEER_ELIMIT = 0, -1, -2, -3, -4, -5, -6
SEER_ACCEPT_STATIC_MAX_PAIRS = 131072

EXPORTS = ("seer_verify_attention_workspace", "seer_verify_attention_status_offset", "seer_verify_attention",
           "seer_verify_attention_timed", "seer_verify_attention_kernel", "seer_verify_attention_shared_tiles_offset",
           "seer_accept_workspace", "seer_accept", "seer_accept_static", "seer_accept_sampled",
           "seer_kv_commit", "seer_mba_draft_lengths", "seer_acceptance_stats", "seer_acceptance_beta", "seer_draft_workspace", "seer_draft", "seer_history_append",
           "seer_strerror")


class SeerAttnParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("T", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("Dqk", ctypes.c_int32), ("Dv", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("num_pages", ctypes.c_int32), ("max_pages_per_seq", ctypes.c_int32),
                ("max_splits", ctypes.c_int32), ("kv_shared_latent", ctypes.c_int32), ("flags", ctypes.c_int32),
                ("scale", ctypes.c_float)]

class SeerDraftParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("n_groups", ctypes.c_int32), ("n_seq", ctypes.c_int32),
                ("pool_tokens", ctypes.c_int64), ("max_group_tokens", ctypes.c_int32), ("gamma_max", ctypes.c_int32),
                ("top_k", ctypes.c_int32), ("pattern_lookup_min", ctypes.c_int32),
                ("pattern_lookup_max", ctypes.c_int32), ("vocab", ctypes.c_int32), ("min_confidence", ctypes.c_float)]


SEER_ATTN_GENERAL_KERNEL = 1
SEER_ATTN_FIXED_SPLIT = 2
SEER_ATTN_STREAM_ONLY = 4
SEER_ATTN_REUSE_PLAN = 8


class SeerError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("seer_verify: %s (%d)" % (text, code))
        self.code = code


_lib = None


def load_library() -> ctypes.CDLL:
    """Load the HIP library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: build it with `python -m paper_2511_14617_amd.build` "
                              "(hipcc, gfx950); there is no fallback path" % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        lib.seer_verify_attention_workspace.argtypes = [ctypes.POINTER(SeerAttnParams)]
        lib.seer_verify_attention_workspace.restype = sz
        lib.seer_verify_attention_status_offset.argtypes = []
        lib.seer_verify_attention_status_offset.restype = sz
        lib.seer_verify_attention.argtypes = [vp] * 7 + [ctypes.POINTER(SeerAttnParams), vp, sz, vp]
        lib.seer_verify_attention.restype = ctypes.c_int
        lib.seer_verify_attention_timed.argtypes = lib.seer_verify_attention.argtypes + [vp, vp]
        lib.seer_verify_attention_timed.restype = ctypes.c_int
        lib.seer_verify_attention_kernel.argtypes = [ctypes.POINTER(SeerAttnParams)]
        lib.seer_verify_attention_kernel.restype = ctypes.c_char_p
        lib.seer_verify_attention_shared_tiles_offset.argtypes = [ctypes.POINTER(SeerAttnParams)]
        lib.seer_verify_attention_shared_tiles_offset.restype = sz
        lib.seer_accept_workspace.argtypes = [i32, i32, i32]
        lib.seer_accept_workspace.restype = sz
        lib.seer_accept.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        lib.seer_accept.restype = ctypes.c_int
        lib.seer_accept_static.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp]
        lib.seer_accept_static.restype = ctypes.c_int
        lib.seer_accept_sampled.argtypes = [vp, vp, vp, i32, i32, i32, ctypes.c_float, ctypes.c_uint64,
                                            vp, vp, vp, vp, vp, sz, vp]
        lib.seer_accept_sampled.restype = ctypes.c_int
        lib.seer_kv_commit.argtypes = [ctypes.POINTER(SeerAttnParams)] + [vp] * 12
        lib.seer_kv_commit.restype = ctypes.c_int
        lib.seer_mba_draft_lengths.argtypes = [i32, i32, vp, i32, i32, ctypes.c_double, vp, vp, vp, vp]
        lib.seer_mba_draft_lengths.restype = ctypes.c_int
        lib.seer_acceptance_stats.argtypes = [vp, vp, vp, i32, i32, vp, vp]
        lib.seer_acceptance_stats.restype = ctypes.c_int
        lib.seer_acceptance_beta.argtypes = [vp, i32, i32, ctypes.c_double, vp]
        lib.seer_acceptance_beta.restype = ctypes.c_int
        lib.seer_draft_workspace.argtypes = [ctypes.POINTER(SeerDraftParams)]
        lib.seer_draft_workspace.restype = sz
        lib.seer_draft.argtypes = [vp] * 8 + [ctypes.POINTER(SeerDraftParams)] + [vp] * 7 + [sz, vp]
        lib.seer_draft.restype = ctypes.c_int
        lib.seer_history_append.argtypes = [vp] * 7 + [i32, i32, i32, ctypes.c_int64, i32, vp, vp, vp, vp]
        lib.seer_history_append.restype = ctypes.c_int
        lib.seer_strerror.argtypes = [ctypes.c_int]
        lib.seer_strerror.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def seer_strerror(code: int) -> str:
    return load_library().seer_strerror(int(code)).decode()


def _check(code: int) -> None:
    if code != 0:
        raise SeerError(code, seer_strerror(code))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream_handle(stream: Optional[torch.cuda.Stream]) -> Optional[int]:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def _want(t: torch.Tensor, dtype, shape, name: str) -> None:
    if t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous() or not t.is_cuda:
        raise ValueError("%s: want contiguous device %s%s, got %s%s on %s" %
                         (name, dtype, tuple(shape), t.dtype, tuple(t.shape), t.device))


def attn_params(q: torch.Tensor, k_pages: torch.Tensor, v_pages: Optional[torch.Tensor],
                block_table: torch.Tensor, scale: float, Dv: Optional[int] = None,
                max_splits: int = 0, flags: int = 0) -> SeerAttnParams:
    B, T, Hq, Dqk = q.shape
    num_pages, Hkv, P, _ = k_pages.shape
    dv = v_pages.shape[3] if v_pages is not None else Dv
    if dv is None:
        raise ValueError("Dv is needed when the latent is shared (v_pages is None)")
    return SeerAttnParams(B, T, Hq, Hkv, Dqk, dv, P, num_pages, block_table.shape[1], max_splits,
                          1 if v_pages is None else 0, flags, float(scale))


def seer_verify_attention_workspace(params: SeerAttnParams) -> int:
    return int(load_library().seer_verify_attention_workspace(ctypes.byref(params)))


def seer_verify_attention_kernel(params: SeerAttnParams) -> Optional[str]:
    """Name of the partition kernel a call with these params launches (None on invalid params)."""
    name = load_library().seer_verify_attention_kernel(ctypes.byref(params))
    return None if name is None else name.decode()


def seer_verify_attention(q: torch.Tensor, k_pages: torch.Tensor, v_pages: Optional[torch.Tensor],
                          block_table: torch.Tensor, ctx_len: torch.Tensor,
                          tree_mask: Optional[torch.Tensor], scale: float, *, Dv: Optional[int] = None,
                          max_splits: int = 0, flags: int = 0, out: Optional[torch.Tensor] = None,
                          workspace: Optional[torch.Tensor] = None,
                          stream: Optional[torch.cuda.Stream] = None,
                          events: Optional[Tuple[int, int]] = None) -> torch.Tensor:
    """out[B,T,Hq,Dv] bf16.  q [B,T,Hq,Dqk] bf16; k_pages [num_pages,Hkv,P,Dqk] bf16; v_pages
    [num_pages,Hkv,P,Dv] bf16 or None (shared latent); block_table [B,max_pages] int32; ctx_len [B]
    int32 (counts the T verify slots); tree_mask [B,T] int64 holding the uint64 ancestor bits, or
    None for a chain.  `out` and `workspace` (uint8) may be passed to avoid allocation.  `events` = two
    hipEvent_t handles (ints) to be recorded around the partition kernel (seer_verify_attention_timed)."""
    lib = load_library()
    p = attn_params(q, k_pages, v_pages, block_table, scale, Dv, max_splits, flags)
    _want(q, torch.bfloat16, (p.B, p.T, p.Hq, p.Dqk), "q")
    _want(k_pages, torch.bfloat16, (p.num_pages, p.Hkv, p.page_size, p.Dqk), "k_pages")
    if v_pages is not None:
        _want(v_pages, torch.bfloat16, (p.num_pages, p.Hkv, p.page_size, p.Dv), "v_pages")
    _want(block_table, torch.int32, (p.B, p.max_pages_per_seq), "block_table")
    _want(ctx_len, torch.int32, (p.B,), "ctx_len")
    if tree_mask is not None:
        _want(tree_mask, torch.int64, (p.B, p.T), "tree_mask")
    if out is None:
        out = torch.empty((p.B, p.T, p.Hq, p.Dv), dtype=torch.bfloat16, device=q.device)
    else:
        _want(out, torch.bfloat16, (p.B, p.T, p.Hq, p.Dv), "out")
    need = int(lib.seer_verify_attention_workspace(ctypes.byref(p)))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    args = (_ptr(out), _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table), _ptr(ctx_len), _ptr(tree_mask),
            ctypes.byref(p), _ptr(workspace), workspace.numel(), _stream_handle(stream))
    if events is None:
        _check(lib.seer_verify_attention(*args))
    else:
        _check(lib.seer_verify_attention_timed(*args, events[0], events[1]))
    return out


def seer_verify_attention_status(workspace: torch.Tensor) -> int:
    """The status word the last call on this workspace left (synchronises)."""
    off = int(load_library().seer_verify_attention_status_offset())
    return int(workspace[off:off + 4].view(torch.int32).item()) & 0xFFFFFFFF


def seer_verify_attention_shared_tiles(workspace: torch.Tensor, params: SeerAttnParams) -> torch.Tensor:
    """int32[B]: the leading tiles of each request that the last plan on this workspace found shared with a
    neighbouring request (a diagnostic read-back; synchronises)."""
    off = int(load_library().seer_verify_attention_shared_tiles_offset(ctypes.byref(params)))
    return workspace[off:off + 4 * params.B].view(torch.int32).cpu()


def seer_accept_workspace(B: int, T: int, V: int) -> int:
    return int(load_library().seer_accept_workspace(B, T, V))


def seer_accept(logits: torch.Tensor, draft_tokens: torch.Tensor, tree_parent: Optional[torch.Tensor], *,
                workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None,
                out: Optional[Tuple[torch.Tensor, torch.Tensor, torch.Tensor, torch.Tensor]] = None,
                temperature: Optional[float] = None, seed: int = 0
                ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor, torch.Tensor]:
    """(accepted_len[B], accepted_path[B,T], bonus_token[B], target_argmax[B,T]), all int32.
    logits [B,T,V] fp32; draft_tokens [B,T] int32; tree_parent [B,T] int32 or None (chain)."""
    lib = load_library()
    B, T, V = logits.shape
    _want(logits, torch.float32, (B, T, V), "logits")
    _want(draft_tokens, torch.int32, (B, T), "draft_tokens")
    if tree_parent is not None:
        _want(tree_parent, torch.int32, (B, T), "tree_parent")
    dev = logits.device
    if out is None:
        alen = torch.empty(B, dtype=torch.int32, device=dev)
        path = torch.empty((B, T), dtype=torch.int32, device=dev)
        bonus = torch.empty(B, dtype=torch.int32, device=dev)
        tgt = torch.empty((B, T), dtype=torch.int32, device=dev)
    else:
        alen, path, bonus, tgt = out
        _want(alen, torch.int32, (B,), "accepted_len")
        _want(path, torch.int32, (B, T), "accepted_path")
        _want(bonus, torch.int32, (B,), "bonus_token")
        _want(tgt, torch.int32, (B, T), "target_argmax")
    need = int(lib.seer_accept_workspace(B, T, V))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    if temperature is None:
        _check(lib.seer_accept(_ptr(logits), _ptr(draft_tokens), _ptr(tree_parent), B, T, V, _ptr(alen), _ptr(path),
                               _ptr(bonus), _ptr(tgt), _ptr(workspace), workspace.numel(), _stream_handle(stream)))
    else:
        _check(lib.seer_accept_sampled(_ptr(logits), _ptr(draft_tokens), _ptr(tree_parent), B, T, V,
                                       float(temperature), int(seed) & 0xFFFFFFFFFFFFFFFF, _ptr(alen), _ptr(path),
                                       _ptr(bonus), _ptr(tgt), _ptr(workspace), workspace.numel(),
                                       _stream_handle(stream)))
    return alen, path, bonus, tgt


def seer_accept_static(logits: torch.Tensor, draft_tokens: torch.Tensor, tree_parent: Optional[torch.Tensor],
                       out: Tuple[torch.Tensor, torch.Tensor, torch.Tensor, torch.Tensor], *,
                       stream: Optional[torch.cuda.Stream] = None):
    """seer_accept without a workspace (the scan's scratch is a fixed array inside the library); the four
    result tensors (accepted_len, accepted_path, bonus_token, target_argmax) must be passed: the call
    allocates nothing."""
    lib = load_library()
    B, T, V = logits.shape
    _want(logits, torch.float32, (B, T, V), "logits")
    _want(draft_tokens, torch.int32, (B, T), "draft_tokens")
    if tree_parent is not None:
        _want(tree_parent, torch.int32, (B, T), "tree_parent")
    alen, path, bonus, tgt = out
    _want(alen, torch.int32, (B,), "accepted_len")
    _want(path, torch.int32, (B, T), "accepted_path")
    _want(bonus, torch.int32, (B,), "bonus_token")
    _want(tgt, torch.int32, (B, T), "target_argmax")
    _check(lib.seer_accept_static(_ptr(logits), _ptr(draft_tokens), _ptr(tree_parent), B, T, V, _ptr(alen), _ptr(path),
                                  _ptr(bonus), _ptr(tgt), _stream_handle(stream)))
    return out


def seer_accept_sampled(logits: torch.Tensor, draft_tokens: torch.Tensor, tree_parent: Optional[torch.Tensor],
                        temperature: float, seed: int, **kw):
    """As seer_accept, with the target token of each slot drawn from softmax(logits / temperature)
    (reproducible Gumbel-max draw keyed by seed); the fourth result holds the drawn tokens."""
    return seer_accept(logits, draft_tokens, tree_parent, temperature=temperature, seed=seed, **kw)


def seer_kv_commit(k_pages: torch.Tensor, v_pages: Optional[torch.Tensor], block_table: torch.Tensor,
                   ctx_len: torch.Tensor, accepted_len: torch.Tensor, accepted_path: torch.Tensor, *,
                   draft_tokens: Optional[torch.Tensor] = None, bonus_token: Optional[torch.Tensor] = None,
                   status: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """Moves the accepted path's K/V rows behind the root, in place, and advances ctx_len in place.
    With draft_tokens and bonus_token also returns (emitted_tokens[B,T], n_emitted[B]), else None."""
    lib = load_library()
    num_pages, Hkv, P, Dqk = k_pages.shape
    B, T = accepted_path.shape
    Dv = v_pages.shape[3] if v_pages is not None else 0
    _want(block_table, torch.int32, (B, block_table.shape[1]), "block_table")
    _want(ctx_len, torch.int32, (B,), "ctx_len")
    _want(accepted_len, torch.int32, (B,), "accepted_len")
    _want(accepted_path, torch.int32, (B, T), "accepted_path")
    if not (k_pages.is_contiguous() and k_pages.is_cuda and k_pages.element_size() == 2):
        raise ValueError("k_pages: want a contiguous 16-bit device tensor")
    if v_pages is not None and not (v_pages.is_contiguous() and v_pages.element_size() == 2
                                    and tuple(v_pages.shape[:3]) == (num_pages, Hkv, P)):
        raise ValueError("v_pages: want a contiguous 16-bit device tensor [num_pages, Hkv, P, Dv]")
    params = SeerAttnParams(B, T, Hkv, Hkv, Dqk, Dv, P, num_pages, block_table.shape[1], 0,
                            1 if v_pages is None else 0, 0, 1.0)
    emitted = n_emitted = None
    if draft_tokens is not None:
        _want(draft_tokens, torch.int32, (B, T), "draft_tokens")
        _want(bonus_token, torch.int32, (B,), "bonus_token")
        emitted = torch.empty((B, T), dtype=torch.int32, device=k_pages.device)
        n_emitted = torch.empty(B, dtype=torch.int32, device=k_pages.device)
    if status is not None:
        _want(status, torch.int32, (1,), "status")
    _check(lib.seer_kv_commit(ctypes.byref(params), _ptr(k_pages), _ptr(v_pages), _ptr(block_table), _ptr(ctx_len),
                              _ptr(accepted_len), _ptr(accepted_path), _ptr(draft_tokens), _ptr(bonus_token),
                              _ptr(emitted), _ptr(n_emitted), _ptr(status), _stream_handle(stream)))
    return None if emitted is None else (emitted, n_emitted)


def seer_mba_draft_lengths(B_h: int, B_l: int, beta, gamma_max: int, lam: float, step_time):
    """(gamma_h, gamma_l, gamma_star) by the paper's Algorithm 1; beta[i] = acceptance probability of
    draft position i + 1, step_time[gamma] = measured time of a step with gamma draft tokens."""
    lib = load_library()
    bt = (ctypes.c_double * len(beta))(*[float(x) for x in beta])
    st = (ctypes.c_double * len(step_time))(*[float(x) for x in step_time])
    if len(step_time) < gamma_max + 1:
        raise ValueError("step_time needs gamma_max + 1 entries")
    gh, gl, gs = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _check(lib.seer_mba_draft_lengths(B_h, B_l, bt, len(beta), gamma_max, float(lam), st, ctypes.byref(gh),
                                      ctypes.byref(gl), ctypes.byref(gs)))
    return gh.value, gl.value, gs.value


def seer_acceptance_stats(accepted_len: torch.Tensor, accepted_path: torch.Tensor, tree_parent: Optional[torch.Tensor],
                          counts: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Adds one verify step to counts [3,T] int64 on the device (offered, tried, accepted by draft position)."""
    B, T = accepted_path.shape
    _want(accepted_len, torch.int32, (B,), "accepted_len")
    _want(accepted_path, torch.int32, (B, T), "accepted_path")
    if tree_parent is not None:
        _want(tree_parent, torch.int32, (B, T), "tree_parent")
    _want(counts, torch.int64, (3, T), "counts")
    _check(load_library().seer_acceptance_stats(_ptr(accepted_len), _ptr(accepted_path), _ptr(tree_parent), B, T,
                                                _ptr(counts), _stream_handle(stream)))
    return counts


def seer_acceptance_beta(counts, conditional: bool = False, prior: float = 0.0):
    """beta for draft positions 1 .. T-1 from a host copy of the counts ([3][T] integers)."""
    T = len(counts[0])
    flat = (ctypes.c_uint64 * (3 * T))(*[int(x) for row in counts for x in row])
    beta = (ctypes.c_double * max(T - 1, 1))()
    _check(load_library().seer_acceptance_beta(flat, T, 1 if conditional else 0, float(prior), beta))
    return [beta[i] for i in range(T - 1)]


def seer_draft_workspace(params: SeerDraftParams) -> int:
    return int(load_library().seer_draft_workspace(ctypes.byref(params)))


def seer_draft(tokens: torch.Tensor, seq_start: torch.Tensor, seq_len: torch.Tensor, group_first: torch.Tensor,
               req_group: torch.Tensor, pattern: torch.Tensor, pattern_len: torch.Tensor, max_spec_tokens: torch.Tensor,
               *, gamma_max: int, top_k: int, pattern_lookup_min: int, vocab: int, max_group_tokens: int,
               min_confidence: float = 0.0, status: Optional[torch.Tensor] = None,
               workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None,
               out: Optional[Tuple[torch.Tensor, ...]] = None):
    """Draft trees from the token histories of each request's prompt group.  All tensors int32 on the device:
    tokens [pool], seq_start/seq_len [n_seq], group_first [n_groups + 1], req_group [B], pattern [B, p_max]
    (right-aligned), pattern_len [B], max_spec_tokens [B].  Returns (draft_tokens [B,T] int32, tree_parent
    [B,T] int32, tree_mask [B,T] int64 holding the uint64 bits, node_count [B,T] int32, match_len [B] int32),
    T = 1 + top_k * gamma_max."""
    lib = load_library()
    B, p_max = pattern.shape
    n_seq, n_groups = seq_start.shape[0], group_first.shape[0] - 1
    T = 1 + top_k * gamma_max
    _want(tokens, torch.int32, (tokens.shape[0],), "tokens")
    _want(seq_start, torch.int32, (n_seq,), "seq_start")
    _want(seq_len, torch.int32, (n_seq,), "seq_len")
    _want(group_first, torch.int32, (n_groups + 1,), "group_first")
    _want(req_group, torch.int32, (B,), "req_group")
    _want(pattern, torch.int32, (B, p_max), "pattern")
    _want(pattern_len, torch.int32, (B,), "pattern_len")
    _want(max_spec_tokens, torch.int32, (B,), "max_spec_tokens")
    p = SeerDraftParams(B, n_groups, n_seq, tokens.shape[0], int(max_group_tokens), gamma_max, top_k,
                        pattern_lookup_min, p_max, vocab, float(min_confidence))
    dev = tokens.device
    if out is None:
        d_tok = torch.empty((B, T), dtype=torch.int32, device=dev)
        d_par = torch.empty((B, T), dtype=torch.int32, device=dev)
        d_msk = torch.empty((B, T), dtype=torch.int64, device=dev)
        d_cnt = torch.empty((B, T), dtype=torch.int32, device=dev)
        d_len = torch.empty(B, dtype=torch.int32, device=dev)
    else:
        d_tok, d_par, d_msk, d_cnt, d_len = out
        _want(d_tok, torch.int32, (B, T), "draft_tokens")
        _want(d_par, torch.int32, (B, T), "tree_parent")
        _want(d_msk, torch.int64, (B, T), "tree_mask")
        _want(d_cnt, torch.int32, (B, T), "node_count")
        _want(d_len, torch.int32, (B,), "match_len")
    if status is not None:
        _want(status, torch.int32, (1,), "status")
    need = int(lib.seer_draft_workspace(ctypes.byref(p)))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    _check(lib.seer_draft(_ptr(tokens), _ptr(seq_start), _ptr(seq_len), _ptr(group_first), _ptr(req_group),
                          _ptr(pattern), _ptr(pattern_len), _ptr(max_spec_tokens), ctypes.byref(p), _ptr(d_tok),
                          _ptr(d_par), _ptr(d_msk), _ptr(d_cnt), _ptr(d_len), _ptr(status), _ptr(workspace),
                          workspace.numel(), _stream_handle(stream)))
    return d_tok, d_par, d_msk, d_cnt, d_len


def seer_history_append(tokens: torch.Tensor, seq_start: torch.Tensor, seq_len: torch.Tensor, seq_capacity: torch.Tensor,
                        req_seq: torch.Tensor, emitted_tokens: torch.Tensor, n_emitted: torch.Tensor, *,
                        pattern: Optional[torch.Tensor] = None, pattern_len: Optional[torch.Tensor] = None,
                        status: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> None:
    """Appends emitted_tokens[b, :n_emitted[b]] to sequence req_seq[b] of the pool (in place), advances seq_len
    (in place) and, if given, refreshes pattern [B, p_max] / pattern_len [B] to the sequences' newest tokens."""
    lib = load_library()
    B, T = emitted_tokens.shape
    n_seq = seq_start.shape[0]
    _want(tokens, torch.int32, (tokens.shape[0],), "tokens")
    _want(seq_start, torch.int32, (n_seq,), "seq_start")
    _want(seq_len, torch.int32, (n_seq,), "seq_len")
    _want(seq_capacity, torch.int32, (n_seq,), "seq_capacity")
    _want(req_seq, torch.int32, (B,), "req_seq")
    _want(emitted_tokens, torch.int32, (B, T), "emitted_tokens")
    _want(n_emitted, torch.int32, (B,), "n_emitted")
    p_max = 1
    if pattern is not None:
        p_max = pattern.shape[1]
        _want(pattern, torch.int32, (B, p_max), "pattern")
        _want(pattern_len, torch.int32, (B,), "pattern_len")
    if status is not None:
        _want(status, torch.int32, (1,), "status")
    _check(lib.seer_history_append(_ptr(tokens), _ptr(seq_start), _ptr(seq_len), _ptr(seq_capacity), _ptr(req_seq),
                                   _ptr(emitted_tokens), _ptr(n_emitted), B, T, n_seq, tokens.shape[0], p_max,
                                   _ptr(pattern), _ptr(pattern_len), _ptr(status), _stream_handle(stream)))
