#!/usr/bin/env python3
"""Benchmark of the verification hot path on one MI355X.

A step = one pass of the whole hot path over one batch of synthetic input that
is already resident in HBM: seer_verify_attention (plan + partition kernel +
combine) followed by seer_accept (vocabulary argmax + acceptance walk), both
through the product entry points.  Headline workload: the "8B-class grouped
rollout" configuration (B=64 requests in 8 prompt groups, Hq=32, Hkv=8, D=128,
16-token pages, lognormal contexts, k=8 chain so T=9, V=152064); the long-tail,
shared-latent and multi-path configurations are measured the same way and
reported under "per_config" of the same JSON line.  Prints ONE JSON line.

Timing protocol.  The memory-side cache (256 MB) must not carry data from one
step to the next: every timed step works on another of R = 3 copies of the KV
pools, queries and logits at distinct addresses ("rotated"); the same loop on
one set of buffers is reported beside it.  Per step, GPU time between events
recorded on the stream: mean (the contract's ms_per_step comes from the wall
clock around exactly K steps), median and minimum.  The partition kernel's
duration comes from a second loop of K steps in which the library records two
events around that kernel on the stream it launches on.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config N | --configs 2,3,4,5] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E bandwidth
# HBM bytes per launch of the partition kernel as rocprofv3 counted them (FETCH_SIZE + WRITE_SIZE, scaled
# against a 1 GiB copy) in separate runs of this script; NOT measured by the run that prints them.
PROFILED_TRAFFIC = {
    2: (1.521e9, "profiles/attn_gqa128_config2_counters.md"),
    3: (3.082e9, "profiles/attn_gqa128_config3_counters.md"),
    4: (0.769e9, "profiles/attn_mla_config4_counters.md"),
    5: (5.818e9, "profiles/attn_gqa128_config5_counters.md"),
}
MFMA_BF16_PEAK_TFLOPS = 2500.0
METRIC = "verified tokens/s and verify-attention HBM GB/s (% of peak) on one MI355X"


class HipEvents:
    """hipEvent_t pairs made through the HIP runtime directly: they have to be recorded by the
    library on the stream it launches on, between its own kernels."""

    def __init__(self, n: int):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.pairs = []
        for _ in range(n):
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(a)) == 0
            assert self.hip.hipEventCreate(ctypes.byref(b)) == 0
            self.pairs.append((a.value, b.value))

    def elapsed_ms(self):
        out = []
        for a, b in self.pairs:
            ms = ctypes.c_float()
            rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
            assert rc == 0, rc
            out.append(ms.value)
        return out

    def close(self):
        for a, b in self.pairs:
            self.hip.hipEventDestroy(a)
            self.hip.hipEventDestroy(b)


def algorithmic_bytes(inp) -> dict:
    """Bytes the method has to move for one attention call: every KV page some request owns once
    (that single read serving all T slots and G heads is the point of verification), plus q and out."""
    cfg = inp.cfg
    q_bytes = cfg.B * cfg.T * cfg.Hq * cfg.Dqk * 2
    out_bytes = cfg.B * cfg.T * cfg.Hq * cfg.Dv * 2
    return {"kv_unique": inp.unique_kv_bytes, "kv_logical": inp.logical_kv_bytes, "q": q_bytes, "out": out_bytes,
            "total": inp.unique_kv_bytes + q_bytes + out_bytes}


def cpu_baseline(att, acc, row_token_budget: float = 4.0e8) -> dict:
    """The oracle, as it stands, on a bounded sample of the same workload: every k-th request by
    length rank (so the sample keeps the length mix), all T slots and heads, plus those requests'
    logits rows.  Reported in the metric's unit (verified tokens/s)."""
    import oracle
    cfg = att.cfg
    order = np.argsort(att.ctx_len, kind="stable")
    # bound the CPU work: (KV tokens) x (query rows per token) of the sample stays under the budget
    work_all = float(att.ctx_len.sum()) * cfg.T * cfg.Hq
    n_sample_requests = int(max(1, min(cfg.B, np.floor(cfg.B * row_token_budget / work_all))))
    step = max(1, cfg.B // n_sample_requests)
    pick = np.sort(order[step // 2::step][:n_sample_requests])
    t0 = time.perf_counter()
    oracle.verify_attention(att.q[pick], att.k_pages, att.v_pages, att.block_table[pick], att.ctx_len[pick],
                            None if att.tree_mask is None else att.tree_mask[pick], att.scale, Dv=cfg.Dv)
    t1 = time.perf_counter()
    oracle.verify_accept(acc.logits[pick], acc.draft_tokens[pick],
                         None if acc.tree_parent is None else acc.tree_parent[pick])
    t2 = time.perf_counter()
    tokens = len(pick) * cfg.T
    return {"value": tokens / (t2 - t0), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%d of %d requests (every %d-th by length rank; %d KV tokens of %d), all T=%d slots and "
                      "Hq=%d heads, and their %d logits rows; attention %.2f s + accept %.2f s" % (
                          len(pick), cfg.B, step, int(att.ctx_len[pick].sum()), int(att.ctx_len.sum()), cfg.T,
                          cfg.Hq, tokens, t1 - t0, t2 - t1)}


def sweep_step_time(torch, binding, W, attention_device_inputs) -> int:
    """T(B, gamma) of the verify step on this GPU for the 8B-class shape (config 2: 32/8 heads, D = 128,
    lognormal contexts), B = 1 .. 256, gamma = 0 .. 8, and what Algorithm 1 of the paper makes of it.
    One KV pool for 256 requests is generated once; batch size B uses its first B requests; queries and
    logits are random device tensors (timing only, no parity here)."""
    base = W.CONFIGS[2]
    gamma_max = 8
    cfg = base.scaled(B=256, group_size=8, T=gamma_max + 1)
    att = W.make_attention_inputs(cfg)
    d = attention_device_inputs(att)
    dev = d["q"].device
    batches = [1, 4, 16, 64, 128, 256]
    att_table, reuse_table, acc_table, draft_table = {}, {}, {}, {}
    busy = torch.randn((8192, 8192), device=dev, dtype=torch.bfloat16)
    busy_out = torch.empty_like(busy)
    # D(B, gamma): seer_draft on the token histories that go with the same 256 requests (chain of gamma tokens)
    dr = W.make_draft_inputs(cfg, gamma_max=gamma_max, top_k=1)
    t32 = lambda x: torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(dev)
    dr_dev = [t32(x) for x in (dr.tokens, dr.seq_start, dr.seq_len, dr.group_first)]
    # one allocation of each tensor at its largest size, cells take leading slices: the place of a buffer in
    # memory (which channels its lines fall on) moves these times by several per cent, and must not differ
    # from cell to cell
    Bmax, Tmax = max(batches), gamma_max + 1
    q_all = torch.randn(Bmax * Tmax * cfg.Hq * cfg.Dqk, device=dev).to(torch.bfloat16)
    logits_all = torch.randn(Bmax * Tmax * cfg.V, device=dev)
    ws_all = torch.empty(binding.seer_verify_attention_workspace(
        binding.attn_params(q_all.view(Bmax, Tmax, cfg.Hq, cfg.Dqk), d["k_pages"], d["v_pages"], d["block_table"], att.scale)),
        dtype=torch.uint8, device=dev)
    for B in batches:
        att_row, reuse_row, acc_row, drow = [], [], [], [0.0]
        for gamma in range(gamma_max + 1):
            T = gamma + 1
            q = q_all[:B * T * cfg.Hq * cfg.Dqk].view(B, T, cfg.Hq, cfg.Dqk)
            logits = logits_all[:B * T * cfg.V].view(B, T, cfg.V)
            draft = torch.zeros((B, T), dtype=torch.int32, device=dev)
            # the pool's contexts count 9 verify slots; shorten by the slots this gamma does not use
            n = (d["ctx_len"][:B] - (gamma_max + 1 - T)).contiguous()
            bt = d["block_table"][:B].contiguous()
            p = binding.attn_params(q, d["k_pages"], d["v_pages"], bt, att.scale)
            need = binding.seer_verify_attention_workspace(p)
            assert need <= ws_all.numel()
            ws = ws_all[:need]
            ws2 = torch.empty(max(16, binding.seer_accept_workspace(B, T, cfg.V)), dtype=torch.uint8, device=dev)

            def timed(fn):
                # a long matrix product first: while the GPU works on it the host enqueues all calls, so
                # the events see GPU time, not the time Python needs to issue a call
                for _ in range(12):         # also lets the stretch lengths settle on the measured speeds
                    fn()
                torch.mm(busy, busy, out=busy_out)
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for _ in range(20):
                    fn()
                b.record()
                torch.cuda.synchronize()
                return a.elapsed_time(b) / 20
            att_row.append(timed(lambda: binding.seer_verify_attention(q, d["k_pages"], d["v_pages"], bt, n, None, att.scale,
                                                                         workspace=ws)))
            reuse_row.append(timed(lambda: binding.seer_verify_attention(q, d["k_pages"], d["v_pages"], bt, n, None, att.scale,
                                                                           workspace=ws, flags=binding.SEER_ATTN_REUSE_PLAN)))
            acc_row.append(timed(lambda: binding.seer_accept(logits, draft, None, workspace=ws2)))
            if gamma >= 1:
                req = [t32(x[:B]) for x in (dr.req_group, dr.pattern, dr.pattern_len)] + [torch.full((B,), gamma, dtype=torch.int32, device=dev)]
                dp = binding.SeerDraftParams(B, len(dr.group_first) - 1, len(dr.seq_start), len(dr.tokens), dr.max_group_tokens,
                                             gamma, 1, dr.p_min, dr.p_max, cfg.V, 0.0)
                wsd = torch.empty(binding.seer_draft_workspace(dp), dtype=torch.uint8, device=dev)
                outs = (torch.empty((B, T), dtype=torch.int32, device=dev), torch.empty((B, T), dtype=torch.int32, device=dev),
                        torch.empty((B, T), dtype=torch.int64, device=dev), torch.empty((B, T), dtype=torch.int32, device=dev),
                        torch.empty(B, dtype=torch.int32, device=dev))
                drow.append(timed(lambda: binding.seer_draft(*dr_dev, *req, gamma_max=gamma, top_k=1, pattern_lookup_min=dr.p_min,
                                                              vocab=cfg.V, max_group_tokens=dr.max_group_tokens, workspace=wsd,
                                                              out=outs)))
        att_table[B], reuse_table[B], acc_table[B], draft_table[B] = att_row, reuse_row, acc_row, drow
    beta = [0.85 ** k for k in range(1, gamma_max + 2)]          # acceptance probability by draft position
    decisions, step_table, n_layers = {}, {}, 32
    for B in batches:
        B_h = max(1, B // 4)
        # the step time the policy sees (Section 3.4.1: D(B, gamma) + T(B, gamma)): the draft call, the attention
        # call once per layer (the first plans, the others reuse its plan), one acceptance call; the model's
        # GEMMs are outside this library
        both = [ta + (n_layers - 1) * tr + tc + td
                for ta, tr, tc, td in zip(att_table[B], reuse_table[B], acc_table[B], draft_table[B])]
        step_table[B] = both
        gh, gl, gs = binding.seer_mba_draft_lengths(B_h, B - B_h, beta, gamma_max, 2.0, both)
        decisions[B] = {"B_h": B_h, "B_l": B - B_h, "gamma_star": gs, "gamma_h": gh, "gamma_l": gl}
    print(json.dumps({"what": "GPU time (ms) of seer_verify_attention (one layer), seer_accept and seer_draft, config-2 shape; "
                              "row = batch size, column = gamma 0..8; step_time = attention + (n_layers - 1) x attention with the "
                              "first layer's plan + accept + draft",
                      "n_layers": n_layers, "attention_ms": att_table, "attention_reuse_plan_ms": reuse_table,
                      "accept_ms": acc_table, "draft_ms": draft_table,
                      "step_time_ms": step_table, "beta": beta, "lambda": 2.0, "policy": decisions}))
    return 0


def sweep_tp8_share(torch, binding, W, attention_device_inputs) -> int:
    """The verify-attention call on one GPU's share of a 72B-class dense model under 8-way tensor parallelism
    (the paper's second model: 64 query / 8 KV heads over 8 GPUs -> Hq = 8, Hkv = 1, G = 8 per GPU), prompt groups
    of 16, lognormal contexts as config 2 / config 5: chains of gamma = 0 .. 8 draft tokens and the 4 x 8
    multi-path tree, by batch size.  Per cell: GPU time of the call (planning included), of the call on the
    first layer's plan, of the partition kernel alone, and that kernel's rate against both rooflines (unique KV
    bytes over 8 TB/s; 4 * D * G * T flop per KV token over 2.5 PFLOP/s): with one KV head per GPU the same read
    serves twice the rows of the 8B-class shape, so the wide shapes are bound by the matrix cores."""
    dev = "cuda"
    rows = []
    shapes = [("chain", W.CONFIGS[2], (0, 2, 4, 8), (16, 64, 256)), ("tree 4x8", W.CONFIGS[5], (8,), (16, 64, 128))]
    for kind, base, gammas, batches in shapes:
        for B in batches:
            for gamma in gammas:
                T = 33 if kind != "chain" else gamma + 1
                cfg = base.scaled(B=B, group_size=16, Hq=8, Hkv=1, T=T)
                att = W.make_attention_inputs(cfg)
                d = attention_device_inputs(att)
                p = binding.attn_params(d["q"], d["k_pages"], d["v_pages"], d["block_table"], att.scale)
                ws = torch.empty(binding.seer_verify_attention_workspace(p), dtype=torch.uint8, device=dev)
                out = torch.empty((cfg.B, cfg.T, cfg.Hq, cfg.Dv), dtype=torch.bfloat16, device=dev)

                def call(flags=0, ev=None):
                    binding.seer_verify_attention(d["q"], d["k_pages"], d["v_pages"], d["block_table"], d["ctx_len"],
                                                  d["tree_mask"], att.scale, out=out, workspace=ws, flags=flags, events=ev)
                for _ in range(10):
                    call()
                ev = HipEvents(20)
                marks = [torch.cuda.Event(enable_timing=True) for _ in range(41)]
                for i in range(20):
                    marks[i].record()
                    call(0, ev.pairs[i])
                for i in range(20, 40):
                    marks[i].record()
                    call(binding.SEER_ATTN_REUSE_PLAN)
                marks[40].record()
                torch.cuda.synchronize()
                kern = float(np.median(ev.elapsed_ms()))
                ev.close()
                call_ms = float(np.median([marks[i].elapsed_time(marks[i + 1]) for i in range(20)]))
                reuse_ms = float(np.median([marks[i].elapsed_time(marks[i + 1]) for i in range(20, 40)]))
                ab = algorithmic_bytes(att)
                flops = 4.0 * cfg.Dqk * cfg.G * cfg.T * float(att.ctx_len.sum()) * cfg.Hkv
                rows.append({"draft": kind, "B": B, "gamma": gamma, "T": T, "rows_per_kv_head": cfg.G * cfg.T,
                             "kernel": binding.seer_verify_attention_kernel(p), "kv_tokens": int(att.ctx_len.sum()),
                             "call_ms": call_ms, "call_reuse_plan_ms": reuse_ms, "kernel_ms": kern,
                             "hbm_GBps": ab["total"] / kern / 1e6, "hbm_frac": ab["total"] / kern / 1e6 / HBM_PEAK_GBPS,
                             "TFLOPs": flops / kern / 1e9, "mfma_frac": flops / kern / 1e9 / MFMA_BF16_PEAK_TFLOPS})
                del d, ws, out
                torch.cuda.empty_cache()
    print(json.dumps({"what": "seer_verify_attention on one GPU's share of a 72B-class model under TP8 (Hq=8, Hkv=1, G=8, "
                              "D=128, page 16, groups of 16): medians of 20 calls, ms", "cells": rows}))
    return 0


def sweep_draft_acceptance(torch, binding, W) -> int:
    """Mean acceptance length (accepted draft tokens + the bonus token) of seer_draft's drafts against the tokens
    each request really produces next, by number of grouped references and by beam width: the measurement of the
    paper's Table 2 on this build's synthetic group histories (groups of 16 like the table's n = 15; one live
    request per group; gamma_max = 8)."""
    cfg = W.CONFIGS[5].scaled(B=16 * 64, group_size=16)
    dev = "cuda"
    t32 = lambda x: torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(dev)
    table = {}
    for top_k in (1, 2, 4):
        full = W.make_draft_inputs(cfg, gamma_max=8, top_k=top_k)
        for refs in (0, 1, 5, 15):
            d = W.restrict_draft_inputs(full, cfg.group_size, refs)
            tok, par, msk, cnt, mlen = binding.seer_draft(
                t32(d.tokens), t32(d.seq_start), t32(d.seq_len), t32(d.group_first), t32(d.req_group), t32(d.pattern),
                t32(d.pattern_len), t32(d.max_spec_tokens), gamma_max=8, top_k=top_k, pattern_lookup_min=d.p_min,
                vocab=cfg.V, max_group_tokens=max(d.max_group_tokens, 1))
            torch.cuda.synchronize()
            h_tok, h_par = tok.cpu().numpy(), par.cpu().numpy()
            total = 0
            for b in range(h_tok.shape[0]):
                depth, ok, best = {0: 0}, {0: True}, 0
                for s_ in range(1, h_tok.shape[1]):
                    p_ = int(h_par[b, s_])
                    if p_ < 0:
                        continue
                    depth[s_] = depth[p_] + 1
                    ok[s_] = ok[p_] and h_tok[b, s_] == d.future[b, depth[s_] - 1]
                    if ok[s_]:
                        best = max(best, depth[s_])
                total += best + 1
            table.setdefault("n=%d" % refs, {})["k=%d" % top_k] = round(total / h_tok.shape[0], 3)
    print(json.dumps({"what": "mean acceptance length incl. bonus token; rows = grouped references, columns = beam width "
                              "(k=1: linear); 64 groups of 16, one live request each, gamma_max 8, pattern 2..8",
                      "acceptance_length": table,
                      "paper_table_2": {"n=0": [1.70, 1.77, 1.85], "n=1": [2.04, 2.14, 2.25], "n=5": [2.32, 2.44, 2.59],
                                        "n=15": [2.53, 2.69, 2.85]}}))
    return 0


def _stats(ms) -> dict:
    a = np.asarray(ms, dtype=np.float64)
    return {"mean": float(a.mean()), "median": float(np.median(a)), "min": float(a.min()), "max": float(a.max())}


def measure_config(torch, binding, W, cfg, args, steps: int, warmup: int, extras: bool) -> dict:
    """One workload: the step (attention + accept) through the product entry points, rotated over R buffer
    sets and on one set; the partition kernel's duration; the reproducible (fixed-split) mode beside the
    default; the memory system's ceiling for the kernel's own load path."""
    from paper_2511_14617_amd.device_inputs import accept_device_inputs, attention_device_inputs
    att = W.make_attention_inputs(cfg)
    acc = W.make_accept_inputs(cfg, tree_parent=att.tree_parent)
    dev = "cuda"
    R = max(1, args.rotate)
    # R sets of everything a step reads in bulk, at distinct addresses (block tables, lengths and masks are
    # small and shared: the page ids are the same in every copy of the pools)
    d0, e0 = attention_device_inputs(att), accept_device_inputs(acc)
    sets = [(d0, e0)]
    for _ in range(1, R):
        d = dict(d0, q=d0["q"].clone(), k_pages=d0["k_pages"].clone(),
                 v_pages=None if d0["v_pages"] is None else d0["v_pages"].clone())
        sets.append((d, dict(e0, logits=e0["logits"].clone())))
    p = binding.attn_params(d0["q"], d0["k_pages"], d0["v_pages"], d0["block_table"], att.scale, Dv=cfg.Dv)
    ws_att = torch.empty(binding.seer_verify_attention_workspace(p), dtype=torch.uint8, device=dev)
    ws_acc = torch.empty(max(16, binding.seer_accept_workspace(cfg.B, cfg.T, cfg.V)), dtype=torch.uint8, device=dev)
    out = torch.empty((cfg.B, cfg.T, cfg.Hq, cfg.Dv), dtype=torch.bfloat16, device=dev)
    acc_out = (torch.empty(cfg.B, dtype=torch.int32, device=dev), torch.empty((cfg.B, cfg.T), dtype=torch.int32, device=dev),
               torch.empty(cfg.B, dtype=torch.int32, device=dev), torch.empty((cfg.B, cfg.T), dtype=torch.int32, device=dev))

    def attention(slot, flags=0, ev=None):
        d = sets[slot][0]
        binding.seer_verify_attention(d["q"], d["k_pages"], d["v_pages"], d["block_table"], d["ctx_len"],
                                      d["tree_mask"], att.scale, Dv=cfg.Dv, out=out, workspace=ws_att, flags=flags,
                                      events=ev)

    def accept(slot):
        e = sets[slot][1]
        binding.seer_accept(e["logits"], e["draft_tokens"], e["tree_parent"], workspace=ws_acc, out=acc_out)

    def step(slot, flags=0, ev=None):
        attention(slot, flags, ev)
        if not args.attention_only:
            accept(slot)

    def timed_steps(n, rotate, flags=0):
        """n steps through the product entry points: (wall-clock ms per step, per-step GPU ms)."""
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            marks[i].record()
            step(i % R if rotate else 0, flags)
        marks[n].record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / n
        return wall, [marks[i].elapsed_time(marks[i + 1]) for i in range(n)]

    def kernel_times(n, rotate, flags=0):
        """Partition-kernel durations of n steps (events recorded by the library around that kernel)."""
        ev = HipEvents(n)
        for i in range(n):
            step(i % R if rotate else 0, flags, ev.pairs[i])
        torch.cuda.synchronize()
        ms = ev.elapsed_ms()
        ev.close()
        return ms

    for i in range(warmup):
        step(i % R)
    # ---- the timed region: exactly `steps` steps, rotated buffers, product entry points
    ms_per_step, step_gpu = timed_steps(steps, rotate=True)
    emitted = None if args.attention_only else int(acc_out[0].sum().item()) + cfg.B
    kern = kernel_times(steps, rotate=True)
    # ---- the same on one set of buffers (what the memory-side cache carries from step to step shows here)
    n_side = max(5, steps // 2)
    same_wall, same_gpu = timed_steps(n_side, rotate=False)
    same_kern = kernel_times(n_side, rotate=False)
    # ---- the reproducible mode: equal stretches, output bits independent of earlier calls
    fixed_wall, fixed_gpu = timed_steps(n_side, rotate=True, flags=binding.SEER_ATTN_FIXED_SPLIT)
    fixed_kern = kernel_times(n_side, rotate=True, flags=binding.SEER_ATTN_FIXED_SPLIT)
    for i in range(4):          # let the default mode's stretch lengths settle again
        step(i % R)

    # ---- split of a step between the calls (GPU time; a queue of matrix products first, so that the host
    # has enqueued the calls before the GPU reaches them)
    busy = torch.randn((4096, 4096), device=dev, dtype=torch.bfloat16)
    busy_out = torch.empty_like(busy)

    def timed(fn, n=10, queue_first=4):
        for _ in range(int(queue_first)):
            torch.mm(busy, busy, out=busy_out)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        for i in range(n):
            marks[i].record()
            fn(i)
        marks[n].record()
        torch.cuda.synchronize()
        return float(np.median([marks[i].elapsed_time(marks[i + 1]) for i in range(n)]))

    att_ms = timed(lambda i: attention(i % R))
    att_reuse_ms = timed(lambda i: attention(0, binding.SEER_ATTN_REUSE_PLAN))   # layers 2.. of a step: same KV
    acc_ms = 0.0 if args.attention_only else timed(lambda i: accept(i % R))
    # gather-read ceiling: the same call with the arithmetic left out of the tiled kernel (D = 128 shapes)
    kernel_name = binding.seer_verify_attention_kernel(p)
    ceiling = None
    if kernel_name.startswith("attn_gqa128"):
        ceiling = _stats(kernel_times(10, rotate=True, flags=binding.SEER_ATTN_STREAM_ONLY)[2:])

    result_extras = {}
    if extras and not args.attention_only:
        e = sets[0][1]
        d = sets[0][0]
        sampled_ms = timed(lambda i: binding.seer_accept_sampled(e["logits"], e["draft_tokens"], e["tree_parent"], 0.8,
                                                                 20251114, workspace=ws_acc, out=acc_out))
        accept(0)
        n_copy = d["ctx_len"].clone()

        def commit(i):
            n_copy.copy_(d["ctx_len"])
            binding.seer_kv_commit(d["k_pages"], d["v_pages"], d["block_table"], n_copy, acc_out[0], acc_out[1])
        commit_ms = timed(commit, queue_first=40)    # two short kernels: timed by the GPU's clock, not by Python's
        # the online acceptance statistics of the step (what the draft-length policy reads), and beta from them
        counts = torch.zeros((3, cfg.T), dtype=torch.int64, device=dev)
        stats_ms = timed(lambda i: binding.seer_acceptance_stats(acc_out[0], acc_out[1], e["tree_parent"], counts),
                         queue_first=40)
        counts.zero_()
        binding.seer_acceptance_stats(acc_out[0], acc_out[1], e["tree_parent"], counts)
        h_counts = counts.cpu().tolist()
        beta = binding.seer_acceptance_beta(h_counts, False, 0.0)[:sum(1 for x in h_counts[0][1:] if x > 0)]
        # the step before verification: drafts from the groups' token histories
        top_k, gamma = cfg.tree if cfg.tree else (1, cfg.T - 1)
        dr = W.make_draft_inputs(cfg, gamma_max=gamma, top_k=top_k)
        t32 = lambda x: torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(dev)
        dd = [t32(x) for x in (dr.tokens, dr.seq_start, dr.seq_len, dr.group_first, dr.req_group, dr.pattern,
                               dr.pattern_len, dr.max_spec_tokens)]
        dp = binding.SeerDraftParams(cfg.B, len(dr.group_first) - 1, len(dr.seq_start), len(dr.tokens),
                                     dr.max_group_tokens, gamma, top_k, dr.p_min, dr.p_max, cfg.V, 0.0)
        ws_dr = torch.empty(binding.seer_draft_workspace(dp), dtype=torch.uint8, device=dev)
        dr_out = (torch.empty((cfg.B, dr.T), dtype=torch.int32, device=dev), torch.empty((cfg.B, dr.T), dtype=torch.int32, device=dev),
                  torch.empty((cfg.B, dr.T), dtype=torch.int64, device=dev), torch.empty((cfg.B, dr.T), dtype=torch.int32, device=dev),
                  torch.empty(cfg.B, dtype=torch.int32, device=dev))

        def draft(i=0):
            binding.seer_draft(*dd, gamma_max=gamma, top_k=top_k, pattern_lookup_min=dr.p_min, vocab=cfg.V,
                               max_group_tokens=dr.max_group_tokens, workspace=ws_dr, out=dr_out)
        draft()
        draft_ms = timed(draft, n=20)
        live_groups = sorted(set(int(g) for g in dr.req_group))
        scanned = int(sum(int(dr.seq_len[dr.group_first[g]:dr.group_first[g + 1]].sum()) for g in live_groups))
        result_extras = {"accept_sampled_ms": sampled_ms, "kv_commit_ms": commit_ms,
                         "acceptance_stats": {"ms": stats_ms, "beta_by_draft_position": [round(x, 4) for x in beta]},
                         "draft": {"draft_ms": draft_ms, "top_k": top_k, "gamma_max": gamma,
                                   "pattern_lookup": [dr.p_min, dr.p_max], "history_tokens": scanned,
                                   "history_bytes": scanned * 4,
                                   "mean_match_len": float(dr_out[4].float().mean().item()),
                                   "max_match_places": int(dr_out[3][:, 0].max().item()),
                                   "mean_draft_nodes": float((dr_out[1][:, 1:] >= 0).sum(1).float().mean().item())}}
    if args.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    status = binding.seer_verify_attention_status(ws_att)

    ab = algorithmic_bytes(att)
    k_rot, k_same, k_fixed = _stats(kern), _stats(same_kern), _stats(fixed_kern)
    traffic = PROFILED_TRAFFIC.get(cfg.config_id) if args.ctx_scale == 1.0 else None
    common = {"kernel": kernel_name + " (verify-attention partition kernel)",
              "traffic": traffic[0] if traffic else None,
              "traffic_source": (traffic[1] + " (rocprofv3 --pmc runs of this script; not measured by this run)") if traffic else None,
              "algorithmic_bytes": ab,
              "kernel_ms_avg": k_rot["mean"], "kernel_ms_median": k_rot["median"], "kernel_ms_min": k_rot["min"],
              "buffers": "rotated over %d sets of KV pools, queries and logits" % R}
    if cfg.shared_latent:
        # the shared-latent shape is bound by the matrix cores: every KV token meets all Hq*T query rows
        flops = 2.0 * float(att.ctx_len.sum()) * cfg.T * cfg.Hq * (cfg.Dqk + cfg.Dv)
        rate = lambda ms: flops / (ms * 1e-3) / 1e12
        roofline = dict({"bound": "mfma", "achieved": rate(k_rot["mean"]), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": rate(k_rot["mean"]) / MFMA_BF16_PEAK_TFLOPS, "algorithmic_flops": flops}, **common)
        peak = MFMA_BF16_PEAK_TFLOPS
    else:
        rate = lambda ms: ab["total"] / (ms * 1e-3) / 1e9
        roofline = dict({"bound": "hbm", "achieved": rate(k_rot["mean"]), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": rate(k_rot["mean"]) / HBM_PEAK_GBPS}, **common)
        peak = HBM_PEAK_GBPS
        if ceiling:
            roofline["gather_read_ceiling"] = {"GBps": rate(ceiling["median"]), "kernel_ms": ceiling["median"],
                                               "achieved_over_ceiling": ceiling["median"] / k_rot["median"]}
    roofline["frac_median"] = rate(k_rot["median"]) / peak
    roofline["same_buffers"] = {"kernel_ms_avg": k_same["mean"], "kernel_ms_median": k_same["median"],
                                "kernel_ms_min": k_same["min"], "frac": rate(k_same["mean"]) / peak}
    roofline["fixed_split"] = {"kernel_ms_avg": k_fixed["mean"], "kernel_ms_median": k_fixed["median"],
                               "kernel_ms_min": k_fixed["min"], "frac": rate(k_fixed["mean"]) / peak,
                               "ms_per_step": fixed_wall, "step_gpu_ms_median": float(np.median(fixed_gpu))}
    tokens = cfg.B * cfg.T
    g = _stats(step_gpu)
    leg = {
        "value": tokens / (ms_per_step * 1e-3), "unit": "tokens/s", "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "step_gpu_ms_median": g["median"], "step_gpu_ms_min": g["min"],
        "step_gpu_ms_mean": g["mean"],
        "same_buffers": {"ms_per_step": same_wall, "step_gpu_ms_median": float(np.median(same_gpu)),
                         "step_gpu_ms_min": float(np.min(same_gpu)), "steps": n_side},
        "config": {"workload": "config%d %s: B=%d (%d groups x %d), Hq=%d, Hkv=%d, Dqk=%d, Dv=%d, page=%d, T=%d, "
                               "V=%d, ctx %s, step = seer_verify_attention + seer_accept" % (
                                   cfg.config_id, cfg.name, cfg.B, cfg.B // cfg.group_size, cfg.group_size, cfg.Hq,
                                   cfg.Hkv, cfg.Dqk, cfg.Dv, cfg.page_size, cfg.T, cfg.V, list(cfg.ctx)),
                   "kv_tokens": int(att.ctx_len.sum()), "seed": cfg.seed,
                   "attention_only": bool(args.attention_only)},
        "roofline": roofline,
        "attention_ms": att_ms, "attention_reuse_plan_ms": att_reuse_ms, "accept_ms": acc_ms,
        "attention_kv_GBps": ab["kv_unique"] / (att_ms * 1e-3) / 1e9,
        "accept_logits_GBps": (acc.logits.nbytes / (acc_ms * 1e-3) / 1e9) if acc_ms > 0 else None,
        "emitted_tokens_per_s": None if emitted is None else emitted / (ms_per_step * 1e-3),
        "mean_emitted_per_request": None if emitted is None else emitted / cfg.B,
        "attention_status_word": status,
    }
    leg.update(result_extras)
    if not args.no_cpu_baseline and extras:
        leg["cpu_baseline"] = cpu_baseline(att, acc)
    del sets, d0, e0, out, ws_att, ws_acc, busy, busy_out
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    return leg


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=6)
    ap.add_argument("--config", type=int, default=None, help="measure this workload (1..5) alone")
    ap.add_argument("--configs", type=str, default="2,3,4,5",
                    help="workloads to measure; the first is the headline of the JSON line, the others go under "
                         "per_config (default: 2 = the headline configuration, then 3, 4, 5)")
    ap.add_argument("--rotate", type=int, default=3, help="sets of KV pools / queries / logits the timed steps cycle through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--attention-only", action="store_true", help="time only seer_verify_attention (profiling aid)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed region, run three 1 GiB device-to-device tensor copies: a plain copy "
                         "kernel of known size against which rocprofv3 FETCH_SIZE / WRITE_SIZE are scaled")
    ap.add_argument("--ctx-scale", type=float, default=1.0,
                    help="experiment aid: scale every context-length bound of the workload (not the headline run)")
    ap.add_argument("--sweep-step-time", action="store_true",
                    help="instead of the benchmark: measure the verify step (attention + accept) of the config-2 "
                         "model shape over batch sizes and draft lengths, the T(B, gamma) table that the "
                         "draft-length policy consumes, and print it with the policy's decisions as JSON")
    ap.add_argument("--sweep-tp8-share", action="store_true",
                    help="instead of the benchmark: the attention call on the tensor-parallel share of a 72B-class "
                         "model (Hq = 8, Hkv = 1, groups of 16), chains and the 4 x 8 tree, by batch size")
    ap.add_argument("--sweep-draft-acceptance", action="store_true",
                    help="instead of the benchmark: mean acceptance length of seer_draft's drafts by number of grouped "
                         "references and beam width (the measurement of the paper's Table 2, on synthetic histories)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path shards by request with no exchange step; "
              "no multi-GPU figure is produced). Re-run with --gpus 1.", file=sys.stderr)
        return 2

    import torch
    from paper_2511_14617_amd import binding, workloads as W
    from paper_2511_14617_amd.device_inputs import attention_device_inputs

    binding.load_library()   # fails loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    if args.sweep_step_time:
        return sweep_step_time(torch, binding, W, attention_device_inputs)
    if args.sweep_tp8_share:
        return sweep_tp8_share(torch, binding, W, attention_device_inputs)
    if args.sweep_draft_acceptance:
        return sweep_draft_acceptance(torch, binding, W)
    ids = [args.config] if args.config is not None else [int(x) for x in args.configs.split(",") if x.strip()]

    def config_of(i):
        cfg = W.CONFIGS[i]
        if args.ctx_scale != 1.0:
            c = cfg.ctx
            scaled = tuple(int(round(x * args.ctx_scale)) if (isinstance(x, (int, float)) and x > 1.5) else x for x in c[1:])
            cfg = cfg.scaled(ctx=(c[0],) + scaled)
        return cfg

    head = measure_config(torch, binding, W, config_of(ids[0]), args, args.steps, args.warmup, extras=True)
    line = {
        "metric": METRIC,
        "value": head["value"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
    }
    for k, v in head.items():
        if k not in line:
            line[k] = v
    # the other named workloads, each measured the same way (fewer steps: the headline is the timed job)
    per_config = {}
    for i in ids[1:]:
        per_config["config%d" % i] = measure_config(torch, binding, W, config_of(i), args, max(10, args.steps // 2),
                                                    args.warmup, extras=False)
    if per_config:
        line["per_config"] = per_config
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
