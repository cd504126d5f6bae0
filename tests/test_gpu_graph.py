"""The calls of a decoding step recorded into a HIP graph (torch.cuda.graph) and replayed: every replay must give
what the same calls give when issued directly.  The library launches kernels only (no memset, no allocation,
no synchronisation), so a caller can capture it as it is; the replays are interleaved with direct work."""
import numpy as np
import pytest
import torch

from paper_2511_14617_amd import workloads as W
from gpu_util import accept_device_inputs, attention_device_inputs

pytestmark = pytest.mark.gpu


def test_step_recorded_in_a_graph_replays_to_the_same_results():
    from paper_2511_14617_amd import binding
    cfg = W.CONFIGS[5].scaled(B=12, group_size=4, V=5003, ctx=("lognormal", 900, 0.8, 100, 2500))
    att = W.make_attention_inputs(cfg, dedup_fraction=0.3)
    acc = W.make_accept_inputs(cfg, tree_parent=att.tree_parent)
    dr = W.make_draft_inputs(cfg, gamma_max=8, top_k=4, n_phrases=64, phrase_prob=0.6)
    d, e = attention_device_inputs(att), accept_device_inputs(acc)
    dev = d["q"].device
    t32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    dd = [t32(x) for x in (dr.tokens, dr.seq_start, dr.seq_len, dr.group_first, dr.req_group, dr.pattern, dr.pattern_len,
                           dr.max_spec_tokens)]
    p = binding.attn_params(d["q"], d["k_pages"], d["v_pages"], d["block_table"], att.scale, Dv=cfg.Dv)
    ws_att = torch.empty(binding.seer_verify_attention_workspace(p), dtype=torch.uint8, device=dev)
    ws_acc = torch.empty(max(16, binding.seer_accept_workspace(cfg.B, cfg.T, cfg.V)), dtype=torch.uint8, device=dev)
    dp = binding.SeerDraftParams(cfg.B, len(dr.group_first) - 1, len(dr.seq_start), len(dr.tokens), dr.max_group_tokens,
                                 8, 4, dr.p_min, dr.p_max, cfg.V, 0.0)
    ws_dr = torch.empty(binding.seer_draft_workspace(dp), dtype=torch.uint8, device=dev)

    def buffers():
        i32 = lambda *s: torch.empty(s, dtype=torch.int32, device=dev)
        return dict(out=torch.empty((cfg.B, cfg.T, cfg.Hq, cfg.Dv), dtype=torch.bfloat16, device=dev),
                    acc=(i32(cfg.B), i32(cfg.B, cfg.T), i32(cfg.B), i32(cfg.B, cfg.T)),
                    dr=(i32(cfg.B, dr.T), i32(cfg.B, dr.T), torch.empty((cfg.B, dr.T), dtype=torch.int64, device=dev),
                        i32(cfg.B, dr.T), i32(cfg.B)))

    def step(buf, q):
        binding.seer_draft(*dd, gamma_max=8, top_k=4, pattern_lookup_min=dr.p_min, vocab=cfg.V,
                           max_group_tokens=dr.max_group_tokens, workspace=ws_dr, out=buf["dr"])
        binding.seer_verify_attention(q, d["k_pages"], d["v_pages"], d["block_table"], d["ctx_len"], d["tree_mask"],
                                      att.scale, Dv=cfg.Dv, out=buf["out"], workspace=ws_att,
                                      flags=binding.SEER_ATTN_FIXED_SPLIT)
        binding.seer_accept(e["logits"], e["draft_tokens"], e["tree_parent"], workspace=ws_acc, out=buf["acc"])

    q_graph = d["q"].clone()                                  # the graph reads its queries from here
    eager, graphed = buffers(), buffers()
    step(eager, d["q"])                                       # warm-up outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step(graphed, q_graph)
    torch.cuda.current_stream().wait_stream(side)

    def same(a, b):
        return torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a, b.view(torch.int16) if b.dtype == torch.bfloat16 else b)

    for replay in range(4):
        # other queries each time ("the next layer"), direct work between the replays
        q_now = torch.roll(d["q"], shifts=replay, dims=2).contiguous()
        step(eager, q_now)
        torch.cuda.synchronize()
        for t in graphed["acc"] + graphed["dr"] + (graphed["out"],):
            t.zero_()
        q_graph.copy_(q_now)
        graph.replay()
        torch.cuda.synchronize()
        assert same(graphed["out"], eager["out"]), "attention, replay %d" % replay
        for g_, e_ in zip(graphed["acc"] + graphed["dr"], eager["acc"] + eager["dr"]):
            assert same(g_, e_), "replay %d" % replay
    assert binding.seer_verify_attention_status(ws_att) == 0
