"""GPU parity for seer_verify_attention against the CPU oracle, through the C ABI.
Sizes here are ones the oracle finishes in seconds; they still span several
KV tiles, several split-K partitions and ragged last pages."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_14617_amd import workloads as W
from gpu_util import assert_attention_close, attention_device_inputs

pytestmark = pytest.mark.gpu


def _oracle(inp):
    return oracle.verify_attention(inp.q, inp.k_pages, inp.v_pages, inp.block_table, inp.ctx_len, inp.tree_mask,
                                   inp.scale, Dv=inp.cfg.Dv)


def _oracle_abs(inp):
    """sum_j p_j |v_j|: the oracle on the same inputs with the sign bit of every V cleared (with a
    shared latent: an explicit V pool made of the latent's first Dv components, sign cleared)."""
    v = inp.v_pages if inp.v_pages is not None else np.ascontiguousarray(inp.k_pages[..., : inp.cfg.Dv])
    return oracle.verify_attention(inp.q, inp.k_pages, v & np.uint16(0x7FFF), inp.block_table,
                                   inp.ctx_len, inp.tree_mask, inp.scale)


def _gpu(inp, **kw):
    from paper_2511_14617_amd import binding
    d = attention_device_inputs(inp)
    out = binding.seer_verify_attention(d["q"], d["k_pages"], d["v_pages"], d["block_table"], d["ctx_len"],
                                        d["tree_mask"], inp.scale, Dv=inp.cfg.Dv, **kw)
    torch.cuda.synchronize()
    return out


CASES = {
    "tiny_chain": (W.CONFIGS[1], {}),
    "chain_T9_multi_split": (W.CONFIGS[2].scaled(B=6, group_size=3, ctx=("uniform", 600, 3000)), {}),
    "chain_T17": (W.CONFIGS[3].scaled(B=2, ctx=("uniform", 1500, 2600)), {}),
    "tree_T33": (W.CONFIGS[5].scaled(B=5, group_size=5, ctx=("lognormal", 900, 0.8, 100, 2500)),
                 {"dedup_fraction": 0.4}),
    "mla_latent": (W.CONFIGS[4].scaled(B=2, Hq=16, ctx=("uniform", 300, 900)), {}),
    "T1_decode": (W.CONFIGS[1].scaled(T=1, B=5, ctx=("uniform", 1, 700)), {}),
    "prefix_shorter_than_draft": (W.CONFIGS[1].scaled(T=9, B=6, ctx=("uniform", 9, 40)), {}),
    "many_short_requests": (W.CONFIGS[2].scaled(B=300, group_size=6, T=4, ctx=("uniform", 4, 150), shared_prefix=32), {}),
    "many_short_mla": (W.CONFIGS[4].scaled(B=40, Hq=32, T=3, ctx=("uniform", 3, 200)), {}),
    # four to eight waves per workgroup of the tiled kernel (32 query rows each)
    "rows100_T25": (W.CONFIGS[2].scaled(B=3, group_size=3, T=25, ctx=("uniform", 300, 1500)), {}),
    "rows168_G8_T21": (W.CONFIGS[2].scaled(B=3, group_size=3, Hq=16, Hkv=2, T=21, ctx=("uniform", 300, 1500)), {}),
    "rows224_G8_T28": (W.CONFIGS[2].scaled(B=2, group_size=2, Hq=16, Hkv=2, T=28, ctx=("uniform", 200, 1200)), {}),
    "rows256_G8_T32": (W.CONFIGS[2].scaled(B=2, group_size=2, Hq=8, Hkv=1, T=32, ctx=("uniform", 200, 1200)), {}),
    # 129 .. 144 rows per KV head: four main waves plus four helper waves that share the leftover rows tile by tile
    # (pieces shorter than four tiles leave some helpers without a tile; ragged tails; chain and tree masks)
    "rows129_G3_T43": (W.CONFIGS[2].scaled(B=4, group_size=4, Hq=6, Hkv=2, T=43, ctx=("uniform", 43, 1500), shared_prefix=0), {}),
    "rows144_G16_T9": (W.CONFIGS[2].scaled(B=5, group_size=5, Hq=32, Hkv=2, T=9, ctx=("uniform", 9, 2500), shared_prefix=64), {}),
    "rows132_tree_short": (W.CONFIGS[5].scaled(B=9, group_size=3, ctx=("uniform", 33, 140), shared_prefix=0),
                           {"dedup_fraction": 0.3}),
    "rows132_tree_page64": (W.CONFIGS[5].scaled(B=4, group_size=4, page_size=64, ctx=("uniform", 500, 4000), shared_prefix=128),
                            {"dedup_fraction": 0.3}),
    # one GPU's share of a 72B-class model under 8-way tensor parallelism (Section 4.1: 64 query / 8 KV
    # heads split over 8 GPUs -> Hq = 8, Hkv = 1, G = 8), groups of 16 requests, gamma = 8 and a 4 x 8 tree
    "tp8_share_72b_chain": (W.CONFIGS[2].scaled(B=16, group_size=16, Hq=8, Hkv=1, T=9, ctx=("uniform", 200, 2500),
                                               shared_prefix=256), {}),
    "tp8_share_72b_tree": (W.CONFIGS[5].scaled(B=16, group_size=16, Hq=8, Hkv=1, ctx=("uniform", 100, 1500),
                                              shared_prefix=256), {"dedup_fraction": 0.3}),
    # 265 rows per KV head: two row blocks of 133 and 132 rows, each four main waves plus four helper waves
    "rows265_two_helper_blocks": (W.CONFIGS[2].scaled(B=3, group_size=3, Hq=5, Hkv=1, T=53, ctx=("uniform", 53, 1500),
                                                     shared_prefix=64), {}),
    # more than 256 query rows per KV head: the tiled kernel cuts them into row blocks (528 rows -> 3 blocks)
    "rows528_G16_T33": (W.CONFIGS[5].scaled(B=3, group_size=3, Hq=32, Hkv=2, ctx=("uniform", 200, 1500),
                                            shared_prefix=0), {"dedup_fraction": 0.3}),
    # prompt pages shared inside a group over more than one 64-page window of the block table, with stretch
    # borders inside the shared run (tiles of the run are loaded under another cache policy than the rest)
    "shared_prompt_1100": (W.CONFIGS[2].scaled(B=6, group_size=3, ctx=("uniform", 1200, 3000), shared_prefix=1100), {}),
    "shared_prompt_rows100": (W.CONFIGS[2].scaled(B=4, group_size=2, T=25, ctx=("uniform", 800, 2000), shared_prefix=700), {}),
    "shared_prompt_tree_helpers": (W.CONFIGS[5].scaled(B=4, group_size=4, ctx=("uniform", 1300, 2500), shared_prefix=1200),
                                   {"dedup_fraction": 0.3}),
    # larger pages with the tiled D = 128 kernel (a 32-token tile lies inside one page)
    "d128_page64": (W.CONFIGS[2].scaled(B=5, group_size=5, page_size=64, ctx=("uniform", 9, 1500), shared_prefix=128), {}),
    "d128_page256_tree": (W.CONFIGS[5].scaled(B=4, group_size=4, page_size=256, ctx=("uniform", 33, 1200),
                                              shared_prefix=256), {"dedup_fraction": 0.3}),
    "mla_page32": (W.CONFIGS[4].scaled(B=2, Hq=16, page_size=32, ctx=("uniform", 100, 700)), {}),
    "mla_page128": (W.CONFIGS[4].scaled(B=2, Hq=16, page_size=128, ctx=("uniform", 100, 700)), {}),
    "mha_d64": (W.CONFIGS[1].scaled(Hq=4, Hkv=4, Dqk=64, Dv=64, page_size=8, ctx=("uniform", 50, 900)), {}),
    # batches whose partial results exceed 64 MB: the kernel variants that write them with plain stores
    # (two waves: through the LDS ring; four waves: directly)
    "large_partials_two_waves": (W.CONFIGS[2].scaled(B=340, group_size=4, T=9, ctx=("uniform", 9, 120), shared_prefix=0), {}),
    "large_partials_four_waves": (W.CONFIGS[2].scaled(B=72, group_size=4, T=32, ctx=("uniform", 32, 200), shared_prefix=0), {}),
    # the most verify slots a call takes (the mask word is full): every kernel, chain and tree
    "T64_chain_rows256": (W.CONFIGS[2].scaled(B=2, group_size=2, Hq=8, Hkv=2, T=64, ctx=("uniform", 64, 1200),
                                              shared_prefix=0), {}),
    "T64_tree_two_row_blocks": (W.CONFIGS[5].scaled(B=3, group_size=3, Hq=16, Hkv=2, T=64, tree=(7, 9),
                                                    ctx=("uniform", 64, 1200), shared_prefix=0), {"dedup_fraction": 0.3}),
    "T64_mla": (W.CONFIGS[4].scaled(B=2, Hq=16, T=64, ctx=("uniform", 100, 700)), {}),
    "T64_mha_d64": (W.CONFIGS[1].scaled(Hq=4, Hkv=4, Dqk=64, Dv=64, page_size=8, T=64, ctx=("uniform", 64, 500)), {}),
    "g8_d256_page32": (W.CONFIGS[1].scaled(Hq=8, Hkv=1, Dqk=256, Dv=256, page_size=32,
                                           ctx=("uniform", 50, 900)), {}),
}


@pytest.mark.parametrize("values", ["paper", "peaked"])
@pytest.mark.parametrize("name", sorted(CASES))
def test_parity_small(name, values):
    cfg, kw = CASES[name]
    inp = W.make_attention_inputs(cfg, values=values, **kw)
    ref = _oracle(inp)
    ref_abs = _oracle_abs(inp) if values == "peaked" else None
    out = _gpu(inp)
    assert_attention_close(out, ref, "%s/%s" % (name, values), hardened=(values == "peaked"), ref_abs=ref_abs)


@pytest.mark.parametrize("name", ["tiny_chain", "chain_T9_multi_split", "tree_T33"])
def test_parity_small_general_kernel(name):
    """The general kernel on shapes that normally take the tiled one."""
    from paper_2511_14617_amd import binding
    cfg, kw = CASES[name]
    inp = W.make_attention_inputs(cfg, values="peaked", **kw)
    ref = _oracle(inp)
    out = _gpu(inp, flags=binding.SEER_ATTN_GENERAL_KERNEL)
    assert_attention_close(out, ref, name + "/general", hardened=True)


@pytest.mark.parametrize("name", ["shared_prompt_1100", "shared_prompt_rows100", "shared_prompt_tree_helpers"])
def test_shared_prompt_long_pieces(name):
    """Few, long pieces (a cap of two pieces per request): the unrolled steady state of the tiled kernel runs through
    the shared run of tiles and out of it."""
    cfg, kw = CASES[name]
    inp = W.make_attention_inputs(cfg, values="peaked", **kw)
    ref = _oracle(inp)
    out = _gpu(inp, max_splits=2)
    assert_attention_close(out, ref, name + "/two pieces", hardened=True, ref_abs=_oracle_abs(inp))


def test_requests_that_map_the_same_pages_throughout():
    """Two requests with one and the same block-table row and length (every tile, the draft slots' included, counts as
    shared: the whole request is read under the keeping cache policy), next to requests that share nothing."""
    cfg = W.CONFIGS[2].scaled(B=4, group_size=1, ctx=("uniform", 700, 1500), shared_prefix=0)
    inp = W.make_attention_inputs(cfg, values="peaked")
    inp.block_table[2] = inp.block_table[1]
    inp.ctx_len[2] = inp.ctx_len[1]
    ref = _oracle(inp)
    out = _gpu(inp)
    assert_attention_close(out, ref, "identical block-table rows", hardened=True, ref_abs=_oracle_abs(inp))


def _leading_common_pages(inp):
    """Per request: the longest run of leading block-table entries equal to those of the request before or after it."""
    P, n = inp.cfg.page_size, inp.ctx_len
    pages = (n + P - 1) // P
    best = np.zeros(len(n), dtype=np.int64)
    for b in range(len(n)):
        for nb in (b - 1, b + 1):
            if 0 <= nb < len(n):
                m = int(min(pages[b], pages[nb]))
                same = inp.block_table[b, :m] == inp.block_table[nb, :m]
                best[b] = max(best[b], m if same.all() else int(np.argmin(same)))
    return best


@pytest.mark.parametrize("prefix", [0, 16, 32, 48, 272, 512, 528, 1040, 4240, 16400])
def test_plan_finds_the_pages_a_group_shares(prefix):
    """The plan's count of leading tiles that a neighbouring request maps too (a cache-policy hint for the tiled
    kernel) against a direct comparison of the block tables: exact for runs of up to 32 pages, else short by less
    than a sixteenth of the run (it probes 16 + 16 entries), never long."""
    from paper_2511_14617_amd import binding
    cfg = W.CONFIGS[2].scaled(B=7, group_size=3, Hq=4, Hkv=1, ctx=("uniform", prefix + 9, prefix + 700), shared_prefix=prefix)
    inp = W.make_attention_inputs(cfg)
    d = attention_device_inputs(inp)
    p = binding.attn_params(d["q"], d["k_pages"], d["v_pages"], d["block_table"], inp.scale, Dv=cfg.Dv)
    ws = torch.zeros(binding.seer_verify_attention_workspace(p), dtype=torch.uint8, device="cuda")
    binding.seer_verify_attention(d["q"], d["k_pages"], d["v_pages"], d["block_table"], d["ctx_len"], d["tree_mask"],
                                  inp.scale, Dv=cfg.Dv, workspace=ws)
    got = binding.seer_verify_attention_shared_tiles(ws, p).numpy().astype(np.int64)
    true_pages = _leading_common_pages(inp)
    if prefix >= cfg.page_size:
        assert true_pages.max() >= prefix // cfg.page_size     # the generator did share the prompt's pages
    per_tile = 32 // cfg.page_size
    assert (got <= true_pages // per_tile).all(), (got, true_pages)
    slack = np.where(true_pages <= 32, 0, (true_pages + 15) // 16)
    assert (got >= (true_pages - slack) // per_tile).all(), (got, true_pages)


def test_split_invariance_and_split_cap():
    cfg = W.CONFIGS[2].scaled(B=3, group_size=3, ctx=("uniform", 2000, 5000))
    inp = W.make_attention_inputs(cfg, values="peaked")
    ref = _oracle(inp)
    ref_abs = _oracle_abs(inp)
    one = _gpu(inp, max_splits=1)
    many = _gpu(inp, max_splits=256)
    two = _gpu(inp, max_splits=2)
    for o, what in ((one, "S=1"), (many, "S<=256"), (two, "S<=2")):
        assert_attention_close(o, ref, what, hardened=True, ref_abs=ref_abs)


def test_constant_V_and_key_shift():
    cfg = W.CONFIGS[2].scaled(B=2, group_size=2, ctx=("uniform", 700, 1800))
    inp = W.make_attention_inputs(cfg, values="peaked")
    c = W.f32_to_bf16_bits(np.array([0.8125], dtype=np.float32))[0]
    v_saved = inp.v_pages.copy()
    inp.v_pages[...] = c
    out = _gpu(inp).float().cpu().numpy()
    assert np.abs(out - 0.8125).max() <= 0.8125 * 2.0 ** -8   # bf16 rounding of an fp32 value next to c
    inp.v_pages = v_saved
    # scores near +-80 before the max is taken off: keys on a coarse grid plus a large common vector
    rng = np.random.default_rng(3)
    kf = rng.integers(-16, 17, size=inp.k_pages.shape).astype(np.float32) / 8.0
    inp.k_pages = W.f32_to_bf16_bits(kf)
    base = _oracle(inp)
    inp.k_pages = W.f32_to_bf16_bits(kf + np.float32(4.0))
    out = _gpu(inp)
    assert_attention_close(out, base, "key shift", hardened=True, ref_abs=_oracle_abs(inp))


def test_needles_at_seams_and_masked_needle():
    cfg = W.CONFIGS[5].scaled(B=3, group_size=3, ctx=("uniform", 700, 1500))
    inp = W.make_attention_inputs(cfg, values="paper")
    P = cfg.page_size
    rng = np.random.default_rng(12)
    for b in range(cfg.B):
        n0 = int(inp.ctx_len[b]) - cfg.T
        for (t, h) in [(0, 0), (5, 9), (17, 31), (32, 16)]:
            kvh = h // cfg.G
            qv = W.bf16_bits_to_f32(inp.q[b, t, h])
            needle = W.f32_to_bf16_bits(qv / np.linalg.norm(qv) * 120.0)
            anc = [s for s in range(cfg.T) if (int(inp.tree_mask[b, t]) >> s) & 1]
            non = [s for s in range(cfg.T) if s not in anc]
            spots = [0, 15, 16, 255, 256, n0 - 1, n0 + anc[-1]]
            pos = spots[int(rng.integers(0, len(spots)))]
            pg, sl = inp.block_table[b, pos // P], pos % P
            inp.k_pages[pg, kvh, sl] = needle
            inp.v_pages[pg, kvh, sl] = W.f32_to_bf16_bits(rng.standard_normal(cfg.Dv).astype(np.float32) * 3)
            if non:     # a louder needle on a draft slot this query must not see
                pos = n0 + non[0]
                pg, sl = inp.block_table[b, pos // P], pos % P
                inp.k_pages[pg, kvh, sl] = W.f32_to_bf16_bits(qv / np.linalg.norm(qv) * 200.0)
                inp.v_pages[pg, kvh, sl] = W.f32_to_bf16_bits(np.full(cfg.Dv, 50.0, dtype=np.float32))
    ref = _oracle(inp)
    out = _gpu(inp)
    assert_attention_close(out, ref, "needles", ref_abs=_oracle_abs(inp))
    assert np.abs(ref).max() > 1.0


def test_nan_in_slots_past_the_end_is_never_read_into_the_result():
    cfg = W.CONFIGS[1].scaled(B=4, ctx=("uniform", 100, 400))
    inp = W.make_attention_inputs(cfg, values="peaked")
    ref = _oracle(inp)
    P = cfg.page_size
    nan = np.uint16(0x7FC0)
    for b in range(cfg.B):
        n = int(inp.ctx_len[b])
        if n % P:
            pg = inp.block_table[b, (n - 1) // P]
            inp.k_pages[pg, :, n % P:, :] = nan
            inp.v_pages[pg, :, n % P:, :] = nan
    ref_abs = _oracle_abs(W.make_attention_inputs(cfg, values="peaked"))
    out = _gpu(inp)
    assert_attention_close(out, ref, "nan tail", hardened=True, ref_abs=ref_abs)


def test_bad_ctx_len_is_flagged_not_faulted():
    from paper_2511_14617_amd import binding
    cfg = W.CONFIGS[1]
    inp = W.make_attention_inputs(cfg, values="peaked")
    ref = _oracle(inp)
    d = attention_device_inputs(inp)
    bad = inp.ctx_len.copy()
    bad[1] = cfg.T - 1
    bad[2] = inp.max_pages_per_seq * cfg.page_size + 1
    d["ctx_len"] = torch.from_numpy(bad).cuda()
    p = binding.attn_params(d["q"], d["k_pages"], d["v_pages"], d["block_table"], inp.scale)
    ws = torch.zeros(binding.seer_verify_attention_workspace(p), dtype=torch.uint8, device="cuda")
    out = binding.seer_verify_attention(d["q"], d["k_pages"], d["v_pages"], d["block_table"], d["ctx_len"], None,
                                        inp.scale, workspace=ws)
    torch.cuda.synchronize()
    assert binding.seer_verify_attention_status(ws) & 1
    got = out.float().cpu().numpy()
    assert (got[1] == 0).all() and (got[2] == 0).all()
    ref_abs = _oracle_abs(inp)
    assert_attention_close(out[0:1], ref[0:1], "valid request beside bad ones", hardened=True, ref_abs=ref_abs[0:1])
    assert_attention_close(out[3:4], ref[3:4], "valid request beside bad ones", hardened=True, ref_abs=ref_abs[3:4])


def test_stream_only_diagnostic_runs_the_load_path_and_writes_zeros():
    from paper_2511_14617_amd import binding
    cfg, kw = CASES["chain_T9_multi_split"]
    inp = W.make_attention_inputs(cfg, **kw)
    out = _gpu(inp, flags=binding.SEER_ATTN_STREAM_ONLY)
    assert float(out.float().abs().max()) == 0.0


@pytest.mark.parametrize("case", ["chain_T9_multi_split", "tree_T33", "mla_latent"])
def test_layers_of_one_step_share_the_plan(case):
    """A second call on the same workspace with other queries (the next layer of the model) and
    SEER_ATTN_REUSE_PLAN gives bit for bit what a call that plans again gives, and matches the oracle."""
    from paper_2511_14617_amd import binding
    cfg, kw = CASES[case]
    inp = W.make_attention_inputs(cfg, **kw)
    d = attention_device_inputs(inp)
    p = binding.attn_params(d["q"], d["k_pages"], d["v_pages"], d["block_table"], inp.scale, Dv=cfg.Dv)
    ws = torch.empty(binding.seer_verify_attention_workspace(p), dtype=torch.uint8, device="cuda")
    fixed = binding.SEER_ATTN_FIXED_SPLIT                    # the cut must not depend on measured speeds here
    q2 = torch.flip(d["q"], dims=[2]).contiguous()           # "another layer": the heads' queries swapped around

    def call(q, flags):
        return binding.seer_verify_attention(q, d["k_pages"], d["v_pages"], d["block_table"], d["ctx_len"], d["tree_mask"],
                                             inp.scale, Dv=cfg.Dv, workspace=ws, flags=flags).clone()
    call(d["q"], fixed)
    reused = call(q2, fixed | binding.SEER_ATTN_REUSE_PLAN)
    planned = call(q2, fixed)
    torch.cuda.synchronize()
    assert torch.equal(reused.view(torch.int16), planned.view(torch.int16))
    assert binding.seer_verify_attention_status(ws) == 0
    inp2 = W.make_attention_inputs(cfg, **kw)
    inp2.q[...] = inp.q[:, :, ::-1, :]
    assert_attention_close(reused, _oracle(inp2), case + " with a shared plan")


def _random_shape(rng):
    """A seeded random small workload: group width, slots, tree or chain, page size, context mix."""
    G = int(rng.choice([1, 2, 4, 5, 8, 16]))
    Hkv = int(rng.choice([1, 2, 4]))
    if rng.random() < 0.5:
        n_paths, path_len = int(rng.integers(1, 5)), int(rng.integers(1, 9))
        T, tree = 1 + n_paths * path_len, (n_paths, path_len)
    else:
        T, tree = int(rng.integers(1, 40)), None
    P = int(rng.choice([16, 16, 32, 64, 128]))
    B = int(rng.integers(1, 7))
    hi = int(rng.choice([T + 3, 100, 700, 2500]))
    lo = int(rng.integers(T, max(T + 1, hi // 2)))
    shared = int(rng.choice([0, 0, 32, 96])) if lo > 200 else 0
    cfg = W.CONFIGS[2].scaled(B=B, group_size=B, Hq=G * Hkv, Hkv=Hkv, T=T, tree=tree, page_size=P,
                              ctx=("uniform", lo, max(lo, hi)), shared_prefix=shared)
    return cfg


@pytest.mark.parametrize("seed", range(64))
def test_parity_random_shapes(seed):
    """Random shapes of the tiled D = 128 kernel against the oracle, hardened values: every combination of
    wave count, row blocks, page size, chain or tree, ragged tails and very short prefixes that the seeds hit."""
    rng = np.random.default_rng(1000 + seed)
    cfg = _random_shape(rng)
    inp = W.make_attention_inputs(cfg, seed=cfg.seed + seed, values="peaked",
                                  **({"dedup_fraction": 0.3} if cfg.tree else {}))
    ref = _oracle(inp)
    out = _gpu(inp)
    what = "random %d: G=%d Hkv=%d T=%d tree=%s P=%d B=%d ctx=%s" % (seed, cfg.G, cfg.Hkv, cfg.T, cfg.tree,
                                                                     cfg.page_size, cfg.B, inp.ctx_len.tolist())
    assert_attention_close(out, ref, what, hardened=True, ref_abs=_oracle_abs(inp))


@pytest.mark.parametrize("seed", range(32))
def test_parity_random_shapes_with_shared_prompts(seed):
    """Random shapes again, now with prompt groups of random size that share 0 .. 2100 leading tokens and with a random
    cap on the pieces per request (long pieces run the unrolled steady state through the shared run and out of it)."""
    rng = np.random.default_rng(5000 + seed)
    G, Hkv = int(rng.choice([1, 2, 4, 5, 8, 16])), int(rng.choice([1, 2, 4]))
    if rng.random() < 0.5:
        n_paths, path_len = int(rng.integers(1, 5)), int(rng.integers(1, 9))
        T, tree = 1 + n_paths * path_len, (n_paths, path_len)
    else:
        T, tree = int(rng.integers(1, 40)), None
    P, B = int(rng.choice([16, 16, 32, 64, 128])), int(rng.integers(2, 8))
    group = int(rng.integers(1, B + 1))
    hi = int(rng.choice([300, 700, 2500, 4000]))
    lo = int(rng.integers(max(T, hi // 4), max(T + 1, hi // 2)))
    shared = min(int(rng.choice([0, 16, 48, 200, 600, 1100, 2100])), max(lo - T - 1, 0))
    cfg = W.CONFIGS[2].scaled(B=B, group_size=group, Hq=G * Hkv, Hkv=Hkv, T=T, tree=tree, page_size=P,
                              ctx=("uniform", lo, max(lo, hi)), shared_prefix=shared)
    max_splits = int(rng.choice([0, 0, 2, 3]))
    inp = W.make_attention_inputs(cfg, seed=cfg.seed + seed, values="peaked",
                                  **({"dedup_fraction": 0.3} if cfg.tree else {}))
    what = "shared %d: G=%d Hkv=%d T=%d tree=%s P=%d B=%d group=%d shared=%d splits=%d" % (
        seed, G, Hkv, T, tree, P, B, group, shared, max_splits)
    assert_attention_close(_gpu(inp, max_splits=max_splits), _oracle(inp), what, hardened=True, ref_abs=_oracle_abs(inp))


@pytest.mark.parametrize("seed", range(24))
def test_parity_random_shapes_shared_latent(seed):
    """Random shapes of the shared-latent form (576/512, one KV head): head counts that fill one row block or
    several, chains and trees, pages of 32 .. 256 tokens, contexts from a single tile (less than one, even) to a few
    dozen, odd and even tile counts, ragged last tiles, draft slots that straddle tiles, several pieces per request."""
    rng = np.random.default_rng(9000 + seed)
    Hq = int(rng.choice([8, 16, 16, 32, 64, 128]))
    if rng.random() < 0.4:
        n_paths, path_len = int(rng.integers(1, 5)), int(rng.integers(1, 9))
        T, tree = 1 + n_paths * path_len, (n_paths, path_len)
    else:
        T, tree = int(rng.integers(1, 40 if Hq <= 32 else 12)), None
    P, B = int(rng.choice([32, 64, 64, 128, 256])), int(rng.integers(1, 6))
    hi = int(rng.choice([40, 100, 300, 900, 1500]))
    lo = int(rng.integers(T, max(T + 1, hi // 2)))
    cfg = W.CONFIGS[4].scaled(B=B, Hq=Hq, T=T, tree=tree, page_size=P, ctx=("uniform", lo, max(lo, hi)))
    max_splits = int(rng.choice([0, 0, 2, 3]))
    inp = W.make_attention_inputs(cfg, seed=cfg.seed + seed, values="peaked",
                                  **({"dedup_fraction": 0.3} if cfg.tree else {}))
    what = "latent %d: Hq=%d T=%d tree=%s P=%d B=%d ctx=%s splits=%d" % (seed, Hq, T, tree, P, B, inp.ctx_len.tolist(),
                                                                        max_splits)
    assert_attention_close(_gpu(inp, max_splits=max_splits), _oracle(inp), what, hardened=True, ref_abs=_oracle_abs(inp))


@pytest.mark.parametrize("case", ["chain_T9_multi_split", "tree_T33", "mla_latent", "rows528_G16_T33", "rows144_G16_T9"])
def test_page_permutation_is_bit_identical_with_the_fixed_split(case):
    """Moving every page to another place of the pool, the block table following, changes nothing: the cut
    of the KV stream is by logical position, so with SEER_ATTN_FIXED_SPLIT the output bits are the same."""
    from paper_2511_14617_amd import binding
    cfg, kw = CASES[case]
    inp = W.make_attention_inputs(cfg, values="peaked", **kw)
    a = _gpu(inp, flags=binding.SEER_ATTN_FIXED_SPLIT)
    perm = np.random.default_rng(7).permutation(inp.num_pages)      # old page -> new page
    k2 = np.empty_like(inp.k_pages)
    k2[perm] = inp.k_pages
    inp.k_pages = k2
    if inp.v_pages is not None:
        v2 = np.empty_like(inp.v_pages)
        v2[perm] = inp.v_pages
        inp.v_pages = v2
    inp.block_table = perm[inp.block_table].astype(np.int32)
    b = _gpu(inp, flags=binding.SEER_ATTN_FIXED_SPLIT)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert_attention_close(b, _oracle(inp), case + "/permuted pages", hardened=True, ref_abs=_oracle_abs(inp))


def test_gqa_equals_mha_on_replicated_kv():
    """Grouped-query heads against the same queries with every KV head stored G times (G = 1, Hkv = Hq):
    another launch shape, another cut of the stream, the same attention."""
    cfg, kw = CASES["chain_T9_multi_split"]
    inp = W.make_attention_inputs(cfg, values="peaked", **kw)
    ref, ref_abs = _oracle(inp), _oracle_abs(inp)
    gqa = _gpu(inp)
    inp.k_pages = np.repeat(inp.k_pages, cfg.G, axis=1)
    inp.v_pages = np.repeat(inp.v_pages, cfg.G, axis=1)
    mha = _gpu(inp)
    assert_attention_close(gqa, ref, "gqa", hardened=True, ref_abs=ref_abs)
    assert_attention_close(mha, ref, "mha on replicated kv", hardened=True, ref_abs=ref_abs)
    assert float((gqa.float() - mha.float()).abs().max()) <= 0.05


def test_shared_latent_equals_explicit_value_pool():
    """V = the first Dv components of the latent, once implicit (the tiled shared-latent kernel) and once as
    a value pool of its own (separate pools of these sizes take the general kernel)."""
    cfg, kw = CASES["mla_latent"]
    inp = W.make_attention_inputs(cfg, values="peaked", **kw)
    assert inp.v_pages is None
    ref = _oracle(inp)
    ref_abs = _oracle_abs(inp)
    shared = _gpu(inp)
    inp.v_pages = np.ascontiguousarray(inp.k_pages[..., : cfg.Dv])
    explicit = _gpu(inp)
    assert_attention_close(shared, ref, "shared latent", hardened=True, ref_abs=ref_abs)
    assert_attention_close(explicit, ref, "explicit value pool", hardened=True, ref_abs=ref_abs)
    assert float((shared.float() - explicit.float()).abs().max()) <= 0.05
