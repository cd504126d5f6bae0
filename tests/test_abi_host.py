"""Host-side checks that need no GPU: the shared library loads, exports every symbol the header
declares, sizes workspaces, and turns bad arguments into SEER_E* codes before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2511_14617_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build_library()
    return binding.load_library()


def _params(**kw):
    from paper_2511_14617_amd.binding import SeerAttnParams
    base = dict(B=4, T=5, Hq=8, Hkv=2, Dqk=128, Dv=128, page_size=16, num_pages=100, max_pages_per_seq=32,
                max_splits=0, kv_shared_latent=0, flags=0, scale=0.088)
    base.update(kw)
    return SeerAttnParams(**base)


def test_every_declared_symbol_is_exported(lib):
    declared = set()
    for name in ("seer_verify.h", "seer_verify_diag.h"):
        header = open(os.path.join(ROOT, "include", name)).read()
        body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        declared |= set(re.findall(r"\b(seer_[a-z_]+)\s*\(", body))
    from paper_2511_14617_amd import binding
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_nothing_but_the_declared_symbols_is_exported(lib):
    """The library is built with hidden visibility: its dynamic symbol table defines the C entry points of
    the header and nothing else (no C++ internals, no kernel stubs)."""
    import subprocess
    from paper_2511_14617_amd import binding
    out = subprocess.run(["nm", "-D", "--defined-only", binding.LIB_PATH], check=True, stdout=subprocess.PIPE,
                         text=True).stdout
    defined = {line.split()[-1] for line in out.splitlines() if line.strip()}
    # what the toolchain itself adds to every shared object
    defined -= {"_init", "_fini", "__bss_start", "_edata", "_end", "__hip_fatbin", "__hip_gpubin_handle"}
    defined = {d for d in defined if not d.startswith("__hip_")}
    assert defined == set(binding.EXPORTS), sorted(defined ^ set(binding.EXPORTS))


def test_params_struct_matches_header():
    from paper_2511_14617_amd.binding import SeerAttnParams
    header = open(os.path.join(ROOT, "include", "seer_verify.h")).read()
    struct = re.search(r"typedef struct seer_attn_params \{(.*?)\} seer_attn_params;", header, flags=re.S).group(1)
    struct = re.sub(r"/\*.*?\*/", "", struct, flags=re.S)
    names = []
    for decl in struct.split(";"):
        decl = decl.strip()
        if decl:
            names += [n.strip() for n in decl.split(None, 1)[1].split(",")]
    assert names == [f[0] for f in SeerAttnParams._fields_]
    assert ctypes.sizeof(SeerAttnParams) == 4 * len(names)


def test_workspace_sizes(lib):
    from paper_2511_14617_amd import binding
    p = _params()
    n = binding.seer_verify_attention_workspace(p)
    assert n > 0 and n % 256 == 0
    assert binding.seer_verify_attention_workspace(_params(T=65)) == 0
    assert binding.seer_verify_attention_workspace(_params(Dqk=100)) == 0
    bigger = binding.seer_verify_attention_workspace(_params(B=64, Hq=32, Hkv=8, T=9))
    assert bigger > n
    assert binding.seer_accept_workspace(4, 5, 1024) == 4 * 5 * 1 * 8
    assert binding.seer_accept_workspace(4, 5, 8193) == 4 * 5 * 2 * 8
    assert binding.seer_accept_workspace(4, 65, 10) == 0


def test_attention_argument_errors_before_any_launch(lib):
    from paper_2511_14617_amd import binding as b
    call = lib.seer_verify_attention
    fake = 0x1000   # never dereferenced: all of these fail on the host

    def run(p, out=fake, q=fake, k=fake, v=fake, bt=fake, cl=fake, mask=None, ws=0x10000, ws_bytes=1 << 40):
        return call(out, q, k, v, bt, cl, mask, ctypes.byref(p) if p is not None else None, ws, ws_bytes, None)

    assert call(fake, fake, fake, fake, fake, fake, None, None, fake, 0, None) == b.SEER_EINVAL
    assert run(_params(T=0)) == b.SEER_ESHAPE
    assert run(_params(T=65)) == b.SEER_ESHAPE
    assert run(_params(Hq=7)) == b.SEER_ESHAPE
    assert run(_params(max_splits=257)) == b.SEER_ESHAPE
    assert run(_params(Dqk=100)) == b.SEER_EUNSUPPORTED
    assert run(_params(Dqk=576, Dv=512, kv_shared_latent=1), v=None, ws_bytes=0) == b.SEER_EWORKSPACE
    assert run(_params(num_pages=0)) == b.SEER_EINVAL
    assert run(_params(flags=16)) == b.SEER_EINVAL                       # unknown flag bit
    assert run(_params(scale=float("nan"))) == b.SEER_EINVAL
    assert run(_params(scale=0.0)) == b.SEER_EINVAL
    assert run(_params(scale=-0.1)) == b.SEER_EINVAL
    assert run(_params(scale=float("inf"))) == b.SEER_EINVAL
    assert run(_params(), q=None) == b.SEER_EINVAL
    assert run(_params(), v=None) == b.SEER_EINVAL                     # separate pools need v_pages
    assert run(_params(kv_shared_latent=1)) == b.SEER_EINVAL           # shared latent forbids v_pages
    assert run(_params(), ws=None) == b.SEER_EWORKSPACE
    assert run(_params(), ws_bytes=1024) == b.SEER_EWORKSPACE
    assert run(_params(), q=fake + 2) == b.SEER_EALIGN
    assert run(_params(), ws=0x10010) == b.SEER_EALIGN
    assert run(_params(B=0)) == b.SEER_OK                              # empty batch: nothing to do
    for code in (0, -1, -2, -3, -4, -5, -6, 1, -99):
        assert isinstance(b.seer_strerror(code), str) and b.seer_strerror(code)


def test_accept_argument_errors_before_any_launch(lib):
    from paper_2511_14617_amd import binding as b
    call = lib.seer_accept
    fake = 0x1000

    def run(B=4, T=5, V=1000, logits=fake, draft=fake, parent=None, alen=fake, path=fake, bonus=None, tgt=fake,
            ws=0x10000, ws_bytes=1 << 30):
        return call(logits, draft, parent, B, T, V, alen, path, bonus, tgt, ws, ws_bytes, None)

    assert run(T=0) == b.SEER_ESHAPE
    assert run(T=65) == b.SEER_ESHAPE
    assert run(V=0) == b.SEER_EINVAL
    assert run(B=-1) == b.SEER_EINVAL
    assert run(logits=None) == b.SEER_EINVAL
    assert run(tgt=None) == b.SEER_EINVAL
    assert run(ws=None) == b.SEER_EWORKSPACE
    assert run(ws_bytes=8) == b.SEER_EWORKSPACE
    assert run(ws=0x10004) == b.SEER_EALIGN
    assert run(logits=fake + 2) == b.SEER_EALIGN
    assert run(B=0) == b.SEER_OK


def test_sampled_accept_and_commit_argument_errors_before_any_launch(lib):
    from paper_2511_14617_amd import binding as b
    fake = 0x1000

    def sampled(tau=1.0, **kw):
        a = dict(B=4, T=5, V=1000, ws=0x10000, ws_bytes=1 << 30)
        a.update(kw)
        return lib.seer_accept_sampled(fake, fake, None, a["B"], a["T"], a["V"], tau, 7, fake, fake, None, fake,
                                       a["ws"], a["ws_bytes"], None)

    assert sampled(tau=0.0) == b.SEER_EINVAL
    assert sampled(tau=-1.0) == b.SEER_EINVAL
    assert sampled(tau=float("nan")) == b.SEER_EINVAL
    assert sampled(tau=float("inf")) == b.SEER_EINVAL
    assert sampled(T=65) == b.SEER_ESHAPE
    assert sampled(ws=None) == b.SEER_EWORKSPACE
    assert sampled(B=0) == b.SEER_OK

    def commit(p, k=fake, v=fake, table=fake, n=fake, alen=fake, path=fake, draft=None, bonus=None, em=None,
               nem=None):
        return lib.seer_kv_commit(ctypes.byref(p), k, v, table, n, alen, path, draft, bonus, em, nem, None, None)

    assert lib.seer_kv_commit(None, fake, fake, fake, fake, fake, fake, None, None, None, None, None, None) == b.SEER_EINVAL
    assert commit(_params(T=65)) == b.SEER_ESHAPE
    assert commit(_params(Dqk=100)) == b.SEER_ESHAPE                    # rows move in 16-byte chunks
    assert commit(_params(num_pages=0)) == b.SEER_EINVAL
    assert commit(_params(), v=None) == b.SEER_EINVAL
    assert commit(_params(), path=None) == b.SEER_EINVAL
    assert commit(_params(), em=fake) == b.SEER_EINVAL                   # emitted tokens need drafts, bonus and a count
    assert commit(_params(), k=fake + 2) == b.SEER_EALIGN
    assert commit(_params(T=64, Dqk=576, Dv=512)) == b.SEER_EUNSUPPORTED  # more than a workgroup holds in registers
    assert commit(_params(B=0)) == b.SEER_OK


def _draft_params(**kw):
    from paper_2511_14617_amd.binding import SeerDraftParams
    base = dict(B=4, n_groups=1, n_seq=4, pool_tokens=5000, max_group_tokens=4000, gamma_max=8, top_k=4,
                pattern_lookup_min=2, pattern_lookup_max=8, vocab=152064, min_confidence=0.0)
    base.update(kw)
    return SeerDraftParams(**base)


def test_draft_params_struct_matches_header():
    from paper_2511_14617_amd.binding import SeerDraftParams
    header = open(os.path.join(ROOT, "include", "seer_verify.h")).read()
    struct = re.search(r"typedef struct seer_draft_params \{(.*?)\} seer_draft_params;", header, flags=re.S).group(1)
    struct = re.sub(r"/\*.*?\*/", "", struct, flags=re.S)
    fields = []
    for decl in struct.split(";"):
        decl = decl.strip()
        if decl:
            ctype, names = decl.split(None, 1)
            fields += [(n.strip(), ctype) for n in names.split(",")]
    want = {"int32_t": ctypes.c_int32, "int64_t": ctypes.c_int64, "float": ctypes.c_float}
    assert [(n, want[t]) for n, t in fields] == list(SeerDraftParams._fields_)


def test_draft_argument_errors_before_any_launch(lib):
    from paper_2511_14617_amd import binding as b
    fake = 0x1000

    def run(p, tokens=fake, out=fake, ws=0x10000, ws_bytes=1 << 40):
        return lib.seer_draft(tokens, fake, fake, fake, fake, fake, fake, fake, ctypes.byref(p), out, fake, fake,
                              None, None, None, ws, ws_bytes, None)

    assert lib.seer_draft(*([fake] * 8), None, fake, fake, fake, None, None, None, fake, 1 << 40, None) == b.SEER_EINVAL
    assert run(_draft_params(top_k=0)) == b.SEER_EINVAL
    assert run(_draft_params(gamma_max=0)) == b.SEER_EINVAL
    assert run(_draft_params(vocab=0)) == b.SEER_EINVAL
    assert run(_draft_params(min_confidence=float("nan"))) == b.SEER_EINVAL
    assert run(_draft_params(min_confidence=1.5)) == b.SEER_EINVAL
    assert run(_draft_params(max_group_tokens=0)) == b.SEER_EINVAL
    assert run(_draft_params(top_k=8, gamma_max=8)) == b.SEER_ESHAPE          # 65 slots
    assert run(_draft_params(pattern_lookup_min=9)) == b.SEER_ESHAPE
    assert run(_draft_params(top_k=17, gamma_max=2)) == b.SEER_EUNSUPPORTED
    assert run(_draft_params(pattern_lookup_max=33)) == b.SEER_EUNSUPPORTED
    assert run(_draft_params(vocab=(1 << 24) + 1)) == b.SEER_EUNSUPPORTED
    assert run(_draft_params(pool_tokens=1 << 31)) == b.SEER_EUNSUPPORTED
    assert run(_draft_params(), tokens=None) == b.SEER_EINVAL
    assert run(_draft_params(), out=None) == b.SEER_EINVAL
    assert run(_draft_params(), ws=None) == b.SEER_EWORKSPACE
    assert run(_draft_params(), ws_bytes=1024) == b.SEER_EWORKSPACE
    assert run(_draft_params(), ws=0x10004) == b.SEER_EALIGN
    assert run(_draft_params(), tokens=fake + 4) == b.SEER_EALIGN
    assert run(_draft_params(B=0)) == b.SEER_OK
    small = b.seer_draft_workspace(_draft_params())
    assert small > 0 and small % 256 == 0
    assert b.seer_draft_workspace(_draft_params(max_group_tokens=800000, B=8)) >= 2 * 8 * 800000 * 4
    assert b.seer_draft_workspace(_draft_params(top_k=17)) == 0


def test_history_append_argument_errors_before_any_launch(lib):
    from paper_2511_14617_amd import binding as b
    fake = 0x1000

    def run(B=4, T=9, n_seq=8, pool=5000, p_max=8, tokens=fake, pattern=fake, plen=fake):
        return lib.seer_history_append(tokens, fake, fake, fake, fake, fake, fake, B, T, n_seq, pool, p_max, pattern, plen,
                                       None, None)

    assert run(B=-1) == b.SEER_EINVAL
    assert run(n_seq=0) == b.SEER_EINVAL
    assert run(pool=0) == b.SEER_EINVAL
    assert run(T=0) == b.SEER_ESHAPE
    assert run(T=65) == b.SEER_ESHAPE
    assert run(p_max=0) == b.SEER_EINVAL
    assert run(p_max=33) == b.SEER_EUNSUPPORTED
    assert run(pool=1 << 31) == b.SEER_EUNSUPPORTED
    assert run(tokens=None) == b.SEER_EINVAL
    assert run(pattern=None) == b.SEER_EINVAL                     # pattern and pattern_len come together
    assert run(B=0) == b.SEER_OK


def test_product_path_fails_loudly_without_the_library(tmp_path, monkeypatch):
    from paper_2511_14617_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libseer_verify.so"))
    with pytest.raises(ImportError):
        binding.load_library()


def test_kernel_name_follows_the_dispatch(lib):
    from paper_2511_14617_amd import binding
    name = binding.seer_verify_attention_kernel
    assert name(_params(B=64, Hq=32, Hkv=8, T=9)) == "attn_gqa128_kernel<2,1>"          # 36 rows: two waves
    assert name(_params(B=8, Hq=32, Hkv=8, T=17)) == "attn_gqa128_kernel<3,3>"          # 68 rows
    assert name(_params(B=128, Hq=32, Hkv=8, T=33)) == "attn_gqa128_kernel<4,2,helpers=4>"   # 132 rows: 128 + 4
    assert name(_params(B=8, Hq=20, Hkv=4, T=30)) == "attn_gqa128_kernel<5,3>"          # 150 rows
    assert name(_params(Hq=128, Hkv=1, Dqk=576, Dv=512, page_size=64, kv_shared_latent=1)) == "attn_mla_kernel"
    assert name(_params(Hq=128, Hkv=1, Dqk=576, Dv=512, page_size=16, kv_shared_latent=1)) == "attn_general_kernel<576,512>"
    assert name(_params(flags=binding.SEER_ATTN_GENERAL_KERNEL)) == "attn_general_kernel<128,128>"
    assert name(_params(page_size=24)) == "attn_general_kernel<128,128>"
    assert name(_params(T=65)) is None
