"""MI355X-native batched draft verification (the verify step of grouped
speculative decoding): `seer_verify_attention` and `seer_accept` (plus `seer_accept_sampled`,
`seer_kv_commit` and `seer_draft`, the calls around them), hand-written
HIP for gfx950 behind a C ABI (include/seer_verify.h).

The binding is imported lazily so that the input generators in `workloads` can
be used on machines without PyTorch-ROCm or the built library."""


def __getattr__(name):
    if name in ("seer_verify_attention", "seer_accept", "seer_verify_attention_workspace",
                "seer_accept_workspace", "seer_verify_attention_status", "seer_strerror", "load_library",
                "seer_accept_sampled", "seer_kv_commit", "seer_mba_draft_lengths", "seer_draft", "seer_draft_workspace", "seer_history_append",
                "SeerDraftParams",
                "SeerAttnParams", "SeerError", "attn_params"):
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
