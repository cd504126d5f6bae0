"""CPU fp64 oracle for batched draft verification.  TEST INFRASTRUCTURE ONLY:
imported by tests/, the smoke check and the benchmark's cpu_baseline leg, never
by the product path."""
from .seer_oracle import (  # noqa: F401
    accept,
    argmax,
    argmax_sampled,
    build,
    emitted_tokens,
    gumbel,
    gumbel_of_words,
    kv_commit,
    log2_det,
    num_threads,
    philox4x32_10,
    verify_accept,
    verify_attention,
    verify_attention_rows,
)
