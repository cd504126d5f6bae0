/*
 * seer_verify_diag -- measurement aids of libseer_verify.so.  Not part of the product surface
 * (seer_verify.h): nothing here changes what a call computes; a benchmark uses them to time the
 * dominant kernel without a profiler and to find the memory system's ceiling for the same access
 * pattern.
 */
#ifndef SEER_VERIFY_DIAG_H
#define SEER_VERIFY_DIAG_H

#include "seer_verify.h"

#ifdef __cplusplus
extern "C" {
#endif

/* flags: measurement aid.  The tiled D = 128 kernel runs its whole load path (plan, page lookups,
 * loads into LDS, waits, partial-result writes) without the arithmetic; out is written as zeros.
 * The time of such a call is the gather-read ceiling of the memory system for this workload and
 * launch shape.  Ignored by the other kernels. */
#define SEER_ATTN_STREAM_ONLY 4

/*
 * Measurement aid: the same call, which also records two caller-created
 * hipEvent_t (passed as void*) on the stream immediately before and after the
 * partition kernel -- the kernel that streams the KV pages and dominates the
 * call -- so that its duration can be read with hipEventElapsedTime without a
 * profiler.  The plan kernel runs before event_begin, the combine after
 * event_end.  Results are identical to seer_verify_attention.
 */
SEER_API int seer_verify_attention_timed(void* out, const void* q, const void* k_pages, const void* v_pages,
                                const int32_t* block_table, const int32_t* ctx_len,
                                const uint64_t* tree_mask, const seer_attn_params* p, void* workspace,
                                size_t workspace_bytes, void* hip_stream, void* event_begin,
                                void* event_end);

/*
 * Where in the workspace the plan of a call with these params leaves, per request, the number of leading
 * 32-token tiles whose pages the request before or after it in the batch maps too (int32[B]; host-only
 * arithmetic, 0 on invalid params).  The partition kernel of the D = 128 shapes reads those tiles with the
 * cache policy that keeps them for the other requests of the prompt group; nothing that a call computes
 * depends on it.  Tests read it back to check what the plan found.
 */
SEER_API size_t seer_verify_attention_shared_tiles_offset(const seer_attn_params* p);

#ifdef __cplusplus
}
#endif
#endif /* SEER_VERIFY_DIAG_H */
