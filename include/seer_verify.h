/*
 * seer_verify -- batched draft verification for grouped speculative decoding on
 * AMD MI355X (gfx950).  C ABI: plain pointers and sizes, no C++ or framework
 * types.  Pointers marked "device" are HIP device memory owned by the caller;
 * the library neither frees nor keeps them.  Pointers marked "host" are read
 * during the call only.
 *
 * The method (paper: Section 2.2, draft-then-verify; Section 3.4, adaptive
 * grouped speculative decoding): every rollout request of a prompt group hands
 * in gamma draft tokens -- one chain, or several candidate paths sharing a root
 * (multi-path drafting, Section 3.4.2) -- and the target model scores all of
 * them in ONE forward pass.  A step emits the accepted draft prefix plus one
 * bonus token, at most gamma + 1 tokens (Section 3.4.1, expected tokens per
 * forward (1 - alpha^(gamma+1)) / (1 - alpha)), and must equal what serial
 * decoding would have produced (Section 3.1, lossless).
 *
 * Two calls make up the data-parallel part of that pass:
 *   seer_verify_attention : attention of the T = gamma + 1 verify positions of
 *                           every request over its paged KV cache (once per layer)
 *   seer_accept           : target token per position from the logits, then the
 *                           longest accepted root path (once per step)
 *
 * Common rules
 *  - Calls are asynchronous on `hip_stream` (a hipStream_t passed as void*,
 *    NULL = the default stream): no device synchronisation, no allocation, no
 *    state inside the library (seer_verify_attention keeps a few hundred bytes
 *    of call-to-call history in the caller's workspace, see
 *    SEER_ATTN_FIXED_SPLIT).  Scratch memory is sized by the *_workspace() functions
 *    (host-only, no HIP call) and supplied by the caller; calls that share a
 *    workspace must be ordered on one stream.
 *  - Return value: 0 = launched; negative = SEER_E* argument error found on the
 *    host BEFORE anything is launched (so they can be exercised without a GPU);
 *    positive = the hipError_t of a failed launch.
 *  - Content of device arrays cannot be checked on the host.  The kernels keep
 *    every access in bounds regardless: page ids are clamped into the pool, and
 *    a request whose ctx_len is below T or beyond max_pages_per_seq*page_size
 *    gets an all-zero output row block and raises bit 0 of the status word (see
 *    seer_verify_attention_status_offset).
 */
#ifndef SEER_VERIFY_H
#define SEER_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The library is built with hidden visibility; these are its only exported symbols. */
#define SEER_API __attribute__((visibility("default")))

#define SEER_OK 0
#define SEER_EINVAL (-1)       /* null pointer, negative or zero size               */
#define SEER_ESHAPE (-2)       /* T not in 1..64, Hq not a multiple of Hkv, ...     */
#define SEER_EUNSUPPORTED (-3) /* head dims / page size no kernel is built for      */
#define SEER_EWORKSPACE (-4)   /* workspace NULL or smaller than *_workspace()      */
#define SEER_EALIGN (-5)       /* a tensor pointer is not 16-byte aligned           */
#define SEER_ELIMIT (-6)       /* problem larger than a fixed-size entry point holds */

#define SEER_MAX_T 64          /* verify slots per request (width of the mask word) */

/* Shape of one verify-attention call.
 * Notation: B requests; T = gamma + 1 verify slots per request (slot 0 = the
 * last accepted token = tree root, slots 1..gamma = draft tokens); Hq query
 * heads, Hkv KV heads, G = Hq / Hkv heads share one KV head. */
typedef struct seer_attn_params {
    int32_t B, T, Hq, Hkv;
    int32_t Dqk;               /* key / query head dim                                */
    int32_t Dv;                /* value / output head dim                             */
    int32_t page_size;         /* tokens per KV page                                  */
    int32_t num_pages;         /* pages in the pool                                   */
    int32_t max_pages_per_seq; /* row stride of block_table                           */
    int32_t max_splits;        /* cap on split-K partitions per request, 1..256; 0 = library default */
    int32_t kv_shared_latent;  /* 0: separate K and V pools; 1: V = first Dv components of K (MLA, absorbed form) */
    int32_t flags;             /* SEER_ATTN_* bits, normally 0                        */
    float scale;               /* softmax scale applied to q.k: positive and finite   */
} seer_attn_params;

/* flags: run the general kernel even where a tiled one exists (for cross-checks). */
#define SEER_ATTN_GENERAL_KERNEL 1
/* flags: cut the KV stream into equal stretches.  By default the library sizes each workgroup's
 * stretch by that workgroup slot's measured speed in earlier calls ON THE SAME WORKSPACE (a few
 * hundred bytes of history kept in it; any contents are valid, unusable ones mean equal stretches).
 * The result is the same up to the rounding order of the partial sums; with this flag the cut, and
 * therefore the result, does not depend on earlier calls. */
#define SEER_ATTN_FIXED_SPLIT 2
/* (bit 4 is a measurement aid, see seer_verify_diag.h) */
/* flags: use the plan that the previous call on this workspace computed instead of planning again.  How the
 * KV stream is cut depends on the shape parameters and on ctx_len only, and a model calls this function
 * once per layer with the same ctx_len: the first layer plans, the others pass this flag (saves a ~10 us
 * kernel per call).  The caller guarantees that the previous call on this workspace had the same
 * parameters (flags apart) and that ctx_len and block_table are unchanged; if not, the output is
 * undefined (every access still stays in bounds).  The status word then accumulates over the calls. */
#define SEER_ATTN_REUSE_PLAN 8

/* Supported shapes: (Dqk, Dv) in {(64,64), (128,128), (256,256), (192,128),
 * (576,512)} with any page_size >= 1.  Tiled matrix-core kernels exist for
 * Dqk = Dv = 128 with separate K and V pools and a power-of-two page_size of
 * 16..1024 (any G*T: more than 256 query rows per KV head are cut into row
 * blocks), and for the shared latent Dqk = 576, Dv = 512 with a power-of-two
 * page_size of 32..1024; every other combination runs a slower general kernel.
 *
 * Shared prompt pages (Section 2.3: the responses of a group are sampled for the same prompt): where a request's
 * block_table row starts with the same page ids as the row before or after it, the D = 128 kernel reads
 * those tiles with the cache policy that keeps them for the other requests and streams everything else,
 * so only the first reader of a group pays DRAM for the shared pages.  Put the requests of a group in
 * adjacent rows to benefit; results do not depend on it. */

/* Bytes of device scratch seer_verify_attention needs for these params; 0 on
 * invalid params.  Host-only arithmetic. */
SEER_API size_t seer_verify_attention_workspace(const seer_attn_params* p);

/* Byte offset, inside the workspace, of a uint32 status word that the call
 * zeroes and its kernels OR into: bit 0 = some request had ctx_len < T or
 * beyond the block table; bit 1 = some page id was outside the pool. */
SEER_API size_t seer_verify_attention_status_offset(void);

/*
 * Multi-token paged-KV attention for the verify pass.
 *
 * For request b with n = ctx_len[b] and n0 = n - T: logical KV position j lives
 * in page block_table[b][j / page_size], slot j % page_size.  The K/V of the T
 * verify slots are already in the cache as the LAST T logical positions, slot s
 * at n0 + s.  Query slot t sees every position j < n0 and position n0 + s iff
 * bit s of tree_mask[b][t] is set; tree_mask == NULL means s <= t (a causal
 * chain).  out[b,t,h,:] = softmax_j(scale * q[b,t,h,:].K[j,h/G,:]) . V[j,h/G,:]
 * over the visible j, accumulated in fp32 and rounded to bf16 (nearest even).
 * A query that sees nothing gets zeros.
 *
 *  out         device [B,T,Hq,Dv]  bf16, written
 *  q           device [B,T,Hq,Dqk] bf16
 *  k_pages     device [num_pages,Hkv,page_size,Dqk] bf16
 *  v_pages     device [num_pages,Hkv,page_size,Dv]  bf16; must be NULL iff kv_shared_latent
 *  block_table device [B,max_pages_per_seq] int32; entries past ceil(n/page_size) are not read
 *  ctx_len     device [B] int32, INCLUDING the T verify slots
 *  tree_mask   device [B,T] uint64 ancestor-or-self bits, or NULL
 *  p           host
 *  workspace   device, >= seer_verify_attention_workspace(p) bytes, 256-byte aligned
 */
SEER_API int seer_verify_attention(void* out, const void* q, const void* k_pages, const void* v_pages,
                          const int32_t* block_table, const int32_t* ctx_len,
                          const uint64_t* tree_mask, const seer_attn_params* p, void* workspace,
                          size_t workspace_bytes, void* hip_stream);

/* Name of the partition kernel (the kernel that streams the KV pages) a call with these params launches,
 * e.g. "attn_gqa128_kernel<2,1>" (waves per workgroup, tiles in flight); NULL on invalid params.
 * Static text, host-only. */
SEER_API const char* seer_verify_attention_kernel(const seer_attn_params* p);

/* Bytes of device scratch seer_accept needs; 0 on invalid sizes.  Host-only. */
SEER_API size_t seer_accept_workspace(int32_t B, int32_t T, int32_t V);

/*
 * Acceptance from target logits.
 *
 * target_argmax[b,t] = lowest index attaining max_v logits[b,t,v] (fp32
 * comparison, +0 == -0, inputs NaN-free; -inf allowed).  Node t >= 1 is accepted
 * iff its parent is accepted and draft_tokens[b,t] == target_argmax[b,parent];
 * the root is accepted.  The winner is the deepest accepted node (lowest slot
 * among equally deep ones -- sibling nodes may carry the same token, so this is
 * a search over paths, not a greedy first-match walk).
 *
 *  logits        device [B,T,V] fp32
 *  draft_tokens  device [B,T] int32; slot 0 (the root's own token) is ignored
 *  tree_parent   device [B,T] int32 or NULL (= chain, parent[t] = t-1).
 *                [b,0] is ignored (root); 0 <= parent[t] < t; -2 = padded slot,
 *                never accepted.  Any other value is treated as padded.
 *  accepted_len  device [B] int32, written: number of accepted DRAFT tokens, 0..T-1
 *  accepted_path device [B,T] int32, written: slots root..winner, then -1
 *  bonus_token   device [B] int32 or NULL, written: target_argmax at the winner
 *  target_argmax device [B,T] int32, written
 *  workspace     device, >= seer_accept_workspace(B,T,V) bytes, 16-byte aligned
 */
SEER_API int seer_accept(const float* logits, const int32_t* draft_tokens, const int32_t* tree_parent,
                int32_t B, int32_t T, int32_t V, int32_t* accepted_len, int32_t* accepted_path,
                int32_t* bonus_token, int32_t* target_argmax, void* workspace,
                size_t workspace_bytes, void* hip_stream);

/*
 * seer_accept for callers that cannot allocate or hand over scratch memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * seer_accept without the workspace: the per-chunk results of the vocabulary scan go to a fixed
 * array of SEER_ACCEPT_STATIC_MAX_PAIRS * 8 bytes (1 MiB) that is part of the library's device
 * image (every GPU the library runs on holds it until the process ends).  The call allocates
 * nothing and frees nothing.
 *
 *  - Limit: B * T * ceil(V / 16384) <= SEER_ACCEPT_STATIC_MAX_PAIRS, else SEER_ELIMIT (checked on
 *    the host before anything else; the multi-path configuration, 4224 rows of 152 064 logits,
 *    needs 42 240 pairs).
 *  - The first call on a device looks up that device's copy of the array (one
 *    hipGetSymbolAddress, no allocation); a call with B = 0 does only that, so a caller can make
 *    it before starting a graph capture.  The device of hip_stream must be the current device.
 *  - All calls on one GPU share the array: calls that may overlap on one GPU (different streams,
 *    different threads) race on it and must be ordered by the caller.  Nothing in it has to be
 *    cleared between calls: every entry a call reads, it has written first.
 */
#define SEER_ACCEPT_STATIC_MAX_PAIRS 131072
SEER_API int seer_accept_static(const float* logits, const int32_t* draft_tokens, const int32_t* tree_parent,
                                int32_t B, int32_t T, int32_t V, int32_t* accepted_len, int32_t* accepted_path,
                                int32_t* bonus_token, int32_t* target_argmax, void* hip_stream);

/*
 * Acceptance under sampling (Section 4.1 of the paper: its workloads sample at
 * temperature 1.0 and 0.8; Section 3.4: its drafts are token sequences, not
 * distributions).  As seer_accept, except that the target token of a slot is a
 * DRAW from softmax(logits[b,t,:] / temperature) instead of the argmax, by the
 * Gumbel-max rule: token = lowest index attaining max_v fma(logits[v],
 * 1/temperature, G(seed, b*T+t, v)) in fp32.  G is a pure function of its
 * arguments (Philox4x32-10 with counter (v/4, row, 0, 0) and key = seed;
 * u = ((word >> 9) + 0.5) * 2^-23; G = -ln(-ln u) through a fixed fp32
 * polynomial log2), so a call is reproducible bit for bit, and accepting a
 * draft token iff it equals the draw at its parent is lossless.
 *
 *  temperature  > 0, finite            seed  any 64-bit value; use a new one per step
 *  target_token device [B,T] int32, written: the drawn token of each slot
 * Everything else, the workspace size included, as for seer_accept.
 */
SEER_API int seer_accept_sampled(const float* logits, const int32_t* draft_tokens, const int32_t* tree_parent,
                        int32_t B, int32_t T, int32_t V, float temperature, uint64_t seed,
                        int32_t* accepted_len, int32_t* accepted_path, int32_t* bonus_token,
                        int32_t* target_token, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Commit of the accepted path: the step right after verification (Section 3.4:
 * of several candidate paths one root path is accepted; Section 3.1: the
 * sequence continues exactly as serial decoding would have).  For every request
 * the key/value rows of accepted_path[b][1..a], a = accepted_len[b], which sit
 * at logical positions n0 + path[i] (n0 = ctx_len[b] - T), are moved to
 * positions n0+1 .. n0+a, and ctx_len[b] becomes n0 + 1 + a (root + accepted
 * draft tokens; the bonus token has no key/value yet, it is the next step's
 * root).  Rows past the new length keep stale contents.  For a chain nothing
 * moves.  Optionally the tokens the step emits are written: the a accepted
 * draft tokens in path order, then the bonus token.
 *
 *  p              shapes as for seer_verify_attention (B, T, Hkv, Dqk, Dv, page_size,
 *                 num_pages, max_pages_per_seq, kv_shared_latent are used); Dqk and Dv
 *                 multiples of 8; (T-1) * (Dqk + Dv) / 8 <= 4608
 *  k_pages, v_pages  device, modified in place; v_pages NULL iff kv_shared_latent
 *  block_table    device [B,max_pages_per_seq] int32
 *  ctx_len        device [B] int32, read and overwritten
 *  accepted_len, accepted_path  device, as written by seer_accept
 *  draft_tokens, bonus_token    device; needed only if emitted_tokens is given
 *  emitted_tokens device [B,T] int32 or NULL, written: a + 1 tokens, then -1
 *  n_emitted      device [B] int32 (NULL iff emitted_tokens is NULL), written: a + 1
 *  status         device [1] int32 or NULL; bits are OR-ed in: 1 = a ctx_len out of
 *                 range, 2 = a page id outside the pool, 4 = accepted_len / accepted_path
 *                 malformed (path[0] != 0, not ascending, >= T).  Such requests are
 *                 left untouched.  The caller clears it.
 * Returns SEER_OK or a negative SEER_E* / positive hipError_t; asynchronous on
 * hip_stream.  Requests must not share the pages that hold their T verify slots.
 */
SEER_API int seer_kv_commit(const seer_attn_params* p, void* k_pages, void* v_pages, const int32_t* block_table,
                   int32_t* ctx_len, const int32_t* accepted_len, const int32_t* accepted_path,
                   const int32_t* draft_tokens, const int32_t* bonus_token, int32_t* emitted_tokens,
                   int32_t* n_emitted, int32_t* status, void* hip_stream);

/*
 * Draft lengths for the next steps (Algorithm 1 of the paper, Marginal-Benefit-Aware adaptive
 * speculation, with the throughput model of Section 3.4.1).  Host arithmetic only, no GPU work.
 *
 *  B_h, B_l    requests of the high- and the low-priority class in the batch (B_h >= 1, B_l >= 0)
 *  beta        host [n_beta] acceptance probability of draft position 1, 2, ... (each in [0, 1]);
 *              n_beta >= gamma_max + 1; position 0, the token already accepted, counts as 1
 *  gamma_max   cap on draft tokens per request, 0 .. 63
 *  lambda      priority factor >= 1 (the paper suggests 2)
 *  step_time   host [gamma_max + 1], > 0: measured time of one draft + verify step of the whole batch
 *              with gamma = 0 .. gamma_max draft tokens per request (gamma = 0: a plain decode step)
 *  gamma_h, gamma_l   written: draft tokens per request of each class
 *  gamma_star  written if not NULL: argmin over gamma of (1 - alpha) step_time[gamma] /
 *              (1 - alpha^(gamma + 1)), alpha = mean of beta[0 .. gamma_max - 1]; ties -> smaller gamma
 * Returns SEER_OK or SEER_EINVAL / SEER_ESHAPE.
 */
SEER_API int seer_mba_draft_lengths(int32_t B_h, int32_t B_l, const double* beta, int32_t n_beta, int32_t gamma_max,
                           double lambda, const double* step_time, int32_t* gamma_h, int32_t* gamma_l,
                           int32_t* gamma_star);

/*
 * Online acceptance statistics: what Algorithm 1 calls the per-position acceptance probabilities
 * beta[1], beta[2], ... and Section 3.4.2 says are collected online.  Called after seer_accept (or
 * seer_accept_sampled) of a step, it ADDS that step to three counters per draft position k = depth of
 * a node under the root (k = 0 is the root):
 *   offered[k]   the request's draft tree has a node of depth k
 *   tried[k]     the accepted path reached depth k - 1 and its node there has a child, i.e. a draft
 *                token of depth k was compared with the target's token
 *   accepted[k]  accepted_len >= k
 * A request whose accepted_len / accepted_path do not describe a root path of its tree is left out.
 *
 *  accepted_len, accepted_path  device, as written by seer_accept
 *  tree_parent   device [B,T] int32 or NULL (= chain), as for seer_accept
 *  counts        device [3][T] uint64 (offered, tried, accepted), 8-byte aligned; read-modify-write:
 *                the caller zeroes it where a statistics window starts
 * Asynchronous on hip_stream; no workspace.  Returns SEER_OK or SEER_EINVAL / SEER_ESHAPE / SEER_EALIGN
 * or a positive hipError_t.
 */
SEER_API int seer_acceptance_stats(const int32_t* accepted_len, const int32_t* accepted_path, const int32_t* tree_parent,
                          int32_t B, int32_t T, uint64_t* counts, void* hip_stream);

/*
 * beta[k - 1], k = 1 .. T - 1, from a HOST copy of those counts: accepted[k] / offered[k] (of the steps
 * that drafted k or more tokens, the share in which the k-th was accepted: the sequence Algorithm 1
 * differences, 1 at k = 0 and non-increasing for drafts of one depth), or, with conditional != 0,
 * accepted[k] / tried[k] (how often a token that was compared was accepted: the per-token rate behind
 * the expected-tokens law of Section 3.4.1).  Positions nothing was counted for get `prior` (in [0, 1]).
 * Host arithmetic only.  Returns SEER_OK or SEER_EINVAL / SEER_ESHAPE.
 */
SEER_API int seer_acceptance_beta(const uint64_t* counts, int32_t T, int32_t conditional, double prior, double* beta);

/*
 * Grouped n-gram drafting: the step right before verification (Section 2.3, pattern level: the
 * token histories of all requests of a prompt group serve as n-gram reference; Section 3.4.2 and
 * Appendix A.2, draft client call batch_speculate with SpeculationArgs max_spec_tokens,
 * pattern_lookup_max, pattern_lookup_min, top_k: confidence scores from the suffix statistics,
 * low-probability candidates dropped, several paths by beam search).  It writes exactly the
 * draft_tokens / tree_parent / tree_mask that seer_verify_attention and seer_accept read.
 *
 * Token histories live in one caller-owned pool: sequence q holds tokens[seq_start[q] ..
 * seq_start[q] + seq_len[q]); group g owns sequences group_first[g] .. group_first[g+1]-1.  The
 * caller appends new tokens in place and raises seq_len (nothing is indexed, so there is nothing
 * else to update).  No n-gram runs from one sequence into another.
 *
 * For request b, with its newest tokens as pattern (pattern[b] is right-aligned: the newest token
 * is pattern[b][pattern_lookup_max - 1], the first pattern_lookup_max - pattern_len[b] entries are
 * not read):
 *   match  = the longest pattern suffix, of max(pattern_lookup_min, 1) .. min(pattern_len[b],
 *            pattern_lookup_max) tokens, that occurs in a sequence of the group FOLLOWED by at
 *            least one more token of that sequence; none -> root-only draft, match_len 0.
 *   count  of a path c_1..c_d = number of places where match c_1..c_d occurs; n_root = number of
 *            places where the match occurs with a continuation.  Confidence = count / n_root.
 *   beam   level d (1 .. min(max_spec_tokens[b], gamma_max)) = the first top_k, ordered by (count
 *            descending, rank of the parent in level d-1 ascending, token ascending), of the
 *            one-token extensions of level d-1 with count >= 1, token in [0, vocab) and
 *            (float)count >= min_confidence * (float)n_root (fp32); stops at an empty level.
 *   slots  T = 1 + top_k * gamma_max <= 64.  Slot 0 = root (token = newest pattern token, parent
 *            -1).  Rank j of level d -> slot 1 + (d-1)*top_k + j, parent = its parent's slot.
 *            Every member of every level is a draft node.  Unused slots: token -1, parent -2,
 *            count 0, mask = own bit.  tree_mask[t] = own bit | tree_mask[parent].
 * The result is unique (integer counts, total order), whatever order the places are found in.
 *
 * Limits: top_k <= 16, pattern_lookup_max <= 32, vocab <= 2^24, at most 128 sequences per group,
 * sequences shorter than 2^20 tokens, pool_tokens <= 2^31 - 2^16, tokens 16-byte aligned.  A request whose group id, sequence
 * table or sequence ranges are out of range gets a root-only draft and raises bit 0 of *status; one
 * whose group holds more than max_group_tokens tokens raises bit 1 (the caller clears status).
 */
typedef struct seer_draft_params {
    int32_t B;                  /* requests                                                   */
    int32_t n_groups, n_seq;    /* entries of group_first minus one; of seq_start / seq_len   */
    int64_t pool_tokens;        /* entries of tokens                                          */
    int32_t max_group_tokens;   /* bound on the sum of seq_len over one group (sizes the workspace) */
    int32_t gamma_max, top_k;
    int32_t pattern_lookup_min, pattern_lookup_max;
    int32_t vocab;
    float min_confidence;       /* 0 .. 1                                                     */
} seer_draft_params;

/* Bytes of device scratch seer_draft needs (two place lists of max_group_tokens entries per
 * request); 0 on invalid params.  Host-only. */
SEER_API size_t seer_draft_workspace(const seer_draft_params* p);

/*
 *  tokens, seq_start, seq_len, group_first   device int32, as above
 *  req_group        device [B] int32
 *  pattern          device [B, pattern_lookup_max] int32;  pattern_len device [B] int32
 *  max_spec_tokens  device [B] int32 (the per-request draft length, e.g. from seer_mba_draft_lengths)
 *  draft_tokens, tree_parent  device [B,T] int32, written;  tree_mask device [B,T] uint64, written
 *  node_count       device [B,T] int32 or NULL, written: count of each node, slot 0 = n_root
 *  match_len        device [B] int32 or NULL, written
 *  status           device [1] int32 or NULL, bits OR-ed in
 *  workspace        device, >= seer_draft_workspace(p) bytes, 16-byte aligned
 * Asynchronous on hip_stream; returns SEER_OK, a negative SEER_E* or a positive hipError_t.
 */
SEER_API int seer_draft(const int32_t* tokens, const int32_t* seq_start, const int32_t* seq_len,
               const int32_t* group_first, const int32_t* req_group, const int32_t* pattern,
               const int32_t* pattern_len, const int32_t* max_spec_tokens, const seer_draft_params* p,
               int32_t* draft_tokens, int32_t* tree_parent, uint64_t* tree_mask, int32_t* node_count,
               int32_t* match_len, int32_t* status, void* workspace, size_t workspace_bytes,
               void* hip_stream);

/*
 * Appending what a step emitted to the token histories that seer_draft reads: the counterpart of
 * the draft server's update call (Appendix A.2: the new tokens of a request go to that request's
 * own sequence of its group), here one store per token because nothing is indexed.
 *
 * For request b with q = req_seq[b] and n = n_emitted[b] (as written by seer_kv_commit): the tokens
 * emitted_tokens[b][0 .. n) are written behind the seq_len[q] tokens of sequence q, seq_len[q]
 * grows by n, and (if pattern is given) pattern[b] / pattern_len[b] are refreshed to the newest
 * min(pattern_lookup_max, seq_len[q]) tokens of the sequence, right-aligned as seer_draft reads them
 * (unused leading entries -1).
 *
 *  tokens         device [pool_tokens] int32, written behind the sequences' current ends
 *  seq_start      device [n_seq] int32;  seq_len device [n_seq] int32, read and written
 *  seq_capacity   device [n_seq] int32: room of each sequence in the pool (>= seq_len)
 *  req_seq        device [B] int32: the sequence that holds request b's own tokens; two requests
 *                 of one call must not name the same sequence
 *  emitted_tokens device [B,T] int32;  n_emitted device [B] int32, 0 .. T
 *  pattern        device [B, pattern_lookup_max] int32 or NULL;  pattern_len device [B] int32,
 *                 NULL iff pattern is NULL
 *  status         device [1] int32 or NULL; bits OR-ed in: 1 = req_seq or the sequence's range out
 *                 of range (request skipped), 2 = no room for n more tokens or n out of range
 *                 (nothing appended, pattern still refreshed).  The caller clears it.
 * Asynchronous on hip_stream; returns SEER_OK, a negative SEER_E* or a positive hipError_t.
 */
SEER_API int seer_history_append(int32_t* tokens, const int32_t* seq_start, int32_t* seq_len,
                        const int32_t* seq_capacity, const int32_t* req_seq,
                        const int32_t* emitted_tokens, const int32_t* n_emitted, int32_t B, int32_t T,
                        int32_t n_seq, int64_t pool_tokens, int32_t pattern_lookup_max, int32_t* pattern,
                        int32_t* pattern_len, int32_t* status, void* hip_stream);

/* Static text for a return code of either call (negative SEER_E*, or a
 * positive hipError_t). */
SEER_API const char* seer_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SEER_VERIFY_H */
