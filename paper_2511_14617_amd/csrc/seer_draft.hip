// seer_draft: grouped n-gram drafting, the step right before verification.
//
// What is computed (Section 2.3, pattern level; Section 3.4.2; Appendix A.2, draft client, call
// batch_speculate with SpeculationArgs max_spec_tokens / pattern_lookup_max / pattern_lookup_min /
// top_k): a request's draft tokens come from the token histories of all requests of its prompt
// group.  The request's newest tokens are the pattern; the longest pattern suffix that occurs in a
// history followed by at least one more token is the match; every continuation string of the
// match is a candidate path whose confidence is (places where match + path occurs) / (places
// where the match occurs with a continuation), i.e. the product of the conditional frequencies
// along the path; candidates below min_confidence are dropped and a beam search of width top_k
// returns several paths.  The paper keeps the histories in a compressed suffix tree that a
// separate server updates; here nothing is indexed: the histories are plain token arrays in HBM
// (appending a token is one store), and a lookup scans the group's history, which at 8 TB/s and
// with the group's tokens resident in L2 after the first request costs less than the tree's
// upkeep would.  Two kernels:
//
//   draft_match_kernel   grid (parts, B): each workgroup scans one stretch of the group's
//                        tokens, measures at every place how many pattern tokens end there,
//                        and keeps the places that reach its running maximum
//   draft_expand_kernel  grid (B): takes the longest match over all parts, gathers its places,
//                        then level by level counts the next tokens of every beam member's
//                        places in an LDS hash table, picks the top_k and splits the places
//
// Counts are integers, the order of the beam is (count descending, parent rank ascending, token
// ascending) and the confidence test is one fp32 product and one comparison, so the result is
// unique and does not depend on the order in which places are found.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/seer_verify.h"

namespace seer {
namespace draft {

constexpr int kThreads = 256;
constexpr int kMaxGroupSeqs = 128;        // sequences per group (7 bits of a place)
constexpr int kMaxSeqLenLog2 = 20;        // tokens per sequence < 2^20 (20 bits of a place)
constexpr int kMaxPattern = 32;           // pattern_lookup_max (5 bits of a place hold match length - 1)
constexpr int kMaxTopK = 16;
constexpr int kTableSlots = 4096;         // LDS hash table: 4096 x (key, count) = 32 KB
constexpr uint32_t kEmpty = 0xffffffffu;
constexpr int kTokensPerPart = 8192;      // target stretch of one match workgroup
constexpr int kMaxParts = 64;

// A place = (sequence inside the group, offset of the token that follows the occurrence); while the
// match is still being searched it also carries the match length.
__device__ __forceinline__ uint32_t pack_place(int seq, int m, int off) {
    return (static_cast<uint32_t>(seq) << 25) | (static_cast<uint32_t>(m - 1) << 20) | static_cast<uint32_t>(off);
}
__device__ __forceinline__ int place_seq(uint32_t e) { return static_cast<int>(e >> 25); }
__device__ __forceinline__ int place_len(uint32_t e) { return static_cast<int>((e >> 20) & 31u) + 1; }
__device__ __forceinline__ int place_off(uint32_t e) { return static_cast<int>(e & ((1u << kMaxSeqLenLog2) - 1)); }

struct Args {
    const int32_t* tokens;
    const int32_t* seq_start;
    const int32_t* seq_len;
    const int32_t* group_first;
    const int32_t* req_group;
    const int32_t* pattern;
    const int32_t* pattern_len;
    const int32_t* max_spec_tokens;
    int32_t* draft_tokens;
    int32_t* tree_parent;
    uint64_t* tree_mask;
    int32_t* node_count;        // may be nullptr
    int32_t* match_len;         // may be nullptr
    int32_t* status;            // may be nullptr
    int2* part_hdr;             // [B, parts] (places kept, longest match) of each match workgroup
    uint32_t* list_a;           // [B, cap]
    uint32_t* list_b;           // [B, cap]
    int64_t pool_tokens;
    int n_groups, n_seq, max_group_tokens;
    int gamma_max, top_k, p_min, p_max, vocab;
    int parts, chunk, cap;      // cap = parts * chunk >= max_group_tokens
    float min_confidence;
};

// The group's sequence table in LDS.  Returns 0 if usable, else the status bits to raise.
struct GroupTable {
    int start[kMaxGroupSeqs];
    int len[kMaxGroupSeqs];
    int flat[kMaxGroupSeqs + 1];          // tokens of the group before sequence j
    int n_seq;
    int bad;
};

__device__ __forceinline__ void load_group(const Args& a, int b, GroupTable& gt) {
    const int tid = threadIdx.x;
    if (tid == 0) {
        gt.bad = 0;
        gt.n_seq = 0;
    }
    __syncthreads();
    const int g = a.req_group[b];
    int q0 = 0, q1 = 0;
    if (g < 0 || g >= a.n_groups) {
        if (tid == 0) gt.bad = 1;
    } else {
        q0 = a.group_first[g];
        q1 = a.group_first[g + 1];
        if (q0 < 0 || q1 < q0 || q1 > a.n_seq || q1 - q0 > kMaxGroupSeqs) {
            if (tid == 0) gt.bad = 1;
            q1 = q0 = 0;
        }
    }
    const int n = q1 - q0;
    if (tid < n) {
        const int st = a.seq_start[q0 + tid], ln = a.seq_len[q0 + tid];
        if (st < 0 || ln < 0 || ln >= (1 << kMaxSeqLenLog2) || static_cast<int64_t>(st) + ln > a.pool_tokens) {
            atomicOr(&gt.bad, 1);
            gt.start[tid] = 0, gt.len[tid] = 0;
        } else {
            gt.start[tid] = st, gt.len[tid] = ln;
        }
    }
    __syncthreads();
    if (tid == 0) {
        int64_t acc = 0;
        for (int j = 0; j < n; ++j) {
            gt.flat[j] = static_cast<int>(acc);
            acc += gt.len[j];
            if (acc > a.max_group_tokens) {
                gt.bad |= 2;
                acc = 0;
            }
        }
        gt.flat[n] = static_cast<int>(acc);
        gt.n_seq = gt.bad ? 0 : n;
    }
    __syncthreads();
}

// ------------------------------------------------------------------------------------------------
// Match: how many pattern tokens end at each place of one stretch of the group's tokens.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void draft_match_kernel(Args a) {
    __shared__ GroupTable gt;
    __shared__ int s_pat[kMaxPattern];
    __shared__ int s_best, s_kept;
    const int b = blockIdx.y, part = blockIdx.x, tid = threadIdx.x;
    load_group(a, b, gt);
    const int plen = min(max(a.pattern_len[b], 0), a.p_max);
    const int need = max(a.p_min, 1);
    if (tid < a.p_max) s_pat[tid] = a.pattern[static_cast<size_t>(b) * a.p_max + tid];
    if (tid == 0) s_best = need, s_kept = 0;
    __syncthreads();
    uint32_t* out = a.list_a + static_cast<size_t>(b) * a.cap + static_cast<size_t>(part) * a.chunk;
    if (gt.n_seq > 0 && plen >= need) {
        const int newest = s_pat[a.p_max - 1];
        const int lo = part * a.chunk, hi = min(lo + a.chunk, gt.flat[gt.n_seq]);
        for (int j = 0; j < gt.n_seq; ++j) {
            // places i of sequence j inside [lo, hi) whose next token exists
            const int i0 = max(lo - gt.flat[j], 0), i1 = min(hi - gt.flat[j], gt.len[j] - 1);
            if (i0 >= i1) continue;
            const int32_t* seq = a.tokens + gt.start[j];
            for (int base = i0; base < i1; base += 4 * kThreads) {
                int tok[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = base + u * kThreads + tid;
                    tok[u] = i < i1 ? seq[i] : ~newest;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (tok[u] != newest) continue;
                    const int i = base + u * kThreads + tid;
                    const int limit = min(plen, i + 1);
                    int m = 1;
                    while (m < limit && seq[i - m] == s_pat[a.p_max - 1 - m]) ++m;
                    if (m >= s_best) {             // a shorter match than one already seen can never win
                        atomicMax(&s_best, m);
                        out[atomicAdd(&s_kept, 1)] = pack_place(j, m, i + 1);
                    }
                }
            }
        }
    }
    __syncthreads();
    if (tid == 0) a.part_hdr[static_cast<size_t>(b) * a.parts + part] = make_int2(s_kept, s_kept > 0 ? s_best : 0);
}

// ------------------------------------------------------------------------------------------------
// Expand: beam search over the continuations of the longest match.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const uint64_t w = __shfl_xor(v, o, 64);
        v = w > v ? w : v;
    }
    return v;
}

struct Member {            // one beam member of the current level
    int base, n, slot;     // its places are list[base .. base + n)
};

__global__ __launch_bounds__(kThreads) void draft_expand_kernel(Args a) {
    __shared__ GroupTable gt;
    __shared__ uint32_t s_key[kTableSlots];
    __shared__ uint32_t s_cnt[kTableSlots];
    __shared__ Member s_mem[kMaxTopK], s_next[kMaxTopK];
    __shared__ uint64_t s_red[kThreads / 64];
    __shared__ uint64_t s_pick[kMaxTopK];          // chosen children: count << 32 | ~key
    __shared__ int s_fill[kMaxTopK];
    __shared__ int s_tok[SEER_MAX_T], s_par[SEER_MAX_T], s_num[SEER_MAX_T];
    __shared__ uint64_t s_msk[SEER_MAX_T];
    __shared__ int s_n, s_best, s_nmem, s_overflow;

    const int b = blockIdx.x, tid = threadIdx.x;
    const int T = 1 + a.top_k * a.gamma_max;
    load_group(a, b, gt);
    const int plen = min(max(a.pattern_len[b], 0), a.p_max);
    if (tid < T) {
        s_tok[tid] = tid == 0 && plen > 0 ? a.pattern[static_cast<size_t>(b) * a.p_max + a.p_max - 1] : -1;
        s_par[tid] = tid == 0 ? -1 : -2;
        s_num[tid] = 0;
        s_msk[tid] = 1ull << tid;
    }
    if (tid == 0) s_n = 0, s_best = 0;
    __syncthreads();
    if (gt.bad && tid == 0 && a.status) atomicOr(a.status, gt.bad);

    // longest match over the parts, then its places
    const int2* hdr = a.part_hdr + static_cast<size_t>(b) * a.parts;
    if (gt.n_seq > 0)
        for (int p = tid; p < a.parts; p += kThreads)
            if (hdr[p].x > 0) atomicMax(&s_best, hdr[p].y);
    __syncthreads();
    const int p_star = s_best;
    uint32_t* cur = a.list_b + static_cast<size_t>(b) * a.cap;
    uint32_t* nxt = a.list_a + static_cast<size_t>(b) * a.cap;
    if (p_star > 0) {
        for (int p = 0; p < a.parts; ++p) {
            const int kept = hdr[p].x;
            if (kept == 0 || hdr[p].y < p_star) continue;
            const uint32_t* src = nxt + static_cast<size_t>(p) * a.chunk;
            for (int e = tid; e < kept; e += kThreads) {
                const uint32_t pl = src[e];
                if (place_len(pl) == p_star) cur[atomicAdd(&s_n, 1)] = pl;
            }
        }
    }
    __syncthreads();
    const int n_root = s_n;
    const int levels = p_star > 0 ? min(max(a.max_spec_tokens[b], 0), a.gamma_max) : 0;
    const float threshold = a.min_confidence * static_cast<float>(n_root);
    if (tid == 0) {
        s_num[0] = n_root;
        s_mem[0] = Member{0, n_root, 0};
        s_nmem = 1;
    }
    __syncthreads();

    for (int d = 1; d <= levels; ++d) {
        const int nmem = s_nmem;
        const int n_level = s_mem[nmem - 1].base + s_mem[nmem - 1].n;
        // the token a place shows at this level, with the rank of the member that owns the place
        auto key_of = [&](int e, uint32_t pl) -> uint32_t {
            int r = 0;
            while (r + 1 < nmem && e >= s_mem[r + 1].base) ++r;
            const int j = place_seq(pl), off = place_off(pl) + d - 1;
            if (off >= gt.len[j]) return kEmpty;
            const int x = a.tokens[gt.start[j] + off];
            if (x < 0 || x >= a.vocab) return kEmpty;
            return (static_cast<uint32_t>(r) << 24) | static_cast<uint32_t>(x);
        };
        int n_pick = 0;
        // Pass 0 counts in a hash table.  Only if more distinct (member, token) pairs turn up than the
        // table has slots do further passes count token ranges in a directly indexed table.
        int table = 64;
        while (table < kTableSlots && table < 2 * n_level) table <<= 1;
        const int range = kTableSlots / nmem;                     // tokens per member in a ranged pass
        const int n_pass_ranged = (a.vocab + range - 1) / range;
        for (int pass = 0; pass <= n_pass_ranged; ++pass) {
            const bool hashed = pass == 0;
            const int slots = hashed ? table : kTableSlots;
            for (int s = tid; s < slots; s += kThreads) s_key[s] = kEmpty, s_cnt[s] = 0;
            if (tid == 0) s_overflow = 0;
            __syncthreads();
            const int shift = 32 - __builtin_ctz(static_cast<unsigned>(table));
            const int lo_tok = (pass - 1) * range;
            for (int e = tid; e < n_level; e += kThreads) {
                const uint32_t key = key_of(e, cur[e]);
                if (key == kEmpty) continue;
                if (hashed) {
                    uint32_t h = (key * 2654435761u) >> shift;
                    int probes = 0;
                    for (; probes < table; ++probes) {
                        const uint32_t old = atomicCAS(&s_key[h], kEmpty, key);
                        if (old == kEmpty || old == key) {
                            atomicAdd(&s_cnt[h], 1u);
                            break;
                        }
                        h = (h + 1) & (table - 1);
                    }
                    if (probes == table) s_overflow = 1;
                } else {
                    const int x = static_cast<int>(key & 0xffffffu) - lo_tok;
                    if (x >= 0 && x < range) {
                        const int s = static_cast<int>(key >> 24) * range + x;
                        s_key[s] = key;
                        atomicAdd(&s_cnt[s], 1u);
                    }
                }
            }
            __syncthreads();
            const bool overflow = s_overflow != 0;
            if (!(hashed && overflow)) {
                // the top_k of this table join the picks so far; the best top_k of both stay
                for (int round = 0; round < a.top_k; ++round) {
                    uint64_t best = 0;
                    for (int s = tid; s < slots; s += kThreads) {
                        const uint32_t c = s_cnt[s];
                        if (c == 0 || static_cast<float>(c) < threshold) continue;
                        const uint64_t v = (static_cast<uint64_t>(c) << 32) | static_cast<uint32_t>(~s_key[s]);
                        best = v > best ? v : best;
                    }
                    best = wave_max_u64(best);
                    if ((tid & 63) == 0) s_red[tid >> 6] = best;
                    __syncthreads();
                    uint64_t win = s_red[0];
#pragma unroll
                    for (int w = 1; w < kThreads / 64; ++w) win = s_red[w] > win ? s_red[w] : win;
                    __syncthreads();
                    if (win == 0) break;
                    const uint32_t win_key = ~static_cast<uint32_t>(win);
                    for (int s = tid; s < slots; s += kThreads)
                        if (s_key[s] == win_key) s_cnt[s] = 0;
                    if (tid == 0) {
                        // insertion into the sorted picks (descending), at most top_k kept
                        int at = n_pick < a.top_k ? n_pick : a.top_k - 1;
                        if (n_pick < a.top_k || win > s_pick[at]) {
                            while (at > 0 && s_pick[at - 1] < win) {
                                s_pick[at] = s_pick[at - 1];
                                --at;
                            }
                            s_pick[at] = win;
                        }
                    }
                    n_pick = min(n_pick + 1, a.top_k);
                    __syncthreads();
                }
            }
            if (hashed && !overflow) break;
        }
        if (n_pick == 0) break;
        // the picks become draft nodes and the members of the next level
        if (tid == 0) {
            int base = 0;
            for (int j = 0; j < n_pick; ++j) {
                const uint32_t key = ~static_cast<uint32_t>(s_pick[j]);
                const int c = static_cast<int>(s_pick[j] >> 32), r = static_cast<int>(key >> 24);
                const int slot = 1 + (d - 1) * a.top_k + j, parent = s_mem[r].slot;
                s_tok[slot] = static_cast<int>(key & 0xffffffu);
                s_par[slot] = parent;
                s_num[slot] = c;
                s_msk[slot] = (1ull << slot) | s_msk[parent];
                s_next[j] = Member{base, c, slot};       // s_mem is still read by the split below
                s_fill[j] = 0;
                base += c;
            }
        }
        __syncthreads();
        if (d < levels) {
            for (int e = tid; e < n_level; e += kThreads) {
                const uint32_t pl = cur[e];
                const uint32_t key = key_of(e, pl);
                if (key == kEmpty) continue;
                for (int j = 0; j < n_pick; ++j)
                    if (~static_cast<uint32_t>(s_pick[j]) == key) {
                        nxt[s_next[j].base + atomicAdd(&s_fill[j], 1)] = pl;
                        break;
                    }
            }
        }
        __syncthreads();
        if (tid < n_pick) s_mem[tid] = s_next[tid];
        if (tid == 0) s_nmem = n_pick;
        uint32_t* t = cur;
        cur = nxt;
        nxt = t;
        __syncthreads();
    }

    if (tid < T) {
        const size_t o = static_cast<size_t>(b) * T + tid;
        a.draft_tokens[o] = s_tok[tid];
        a.tree_parent[o] = s_par[tid];
        a.tree_mask[o] = s_msk[tid];
        if (a.node_count) a.node_count[o] = s_num[tid];
    }
    if (tid == 0 && a.match_len) a.match_len[b] = p_star;
}

}  // namespace draft
}  // namespace seer

namespace {

struct DraftShape {
    int parts, chunk, cap;
    size_t off_hdr, off_a, off_b, total;
};

int draft_shape(const seer_draft_params* p, DraftShape* s) {
    using namespace seer::draft;
    if (!p || p->B < 0 || p->n_groups < 1 || p->n_seq < 1 || p->pool_tokens < 1 || p->max_group_tokens < 1) return SEER_EINVAL;
    if (p->gamma_max < 1 || p->top_k < 1 || p->pattern_lookup_max < 1 || p->pattern_lookup_min < 0 || p->vocab < 1)
        return SEER_EINVAL;
    if (!(p->min_confidence >= 0.0f) || !(p->min_confidence <= 1.0f)) return SEER_EINVAL;
    if (p->pattern_lookup_min > p->pattern_lookup_max) return SEER_ESHAPE;
    if (1 + static_cast<int64_t>(p->top_k) * p->gamma_max > SEER_MAX_T) return SEER_ESHAPE;
    if (p->top_k > kMaxTopK || p->pattern_lookup_max > kMaxPattern || p->vocab > (1 << 24) ||
        p->pool_tokens > 0x7fffffffll)
        return SEER_EUNSUPPORTED;
    int parts = (p->max_group_tokens + kTokensPerPart - 1) / kTokensPerPart;
    parts = parts < 1 ? 1 : (parts > kMaxParts ? kMaxParts : parts);
    int chunk = (p->max_group_tokens + parts - 1) / parts;
    chunk = (chunk + 3) & ~3;
    s->parts = parts, s->chunk = chunk, s->cap = parts * chunk;
    auto up = [](size_t v) { return (v + 255) & ~static_cast<size_t>(255); };
    const size_t B = static_cast<size_t>(p->B > 0 ? p->B : 1);
    s->off_hdr = 0;
    s->off_a = up(B * parts * sizeof(int2));
    s->off_b = s->off_a + up(B * s->cap * sizeof(uint32_t));
    s->total = s->off_b + up(B * s->cap * sizeof(uint32_t));
    return SEER_OK;
}

}  // namespace

extern "C" size_t seer_draft_workspace(const seer_draft_params* p) {
    DraftShape s;
    return draft_shape(p, &s) == SEER_OK ? s.total : 0;
}

extern "C" int seer_draft(const int32_t* tokens, const int32_t* seq_start, const int32_t* seq_len,
                          const int32_t* group_first, const int32_t* req_group, const int32_t* pattern,
                          const int32_t* pattern_len, const int32_t* max_spec_tokens, const seer_draft_params* p,
                          int32_t* draft_tokens, int32_t* tree_parent, uint64_t* tree_mask, int32_t* node_count,
                          int32_t* match_len, int32_t* status, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
    DraftShape s;
    const int shape_rc = draft_shape(p, &s);
    if (shape_rc != SEER_OK) return shape_rc;
    if (p->B == 0) return SEER_OK;
    if (!tokens || !seq_start || !seq_len || !group_first || !req_group || !pattern || !pattern_len || !max_spec_tokens ||
        !draft_tokens || !tree_parent || !tree_mask)
        return SEER_EINVAL;
    if (!workspace || workspace_bytes < s.total) return SEER_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) % 16 != 0) return SEER_EALIGN;
    seer::draft::Args a{};
    a.tokens = tokens, a.seq_start = seq_start, a.seq_len = seq_len, a.group_first = group_first;
    a.req_group = req_group, a.pattern = pattern, a.pattern_len = pattern_len, a.max_spec_tokens = max_spec_tokens;
    a.draft_tokens = draft_tokens, a.tree_parent = tree_parent, a.tree_mask = tree_mask;
    a.node_count = node_count, a.match_len = match_len, a.status = status;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    a.part_hdr = reinterpret_cast<int2*>(ws + s.off_hdr);
    a.list_a = reinterpret_cast<uint32_t*>(ws + s.off_a);
    a.list_b = reinterpret_cast<uint32_t*>(ws + s.off_b);
    a.pool_tokens = p->pool_tokens;
    a.n_groups = p->n_groups, a.n_seq = p->n_seq, a.max_group_tokens = p->max_group_tokens;
    a.gamma_max = p->gamma_max, a.top_k = p->top_k, a.p_min = p->pattern_lookup_min, a.p_max = p->pattern_lookup_max;
    a.vocab = p->vocab, a.parts = s.parts, a.chunk = s.chunk, a.cap = s.cap, a.min_confidence = p->min_confidence;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipLaunchKernelGGL(seer::draft::draft_match_kernel, dim3(s.parts, p->B), dim3(seer::draft::kThreads), 0, stream, a);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return static_cast<int>(err);
    hipLaunchKernelGGL(seer::draft::draft_expand_kernel, dim3(p->B), dim3(seer::draft::kThreads), 0, stream, a);
    err = hipGetLastError();
    return err == hipSuccess ? SEER_OK : static_cast<int>(err);
}
