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
//   draft_match_kernel   grid (stretches, groups): a workgroup reads one stretch of a group's tokens
//                        once and, for every request of the group, measures at every place how many
//                        of the request's newest tokens end there; the places that reach the
//                        stretch's running maximum go to the request's place list
//   draft_expand_kernel  grid (requests): takes the longest match over all stretches, gathers its
//                        places, then searches level by level: the (member, next token) pairs of
//                        the live places are counted, the top_k picked, the places reassigned.
//                        Few places live in registers (one wave alone, or the whole workgroup),
//                        many in two lists in global memory.
//
// Counts are integers, the order of the beam is (count descending, parent rank ascending, token
// ascending) and the confidence test is one fp32 product and one comparison, so the result is
// unique and does not depend on the order in which places are found or atomics land.
//
// Both kernels are bound by the length of their dependent chains (a global round trip, an LDS round
// trip, a barrier), not by bandwidth: loads are requested in batches from addresses clamped into
// the pool and selected afterwards, so that a thread waits once per batch, not once per load.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/seer_verify.h"

namespace seer {
namespace draft {

constexpr int kMatchThreads = 256;        // match workgroup
constexpr int kThreads = 1024;            // expansion workgroup
constexpr int kMaxGroupSeqs = 128;        // sequences per group (7 bits of a place)
constexpr int kMaxSeqLenLog2 = 20;        // tokens per sequence < 2^20 (20 bits of a place)
constexpr int kMaxPattern = 32;           // pattern_lookup_max (5 bits of a place hold match length - 1)
constexpr int kMaxTopK = 16;
constexpr int kTableSlots = 4096;         // LDS hash table: 4096 x (key, count) = 32 KB
constexpr uint32_t kEmpty = 0xffffffffu;
constexpr int kMaxParts = 256;            // stretches a group's tokens are cut into, at most
constexpr int kReqWindow = 64;            // request ids a match workgroup looks at per round
constexpr int kQuads = 4;                 // 16-byte loads a match thread has in flight
constexpr int kTile = 4 * kQuads * kMatchThreads;   // tokens a match workgroup takes per round
constexpr int kTokensPerPart = kTile;     // target length of a stretch: one round
constexpr int kSmall = 2048;              // up to this many places the expansion holds in registers
constexpr int kAhead = 8;                 // levels whose tokens it fetches at a time
constexpr int kRankAll = 32;              // up to this many candidates of a level are ranked against each other
constexpr int kSolo = 256;                // at most this many live places: one wave finishes the search alone

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

__device__ __forceinline__ int lane_id() { return static_cast<int>(threadIdx.x) & 63; }

// Index for each lane whose `hit` is set, from a counter in LDS: one atomic per wave instead of one per lane.
__device__ __forceinline__ int wave_append(int* counter, bool hit) {
    const uint64_t mask = __ballot(hit);
    if (mask == 0) return 0;
    const int leader = __ffsll(static_cast<long long>(mask)) - 1;
    int base = 0;
    if (lane_id() == leader) base = atomicAdd(counter, __popcll(mask));
    base = __builtin_amdgcn_readlane(base, leader);
    return base + __popcll(mask & ((1ull << lane_id()) - 1));
}

// The group's sequence table in LDS; n_seq = 0 and bad != 0 if it cannot be used.
struct GroupTable {
    int start[kMaxGroupSeqs];
    int len[kMaxGroupSeqs];
    int flat[kMaxGroupSeqs + 1];          // tokens of the group before sequence j
    int n_seq;
    int bad;
};

__device__ __forceinline__ void load_group(const Args& a, int g, GroupTable& gt) {
    const int tid = threadIdx.x;
    if (tid == 0) {
        gt.bad = 0;
        gt.n_seq = 0;
    }
    __syncthreads();
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
    if (tid <= n) {                               // tokens of the group before sequence tid (lengths are below 2^20)
        int acc = 0;
        for (int j = 0; j < tid; ++j) acc += gt.len[j];
        gt.flat[tid] = acc;
        if (tid == n && acc > a.max_group_tokens) gt.bad |= 2;
    }
    __syncthreads();
    if (tid == 0) gt.n_seq = gt.bad ? 0 : n;
    __syncthreads();
}

// ------------------------------------------------------------------------------------------------
// Match: how many pattern tokens end at each place of one stretch of a group's tokens, for every
// request of the group at once (the stretch is read once, whatever the number of requests).
// ------------------------------------------------------------------------------------------------
struct MatchShared {
    GroupTable gt;
    __attribute__((aligned(16))) int tile[kMaxPattern + kTile];   // the tokens before the tile, then the tile
    int pat[kReqWindow][kMaxPattern];
    int req[kReqWindow], plen[kReqWindow], best[kReqWindow], kept[kReqWindow];
    int4 info[kReqWindow + 1];                     // (newest token, the one before it, pattern length, -) per request
    int4 older[kReqWindow + 1];                    // the four pattern tokens before those two
    int n_req;
    int first_seq;                                 // the sequence that holds the first token a tile needs
};

// A tile is a run of kTile places of the group's tokens counted through all its sequences one after the
// other ("flat" positions), so a workgroup takes its whole stretch in one round however many sequences it
// touches.  No match runs from one sequence into the next: a place's match is bounded by its distance
// from the start of its own sequence.
__global__ __launch_bounds__(kMatchThreads) void draft_match_kernel(Args a, int B) {
    __shared__ MatchShared sh;
    const int g = blockIdx.y, part = blockIdx.x, tid = threadIdx.x;
    load_group(a, g, sh.gt);
    const int need = max(a.p_min, 1);
    const bool two = need >= 2;
    const int n_seq = sh.gt.n_seq;
    const int total = n_seq > 0 ? sh.gt.flat[n_seq] : 0;
    const int lo = part * a.chunk, hi = min(lo + a.chunk, total);
    // requests are taken in windows of kReqWindow consecutive ids: at most that many belong to this group
    for (int b0 = 0; b0 < B; b0 += kReqWindow) {
        if (tid == 0) sh.n_req = 0;
        __syncthreads();
        if (tid < kReqWindow && b0 + tid < B && a.req_group[b0 + tid] == g) {
            const int r = atomicAdd(&sh.n_req, 1);
            sh.req[r] = b0 + tid;
            sh.plen[r] = min(max(a.pattern_len[b0 + tid], 0), a.p_max);
            sh.best[r] = need, sh.kept[r] = 0;
        }
        __syncthreads();
        const int n_req = sh.n_req;
        if (n_req == 0) continue;
        for (int i = tid; i < n_req * a.p_max; i += kMatchThreads) {
            const int r = i / a.p_max, c = i - r * a.p_max;
            sh.pat[r][c] = a.pattern[static_cast<size_t>(sh.req[r]) * a.p_max + c];
        }
        __syncthreads();
        if (tid <= n_req) {
            auto back = [&](int k) { return tid < n_req && a.p_max > k ? sh.pat[tid][a.p_max - 1 - k] : 0; };
            sh.info[tid] = make_int4(back(0), back(1), tid < n_req ? sh.plen[tid] : 0, 0);
            sh.older[tid] = make_int4(back(2), back(3), back(4), back(5));
        }
        for (int t0 = lo; t0 < hi; t0 += kTile) {
            const int t1 = min(t0 + kTile, hi);                    // places of this tile: [t0, t1)
            const int halo0 = max(t0 - kMaxPattern, 0);            // first flat position the tile needs
            if (tid < n_seq && sh.gt.flat[tid] <= halo0 && halo0 < sh.gt.flat[tid + 1]) sh.first_seq = tid;
            __syncthreads();                                        // also: the previous tile is no longer read
            // Loads: for every sequence that reaches into the tile, each thread requests its 16 places (four
            // quads) and one token of the run before the tile, all from addresses clamped into the pool, then
            // keeps those that belong to the sequence.
            int tok[4 * kQuads];
#pragma unroll
            for (int c = 0; c < 4 * kQuads; ++c) tok[c] = 0;
            int before = 0;
            uint32_t inside = 0, has_prev = 0;                      // per place: may end a match; has a token before it
            for (int j = sh.first_seq; j < n_seq && sh.gt.flat[j] < t1; ++j) {
                const int f0 = sh.gt.flat[j], f1 = sh.gt.flat[j + 1];
                const int at0 = sh.gt.start[j] - f0;                // pool index of flat position 0 of this sequence
                int got[4 * kQuads];
#pragma unroll
                for (int c = 0; c < 4 * kQuads; ++c) {
                    const int p = t0 + 4 * tid + (c >> 2) * 4 * kMatchThreads + (c & 3);
                    const bool in = p >= f0 && p < f1 && p < t1;
                    got[c] = a.tokens[in ? at0 + p : 0];
                }
                const int ph = t0 - kMaxPattern + tid;
                const bool in_h = tid < kMaxPattern && ph >= f0 && ph < f1;
                const int got_h = a.tokens[in_h ? at0 + ph : 0];
#pragma unroll
                for (int c = 0; c < 4 * kQuads; ++c) {
                    const int p = t0 + 4 * tid + (c >> 2) * 4 * kMatchThreads + (c & 3);
                    const bool in = p >= f0 && p < f1 && p < t1;
                    tok[c] = in ? got[c] : tok[c];
                    if (in && p + 1 < f1) inside |= 1u << c;       // the token that follows exists
                    if (in && p > f0) has_prev |= 1u << c;
                }
                before = in_h ? got_h : before;
            }
            if (tid < kMaxPattern) sh.tile[tid] = before;
#pragma unroll
            for (int u = 0; u < kQuads; ++u)
                *reinterpret_cast<int4*>(&sh.tile[kMaxPattern + 4 * tid + u * 4 * kMatchThreads]) =
                    make_int4(tok[4 * u], tok[4 * u + 1], tok[4 * u + 2], tok[4 * u + 3]);
            __syncthreads();
            // the token before each of this thread's quads (the others are in its registers)
            int prev_quad[kQuads];
#pragma unroll
            for (int u = 0; u < kQuads; ++u) prev_quad[u] = sh.tile[kMaxPattern + 4 * tid + u * 4 * kMatchThreads - 1];
            int4 info = sh.info[0], older = sh.older[0];
            for (int r = 0; r < n_req; ++r) {
                // A place counts only if at least `need` pattern tokens end there: with need >= 2 the token
                // before it is tested too, in registers, which leaves few places to look at closely.
                // (The next request's constants are requested before this one's are used.)
                const int newest = info.x, second = info.y, plen = info.z;
                const int p2 = older.x, p3 = older.y, p4 = older.z, p5 = older.w;
                info = sh.info[r + 1], older = sh.older[r + 1];
                if (plen < need) continue;
                // first only whether any lane holds a candidate at all: two compares per place
                bool any = false;
#pragma unroll
                for (int c = 0; c < 4 * kQuads; ++c) {
                    const int prev = (c & 3) ? tok[c - 1] : prev_quad[c >> 2];
                    any |= (tok[c] == newest) & (!two | (prev == second));
                }
                if (__ballot(any) == 0) continue;
                uint32_t hits = 0;
#pragma unroll
                for (int c = 0; c < 4 * kQuads; ++c) {
                    const int prev = (c & 3) ? tok[c - 1] : prev_quad[c >> 2];
                    bool h = tok[c] == newest && ((inside >> c) & 1u) != 0;
                    if (two) h = h && prev == second && ((has_prev >> c) & 1u) != 0;
                    hits |= static_cast<uint32_t>(h) << c;
                }
                if (__ballot(hits != 0) == 0) continue;
                uint32_t* out = a.list_a + static_cast<size_t>(sh.req[r]) * a.cap + static_cast<size_t>(part) * a.chunk;
                int best = sh.best[r];
                // every lane that has candidate places takes one of them per round
                while (__ballot(hits != 0) != 0) {
                    int m = 0, seq_of = 0, off = 0;
                    if (hits != 0) {
                        const int c = __builtin_ctz(hits);
                        hits &= hits - 1;
                        const int p = t0 + 4 * tid + (c >> 2) * 4 * kMatchThreads + (c & 3);
                        int j = sh.first_seq;                              // the sequence that holds place p
                        while (p >= sh.gt.flat[j + 1]) ++j;
                        seq_of = j, off = p - sh.gt.flat[j];
                        const int limit = min(plen, off + 1);             // not past the start of the sequence
                        const int* at = &sh.tile[kMaxPattern + (p - t0)];
                        // the five tokens before the place are requested together and compared in registers;
                        // only a longer match goes on through LDS
                        const int v1 = at[-1], v2 = at[-2], v3 = at[-3], v4 = at[-4], v5 = at[-5];
                        m = 1;
                        if (1 < limit && v1 == second) {
                            m = 2;
                            if (2 < limit && v2 == p2) {
                                m = 3;
                                if (3 < limit && v3 == p3) {
                                    m = 4;
                                    if (4 < limit && v4 == p4) {
                                        m = 5;
                                        if (5 < limit && v5 == p5) {
                                            m = 6;
                                            while (m < limit && at[-m] == sh.pat[r][a.p_max - 1 - m]) ++m;
                                        }
                                    }
                                }
                            }
                        }
                    }
                    // a shorter match than one already seen in this stretch can never win
                    const bool keep = m >= best;
                    if (__ballot(keep) == 0) continue;
                    if (keep && m > best) {
                        atomicMax(&sh.best[r], m);
                        best = m;
                    }
                    const int slot = wave_append(&sh.kept[r], keep);
                    if (keep) out[slot] = pack_place(seq_of, m, off + 1);
                }
            }
            __syncthreads();                                        // sh.first_seq and the tile are free again
        }
        __syncthreads();
        if (tid < n_req)
            a.part_hdr[static_cast<size_t>(sh.req[tid]) * a.parts + part] = make_int2(sh.kept[tid], sh.kept[tid] > 0 ? sh.best[tid] : 0);
        __syncthreads();
    }
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
    int base, n, slot;     // its places are list[base .. base + n) while the places live in global memory
};

// What the expansion keeps in LDS.
struct Expand {
    GroupTable gt;
    uint32_t key[kTableSlots];
    uint32_t cnt[kTableSlots];
    uint64_t cand[kSmall];                 // candidates of a level: count << 32 | ~key
    uint32_t place[kSmall];                // hand-over of places between the phases
    int8_t owner[kSmall];                  // rank of the member a place belongs to, -1 = dropped
    int2 hdr[kMaxParts];
    int first[kMaxParts + 1];              // places of the longest match before part p
    Member mem[kMaxTopK], next[kMaxTopK];  // members while the places live in global memory
    int mem_slot[2][kMaxTopK];             // members while the places live in registers: slot and ancestor mask,
    uint64_t mem_msk[2][kMaxTopK];         //   level d - 1 in buffer (d - 1) & 1
    uint64_t red[kThreads / 64];
    uint64_t best[kMaxTopK];
    int ref[kMaxTopK], ref_cnt[kMaxTopK];  // the token all places of a member show, and how many show it
    uint64_t pick[kMaxTopK];               // chosen children: count << 32 | ~key, best first
    int fill[kMaxTopK];
    int tok[SEER_MAX_T], par[SEER_MAX_T], num[SEER_MAX_T];
    uint64_t msk[SEER_MAX_T];
    int n, best_len, nmem, overflow, n_cand;
};

// Workgroup barrier, or (SOLO: wave 0 works alone) only an ordering point for the wave's own LDS traffic.
template <bool SOLO>
__device__ __forceinline__ void level_sync() {
    if (SOLO) {
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
    } else {
        __syncthreads();
    }
}

// count[key] += n in the hash table (open addressing, linear probing).
__device__ __forceinline__ void hash_add(Expand& x, int table, int shift, uint32_t key, uint32_t n) {
    uint32_t h = (key * 2654435761u) >> shift;
    for (int probes = 0; probes < table; ++probes) {
        const uint32_t old = atomicCAS(&x.key[h], kEmpty, key);
        if (old == kEmpty || old == key) {
            atomicAdd(&x.cnt[h], n);
            return;
        }
        h = (h + 1) & (table - 1);
    }
    x.overflow = 1;
}

// Places in global memory: the first top_k table entries in the order (count descending, key ascending)
// that pass the confidence test join x.pick (kept sorted, best first, at most top_k long).  Every thread
// returns the new length.
__device__ __forceinline__ int pick_top(Expand& x, int slots, float threshold, int top_k, int n_pick) {
    const int tid = threadIdx.x;
    for (int round = 0; round < top_k; ++round) {
        uint64_t best = 0;
        for (int s = tid; s < slots; s += kThreads) {
            const uint32_t c = x.cnt[s];
            if (c == 0 || static_cast<float>(c) < threshold) continue;
            const uint64_t v = (static_cast<uint64_t>(c) << 32) | static_cast<uint32_t>(~x.key[s]);
            best = v > best ? v : best;
        }
        uint64_t win = wave_max_u64(best);
        if (lane_id() == 0) x.red[tid >> 6] = win;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < kThreads / 64; ++w) win = x.red[w] > win ? x.red[w] : win;
        if (win == 0) {
            __syncthreads();
            break;
        }
        const uint32_t win_key = ~static_cast<uint32_t>(win);
        for (int s = tid; s < slots; s += kThreads)
            if (x.key[s] == win_key) x.cnt[s] = 0;
        if (tid == 0) {
            int at = n_pick < top_k ? n_pick : top_k - 1;
            if (n_pick < top_k || win > x.pick[at]) {
                while (at > 0 && x.pick[at - 1] < win) {
                    x.pick[at] = x.pick[at - 1];
                    --at;
                }
                x.pick[at] = win;
            }
        }
        n_pick = min(n_pick + 1, top_k);
        __syncthreads();
    }
    return n_pick;
}

// Places in global memory: the picks of level d become draft nodes (one thread).
__device__ __forceinline__ void emit_nodes(Expand& x, int d, int top_k, int n_pick) {
    int base = 0;
    for (int j = 0; j < n_pick; ++j) {
        const uint32_t key = ~static_cast<uint32_t>(x.pick[j]);
        const int c = static_cast<int>(x.pick[j] >> 32), r = static_cast<int>(key >> 24);
        const int slot = 1 + (d - 1) * top_k + j, parent = x.mem[r].slot;
        x.tok[slot] = static_cast<int>(key & 0xffffffu);
        x.par[slot] = parent;
        x.num[slot] = c;
        x.msk[slot] = (1ull << slot) | x.msk[parent];
        x.next[j] = Member{base, c, slot};            // x.mem is still needed until the places are reassigned
        x.fill[j] = 0;
        base += c;
    }
}

// One level for the places a thread holds in registers (own[u] = rank of the member the place belongs to
// or -1, t[u] = the token the place shows at this level or -1).  Counting in the LDS hash table, then the
// candidates (one per distinct (member, token) pair, held by the thread that entered the pair) are ranked:
// against each other if they are few, else by top_k rounds of a maximum.  The thread that holds the pick
// of rank j writes draft node j of the level.  Returns the number of picks; n_alive = places they own.
template <bool SOLO, int PER>
__device__ __forceinline__ int reg_level(const Args& a, Expand& x, int d, float threshold, int n_mem, int (&own)[PER],
                                         const int (&t)[PER], int& n_alive, int& chain_slot, uint64_t& chain_mask) {
    const int me = SOLO ? lane_id() : static_cast<int>(threadIdx.x), stride = SOLO ? 64 : kThreads;
    const uint64_t below = (1ull << lane_id()) - 1;
    uint32_t k[PER];
    bool act[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        act[u] = own[u] >= 0 && t[u] >= 0;       // else the sequence ends here, or the token cannot be proposed
        k[u] = (static_cast<uint32_t>(own[u]) << 24) | static_cast<uint32_t>(t[u]);
    }
    uint64_t v[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) v[u] = 0;
    // Inside a phrase that recurs, all places of a member show the same token: then there is nothing to
    // count pair by pair.
    // One wave, one member: ballots settle it without touching LDS (chain_slot < 0: the member's slot and
    // ancestor mask are not in registers yet).
    if (SOLO && n_mem == 1) {
        int count = 0, ref = -1;
        bool have = false;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const uint64_t m = __ballot(act[u]);
            count += __popcll(m);
            if (!have && m != 0) {
                ref = __builtin_amdgcn_readlane(t[u], __builtin_amdgcn_readfirstlane(__ffsll(static_cast<long long>(m)) - 1));
                have = true;
            }
        }
        if (!have) return 0;                                         // no place goes on
        bool differ = false;
#pragma unroll
        for (int u = 0; u < PER; ++u) differ = differ || __ballot(act[u] && t[u] != ref) != 0;
        if (!differ) {
            if (static_cast<float>(count) < threshold) return 0;
            const int from = (d - 1) & 1, slot = 1 + (d - 1) * a.top_k;
            if (chain_slot < 0) chain_slot = x.mem_slot[from][0], chain_mask = x.mem_msk[from][0];
            const uint64_t m = (1ull << slot) | chain_mask;
            if (me == 0) {
                x.tok[slot] = ref, x.par[slot] = chain_slot, x.num[slot] = count, x.msk[slot] = m;
                x.mem_slot[from ^ 1][0] = slot, x.mem_msk[from ^ 1][0] = m;
            }
            chain_slot = slot, chain_mask = m;
#pragma unroll
            for (int u = 0; u < PER; ++u) own[u] = act[u] ? 0 : -1;
            n_alive = count;
            return 1;
        }
    }
    chain_slot = -1;
    // The whole workgroup, one member: every place writes its token as the member's reference (any one
    // wins), and if all places agree with it the member itself is the candidate.
    bool unanimous = false;
    if (!SOLO && n_mem == 1) {                   // (several members are rarely all of one mind: not tried)
        if (me < kMaxTopK) x.ref_cnt[me] = 0;
        if (me == 0) x.n_cand = 0;
#pragma unroll
        for (int u = 0; u < PER; ++u)
            if (act[u]) x.ref[own[u]] = t[u];
        __syncthreads();
        bool agree = true;
#pragma unroll
        for (int u = 0; u < PER; ++u)
            if (act[u]) agree = agree && t[u] == x.ref[own[u]];
        unanimous = __syncthreads_and(agree ? 1 : 0) != 0;
    }
    if (unanimous) {
        for (int r = 0; r < n_mem; ++r) {
            int c = 0;
#pragma unroll
            for (int u = 0; u < PER; ++u) c += __popcll(__ballot(act[u] && own[u] == r));
            if (lane_id() == 0 && c) atomicAdd(&x.ref_cnt[r], c);
        }
        __syncthreads();
        if (me < n_mem) {
            const uint32_t c = static_cast<uint32_t>(x.ref_cnt[me]);
            if (c > 0 && static_cast<float>(c) >= threshold)
                v[0] = (static_cast<uint64_t>(c) << 32) |
                       static_cast<uint32_t>(~((static_cast<uint32_t>(me) << 24) | static_cast<uint32_t>(x.ref[me])));
        }
    } else {
        int table = 64;
        while (table < kTableSlots && table < 2 * n_alive) table <<= 1;      // at most n_alive distinct keys
        const int shift = 32 - __builtin_ctz(static_cast<unsigned>(table));
        for (int s = me; s < table; s += stride) x.key[s] = kEmpty, x.cnt[s] = 0;
        if (me < kMaxTopK) x.best[me] = 0;
        if (me == 0) x.n_cand = 0;
        level_sync<SOLO>();
        uint32_t h[PER], old[PER];
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            h[u] = (k[u] * 2654435761u) >> shift;
            old[u] = kEmpty;
            if (act[u]) old[u] = atomicCAS(&x.key[h[u]], kEmpty, k[u]);
        }
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            if (!act[u]) continue;
            for (int probes = 0; old[u] != kEmpty && old[u] != k[u] && probes < table; ++probes) {
                h[u] = (h[u] + 1) & (table - 1);
                old[u] = atomicCAS(&x.key[h[u]], kEmpty, k[u]);
            }
            atomicAdd(&x.cnt[h[u]], 1u);
        }
        level_sync<SOLO>();
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            if (act[u] && old[u] == kEmpty) {                       // this thread entered the pair: it speaks for it
                const uint32_t c = x.cnt[h[u]];
                if (static_cast<float>(c) >= threshold) v[u] = (static_cast<uint64_t>(c) << 32) | static_cast<uint32_t>(~k[u]);
            }
        }
    }
    int wave_total = 0;
#pragma unroll
    for (int u = 0; u < PER; ++u) wave_total += __popcll(__ballot(v[u] != 0));
    int base = 0;
    if (!SOLO) {
        if (lane_id() == 0 && wave_total) base = atomicAdd(&x.n_cand, wave_total);
        base = __builtin_amdgcn_readfirstlane(base);
    }
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const uint64_t mask = __ballot(v[u] != 0);
        if (v[u] != 0) x.cand[base + __popcll(mask & below)] = v[u];
        base += __popcll(mask);
    }
    level_sync<SOLO>();
    const int n_cand = SOLO ? base : x.n_cand;
    const int n_pick = min(n_cand, a.top_k);
    if (n_pick == 0) return 0;
    const int from = (d - 1) & 1;
    auto emit = [&](int rank, uint64_t val) {
        const uint32_t key = ~static_cast<uint32_t>(val);
        const int r = static_cast<int>(key >> 24), slot = 1 + (d - 1) * a.top_k + rank;
        const int parent = x.mem_slot[from][r];
        const uint64_t m = (1ull << slot) | x.mem_msk[from][r];
        x.tok[slot] = static_cast<int>(key & 0xffffffu);
        x.par[slot] = parent;
        x.num[slot] = static_cast<int>(val >> 32);
        x.msk[slot] = m;
        x.mem_slot[from ^ 1][rank] = slot;
        x.mem_msk[from ^ 1][rank] = m;
        x.pick[rank] = val;
    };
    if (n_cand <= kRankAll) {
        // few candidates: every holder counts how many of the others beat its own (reads in batches that
        // do not wait for each other; entries past n_cand are stale and masked)
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            if (v[u] == 0) continue;
            int rank = 0;
            for (int j0 = 0; j0 < n_cand; j0 += 8) {
                uint64_t other[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) other[j] = x.cand[j0 + j];
#pragma unroll
                for (int j = 0; j < 8; ++j) rank += (j0 + j < n_cand && other[j] > v[u]) ? 1 : 0;
            }
            if (rank < a.top_k) emit(rank, v[u]);
        }
    } else {
        for (int round = 0; round < n_pick; ++round) {
            uint64_t mine = 0;
#pragma unroll
            for (int u = 0; u < PER; ++u) mine = v[u] > mine ? v[u] : mine;
            if (mine != 0) atomicMax(reinterpret_cast<unsigned long long*>(&x.best[round]), static_cast<unsigned long long>(mine));
            level_sync<SOLO>();
            const uint64_t win = x.best[round];
#pragma unroll
            for (int u = 0; u < PER; ++u)
                if (v[u] == win && win != 0) {
                    emit(round, win);
                    v[u] = 0;
                }
        }
    }
    level_sync<SOLO>();
    int alive = 0;
    int now[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) now[u] = -1;
    uint64_t picks[kMaxTopK];
#pragma unroll
    for (int j = 0; j < kMaxTopK; ++j) picks[j] = j < n_pick ? x.pick[j] : 0;
#pragma unroll
    for (int j = 0; j < kMaxTopK; ++j) {
        if (j >= n_pick) continue;
        alive += static_cast<int>(picks[j] >> 32);
#pragma unroll
        for (int u = 0; u < PER; ++u)
            if (act[u] && k[u] == ~static_cast<uint32_t>(picks[j])) now[u] = j;
    }
#pragma unroll
    for (int u = 0; u < PER; ++u) own[u] = now[u];
    n_alive = alive;
    return n_pick;
}

// Levels d .. levels with the places in registers, PER per thread, taken from x.place / x.owner.  The next
// kAhead tokens of every place are fetched at once, so that most levels run without touching global memory.
// !SOLO: the whole workgroup, until at most kSolo places are alive; then the live places go back to
// x.place / x.owner.  SOLO: wave 0 alone, no workgroup barriers.  Returns the next level (levels + 1 = finished).
template <bool SOLO, int PER>
__device__ __forceinline__ int reg_levels(const Args& a, Expand& x, int d, int levels, float threshold, int& n_places,
                                          int& n_alive, int& n_mem) {
    const int me = SOLO ? lane_id() : static_cast<int>(threadIdx.x), stride = SOLO ? 64 : kThreads;
    uint32_t place[PER];
    int own[PER];
    int chain_slot = -1;                       // one member: its slot and ancestor mask, once they are in registers
    uint64_t chain_mask = 0;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int i = me + u * stride;
        own[u] = i < n_places ? x.owner[i] : -1;
        place[u] = i < n_places ? x.place[i] : 0u;
    }
    while (d <= levels && (SOLO || n_alive > kSolo)) {
        int cont[PER][kAhead];
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int j = place_seq(place[u]), off = place_off(place[u]) + d - 1;
            const int have = own[u] >= 0 ? min(x.gt.len[j] - off, levels - d + 1) : 0;
            const int32_t* src = a.tokens + x.gt.start[j] + off;
#pragma unroll
            for (int l = 0; l < kAhead; ++l) {
                int t = -1;
                if (l < have) t = src[l];
                cont[u][l] = t >= a.vocab ? -1 : t;
            }
        }
        // One copy of the level's code, whatever the level: the fetched tokens are picked out of the registers
        // by compares (unrolled eight times the code would not stay in the instruction cache).
        bool done = false;
#pragma nounroll
        for (int l = 0; l < kAhead && !done && d <= levels && (SOLO || n_alive > kSolo); ++l) {
            int t[PER];
#pragma unroll
            for (int u = 0; u < PER; ++u) {
                t[u] = cont[u][0];
#pragma unroll
                for (int i = 1; i < kAhead; ++i) t[u] = l == i ? cont[u][i] : t[u];
            }
            const int n_pick = reg_level<SOLO, PER>(a, x, d, threshold, n_mem, own, t, n_alive, chain_slot, chain_mask);
            if (n_pick == 0) {
                done = true;
                d = levels + 1;
            } else {
                n_mem = n_pick;
                ++d;
            }
        }
    }
    if (!SOLO && d <= levels) {
        // the live places go to wave 0
        if (threadIdx.x == 0) x.n = 0;
        __syncthreads();
        int wave_total = 0;
#pragma unroll
        for (int u = 0; u < PER; ++u) wave_total += __popcll(__ballot(own[u] >= 0));
        int base = 0;
        if (lane_id() == 0 && wave_total) base = atomicAdd(&x.n, wave_total);
        base = __builtin_amdgcn_readfirstlane(base);
        const uint64_t below = (1ull << lane_id()) - 1;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const uint64_t mask = __ballot(own[u] >= 0);
            if (own[u] >= 0) {
                const int at = base + __popcll(mask & below);
                x.place[at] = place[u], x.owner[at] = static_cast<int8_t>(own[u]);
            }
            base += __popcll(mask);
        }
        __syncthreads();
        n_places = x.n;
    }
    return d;
}

__global__ __launch_bounds__(kThreads) void draft_expand_kernel(Args a) {
    __shared__ Expand x;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int T = 1 + a.top_k * a.gamma_max;
    // what the match workgroups left (requested before the group table, whose loads it does not depend on)
    int2 h = make_int2(0, 0);
    if (tid < a.parts) h = a.part_hdr[static_cast<size_t>(b) * a.parts + tid];
    const int plen = min(max(a.pattern_len[b], 0), a.p_max);
    const int want = a.max_spec_tokens[b];
    load_group(a, a.req_group[b], x.gt);
    if (tid < T) {
        x.tok[tid] = tid == 0 && plen > 0 ? a.pattern[static_cast<size_t>(b) * a.p_max + a.p_max - 1] : -1;
        x.par[tid] = tid == 0 ? -1 : -2;
        x.num[tid] = 0;
        x.msk[tid] = 1ull << tid;
    }
    if (tid == 0) x.n = 0, x.best_len = 0;
    __syncthreads();
    if (x.gt.bad && tid == 0 && a.status) atomicOr(a.status, x.gt.bad);
    if (x.gt.n_seq == 0) h = make_int2(0, 0);
    if (h.x > 0) atomicMax(&x.best_len, h.y);
    __syncthreads();
    const int p_star = x.best_len;
    // places of the longest match, part by part: how many come before part p
    if (tid < a.parts) x.hdr[tid] = make_int2(h.y == p_star ? h.x : 0, h.y);
    __syncthreads();
    if (tid <= a.parts) {
        int acc = 0;
        for (int p = 0; p < tid; ++p) acc += x.hdr[p].x;
        x.first[tid] = acc;
    }
    __syncthreads();
    const int n_kept = p_star > 0 ? x.first[a.parts] : 0;        // >= the places of the longest match
    uint32_t* cur = a.list_b + static_cast<size_t>(b) * a.cap;
    uint32_t* nxt = a.list_a + static_cast<size_t>(b) * a.cap;
    bool handed_over = n_kept <= kSmall;
    for (int i0 = 0; i0 < n_kept; i0 += kThreads) {
        const int i = i0 + tid;
        uint32_t pl = 0;
        if (i < n_kept) {
            int lo = 0, hi = a.parts;                              // the part that holds kept place i
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (x.first[mid] <= i) lo = mid; else hi = mid;
            }
            pl = nxt[static_cast<size_t>(lo) * a.chunk + (i - x.first[lo])];
        }
        const bool hit = i < n_kept && place_len(pl) == p_star;
        const int at = wave_append(&x.n, hit);
        if (hit) {
            if (handed_over)
                x.place[at] = pl, x.owner[at] = 0;
            else
                cur[at] = pl;
        }
    }
    __syncthreads();
    const int n_root = x.n;
    const int levels = p_star > 0 ? min(max(want, 0), a.gamma_max) : 0;
    const float threshold = a.min_confidence * static_cast<float>(n_root);
    if (tid == 0) {
        x.num[0] = n_root;
        x.mem[0] = Member{0, n_root, 0};
        x.nmem = 1;
    }
    __syncthreads();

    int d = 1;
    // ---- places in global memory: as long as a level holds more than kSmall places ----
    for (; d <= levels && !handed_over; ++d) {
        const int nmem = x.nmem;
        const int n_level = x.mem[nmem - 1].base + x.mem[nmem - 1].n;
        if (n_level <= kSmall) {
            for (int e = tid; e < n_level; e += kThreads) {
                int r = 0;
                while (r + 1 < nmem && e >= x.mem[r + 1].base) ++r;
                x.place[e] = cur[e], x.owner[e] = static_cast<int8_t>(r);
            }
            handed_over = true;
            __syncthreads();
            break;
        }
        // The tokens that four places per thread show at this level, with the rank of the member that owns
        // each place, as keys.  The four places are requested together, then the four tokens (from addresses
        // clamped into the pool), so that a thread waits twice per round, not eight times.
        auto keys_of = [&](int e0, uint32_t (&pl)[4], uint32_t (&key)[4], bool (&outside)[4]) {
            int at[4];
            bool ok[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) pl[u] = cur[min(e0 + u * kThreads + tid, n_level - 1)];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = place_seq(pl[u]), off = place_off(pl[u]) + d - 1;
                ok[u] = e0 + u * kThreads + tid < n_level && off < x.gt.len[j];
                at[u] = ok[u] ? x.gt.start[j] + off : 0;
            }
            int t[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) t[u] = a.tokens[at[u]];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = e0 + u * kThreads + tid;
                int r = 0;
                while (r + 1 < nmem && e >= x.mem[r + 1].base) ++r;
                outside[u] = ok[u] && (t[u] < 0 || t[u] >= a.vocab);       // a token that cannot be proposed
                key[u] = ok[u] && !outside[u] ? (static_cast<uint32_t>(r) << 24) | static_cast<uint32_t>(t[u]) : kEmpty;
            }
        };
        // A level of up to 8 places per thread is fetched once (two dependent round trips) and kept in registers
        // for the three passes below (agreement, counting, reassignment); longer levels are fetched pass by pass.
        constexpr int kHeld = 8;
        const bool held = n_level <= kHeld * kThreads;
        uint32_t hpl[kHeld], hkey[kHeld];
        bool hout[kHeld];
        if (held) {
            keys_of(0, *reinterpret_cast<uint32_t(*)[4]>(&hpl[0]), *reinterpret_cast<uint32_t(*)[4]>(&hkey[0]),
                    *reinterpret_cast<bool(*)[4]>(&hout[0]));
            keys_of(4 * kThreads, *reinterpret_cast<uint32_t(*)[4]>(&hpl[4]), *reinterpret_cast<uint32_t(*)[4]>(&hkey[4]),
                    *reinterpret_cast<bool(*)[4]>(&hout[4]));
        }
        // f(round, places, keys, outside) for every round of four places per thread
        auto for_each_round = [&](auto&& f) {
            if (held) {
                f(0, *reinterpret_cast<uint32_t(*)[4]>(&hpl[0]), *reinterpret_cast<uint32_t(*)[4]>(&hkey[0]),
                  *reinterpret_cast<bool(*)[4]>(&hout[0]));
                if (n_level > 4 * kThreads)
                    f(1, *reinterpret_cast<uint32_t(*)[4]>(&hpl[4]), *reinterpret_cast<uint32_t(*)[4]>(&hkey[4]),
                      *reinterpret_cast<bool(*)[4]>(&hout[4]));
            } else {
                for (int e0 = 0; e0 < n_level; e0 += 4 * kThreads) {
                    uint32_t pl[4], key[4];
                    bool outside[4];
                    keys_of(e0, pl, key, outside);
                    f(e0 / (4 * kThreads), pl, key, outside);
                }
            }
        };
        // A single member whose places all show the same token (inside a phrase that recurs): one pass finds
        // that out and counts them; the place list stays as it is (places whose sequence ended stay ended).
        if (nmem == 1) {
            if (tid == 0) x.ref[0] = -1, x.ref_cnt[0] = 0;
            __syncthreads();
            bool agree = true;
            int wave_count = 0;
            for_each_round([&](int round, uint32_t (&pl)[4], uint32_t (&key)[4], bool (&outside)[4]) {
                if (round == 0) {                  // any token of the first round serves as the reference
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (key[u] != kEmpty) x.ref[0] = static_cast<int>(key[u] & 0xffffffu);
                    __syncthreads();
                }
                const int ref = x.ref[0];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (outside[u]) agree = false;
                    if (key[u] != kEmpty && static_cast<int>(key[u] & 0xffffffu) != ref) agree = false;
                    wave_count += __popcll(__ballot(key[u] != kEmpty));
                }
            });
            if (lane_id() == 0 && wave_count) atomicAdd(&x.ref_cnt[0], wave_count);
            if (__syncthreads_and(agree ? 1 : 0)) {
                const int c = x.ref_cnt[0];
                if (c == 0 || static_cast<float>(c) < threshold) {
                    d = levels + 1;
                    break;
                }
                if (tid == 0) {
                    x.pick[0] = (static_cast<uint64_t>(c) << 32) | static_cast<uint32_t>(~static_cast<uint32_t>(x.ref[0]));
                    emit_nodes(x, d, a.top_k, 1);
                    x.mem[0] = Member{0, n_level, x.next[0].slot};
                }
                __syncthreads();
                continue;
            }
        }
        int n_pick = 0;
        // Pass 0 counts in a hash table.  Only if more distinct (member, token) pairs turn up than the
        // table has slots do further passes count token ranges in a directly indexed table.
        const int range = kTableSlots / nmem;                     // tokens per member in a ranged pass
        const int n_pass_ranged = (a.vocab + range - 1) / range;
        const int shift = 32 - __builtin_ctz(static_cast<unsigned>(kTableSlots));
        for (int pass = 0; pass <= n_pass_ranged; ++pass) {
            const bool hashed = pass == 0;
            for (int s = tid; s < kTableSlots; s += kThreads) x.key[s] = kEmpty, x.cnt[s] = 0;
            if (tid == 0) x.overflow = 0;
            __syncthreads();
            const int lo_tok = (pass - 1) * range;
            for_each_round([&](int, uint32_t (&pl)[4], uint32_t (&key)[4], bool (&outside)[4]) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (hashed) {
                        if (key[u] != kEmpty) hash_add(x, kTableSlots, shift, key[u], 1u);
                    } else if (key[u] != kEmpty) {
                        const int t = static_cast<int>(key[u] & 0xffffffu) - lo_tok;
                        if (t >= 0 && t < range) {
                            const int s = static_cast<int>(key[u] >> 24) * range + t;
                            x.key[s] = key[u];
                            atomicAdd(&x.cnt[s], 1u);
                        }
                    }
                }
            });
            __syncthreads();
            const bool overflow = x.overflow != 0;
            if (!(hashed && overflow)) n_pick = pick_top(x, kTableSlots, threshold, a.top_k, n_pick);
            if (hashed && !overflow) break;
        }
        if (n_pick == 0) {
            d = levels + 1;
            break;
        }
        if (tid == 0) emit_nodes(x, d, a.top_k, n_pick);
        __syncthreads();
        if (d < levels) {
            for_each_round([&](int, uint32_t (&pl)[4], uint32_t (&key)[4], bool (&outside)[4]) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    int child = -1;
                    if (key[u] != kEmpty)
                        for (int j = 0; j < n_pick; ++j)
                            if (~static_cast<uint32_t>(x.pick[j]) == key[u]) child = j;
                    // one member's places mostly go to one child: append wave by wave, child by child
                    for (int j = 0; j < n_pick; ++j) {
                        if (__ballot(child == j) == 0) continue;
                        const int at = wave_append(&x.fill[j], child == j);
                        if (child == j) nxt[x.next[j].base + at] = pl[u];
                    }
                }
            });
        }
        __syncthreads();
        if (tid < n_pick) x.mem[tid] = x.next[tid];
        if (tid == 0) x.nmem = n_pick;
        uint32_t* t = cur;
        cur = nxt;
        nxt = t;
        __syncthreads();
    }

    // ---- few enough places: they move into registers; the whole workgroup works while many are alive,
    //      then wave 0 finishes alone without barriers ----
    if (handed_over && d <= levels) {
        int n_places = min(x.mem[x.nmem - 1].base + x.mem[x.nmem - 1].n, kSmall);
        int n_alive = n_places;
        if (tid < x.nmem) {
            x.mem_slot[(d - 1) & 1][tid] = x.mem[tid].slot;
            x.mem_msk[(d - 1) & 1][tid] = x.msk[x.mem[tid].slot];
        }
        __syncthreads();
        int n_mem = x.nmem;
        if (n_alive > kSolo) d = reg_levels<false, kSmall / kThreads>(a, x, d, levels, threshold, n_places, n_alive, n_mem);
        if (d <= levels && tid < 64) reg_levels<true, kSolo / 64>(a, x, d, levels, threshold, n_places, n_alive, n_mem);
    }
    __syncthreads();

    if (tid < T) {
        const size_t o = static_cast<size_t>(b) * T + tid;
        a.draft_tokens[o] = x.tok[tid];
        a.tree_parent[o] = x.par[tid];
        a.tree_mask[o] = x.msk[tid];
        if (a.node_count) a.node_count[o] = x.num[tid];
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
    if (!p || p->B < 0 || p->n_groups < 1 || p->n_seq < 1 || p->pool_tokens < 4 || p->max_group_tokens < 1) return SEER_EINVAL;
    if (p->gamma_max < 1 || p->top_k < 1 || p->pattern_lookup_max < 1 || p->pattern_lookup_min < 0 || p->vocab < 1)
        return SEER_EINVAL;
    if (!(p->min_confidence >= 0.0f) || !(p->min_confidence <= 1.0f)) return SEER_EINVAL;
    if (p->pattern_lookup_min > p->pattern_lookup_max) return SEER_ESHAPE;
    if (1 + static_cast<int64_t>(p->top_k) * p->gamma_max > SEER_MAX_T) return SEER_ESHAPE;
    if (p->top_k > kMaxTopK || p->pattern_lookup_max > kMaxPattern || p->vocab > (1 << 24) ||
        p->pool_tokens > 0x7fff0000ll || p->n_groups > 65535)
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
    if (reinterpret_cast<uintptr_t>(workspace) % 16 != 0 || reinterpret_cast<uintptr_t>(tokens) % 16 != 0) return SEER_EALIGN;
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
    hipLaunchKernelGGL(seer::draft::draft_match_kernel, dim3(s.parts, p->n_groups), dim3(seer::draft::kMatchThreads), 0, stream, a,
                       p->B);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return static_cast<int>(err);
    hipLaunchKernelGGL(seer::draft::draft_expand_kernel, dim3(p->B), dim3(seer::draft::kThreads), 0, stream, a);
    err = hipGetLastError();
    return err == hipSuccess ? SEER_OK : static_cast<int>(err);
}

// ------------------------------------------------------------------------------------------------
// Appending the tokens a step emitted to the histories (the counterpart of the draft server's
// update call, Appendix A.2: new tokens of one request go to that request's own sequence).
// ------------------------------------------------------------------------------------------------
namespace seer {
namespace draft {

struct AppendArgs {
    int32_t* tokens;
    const int32_t* seq_start;
    int32_t* seq_len;
    const int32_t* seq_capacity;
    const int32_t* req_seq;
    const int32_t* emitted_tokens;
    const int32_t* n_emitted;
    int32_t* pattern;
    int32_t* pattern_len;
    int32_t* status;
    int64_t pool_tokens;
    int T, n_seq, p_max;
};

__global__ __launch_bounds__(64) void history_append_kernel(AppendArgs a) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const int q = a.req_seq[b];
    int n = a.n_emitted[b];
    int bad = 0;
    int start = 0, len = 0;
    if (q < 0 || q >= a.n_seq) {
        bad = 1;
    } else {
        start = a.seq_start[q];
        len = a.seq_len[q];
        const int cap = a.seq_capacity[q];
        if (start < 0 || len < 0 || cap < len || static_cast<int64_t>(start) + cap > a.pool_tokens) bad = 1;
        else if (n < 0 || n > a.T || len + n > cap) bad = 2;
    }
    if (bad) {
        if (lane == 0 && a.status) atomicOr(a.status, bad);
        if (bad == 1) return;                        // no sequence to speak of: nothing is touched
        n = 0;                                       // no room (or a count out of range): nothing is appended
    }
    if (lane < n) a.tokens[start + len + lane] = a.emitted_tokens[static_cast<size_t>(b) * a.T + lane];
    const int total = len + n;
    if (lane == 0) {
        a.seq_len[q] = total;
        if (a.pattern_len) a.pattern_len[b] = min(total, a.p_max);
    }
    if (a.pattern && lane < a.p_max) {
        // the request's newest tokens, right-aligned: the appended ones come from the emitted row, the
        // older ones from the pool
        const int back = a.p_max - 1 - lane;         // 0 = the newest token
        int t = -1;
        if (back < n) t = a.emitted_tokens[static_cast<size_t>(b) * a.T + (n - 1 - back)];
        else if (back < total) t = a.tokens[start + total - 1 - back];
        a.pattern[static_cast<size_t>(b) * a.p_max + lane] = t;
    }
}

}  // namespace draft
}  // namespace seer

extern "C" int seer_history_append(int32_t* tokens, const int32_t* seq_start, int32_t* seq_len,
                                   const int32_t* seq_capacity, const int32_t* req_seq,
                                   const int32_t* emitted_tokens, const int32_t* n_emitted, int32_t B, int32_t T,
                                   int32_t n_seq, int64_t pool_tokens, int32_t pattern_lookup_max, int32_t* pattern,
                                   int32_t* pattern_len, int32_t* status, void* hip_stream) {
    if (B < 0 || n_seq < 1 || pool_tokens < 1) return SEER_EINVAL;
    if (T < 1 || T > SEER_MAX_T) return SEER_ESHAPE;
    if (pattern_lookup_max < 1 || pattern_lookup_max > seer::draft::kMaxPattern) return pattern_lookup_max < 1 ? SEER_EINVAL : SEER_EUNSUPPORTED;
    if (pool_tokens > 0x7fff0000ll) return SEER_EUNSUPPORTED;
    if (B == 0) return SEER_OK;
    if (!tokens || !seq_start || !seq_len || !seq_capacity || !req_seq || !emitted_tokens || !n_emitted) return SEER_EINVAL;
    if ((pattern == nullptr) != (pattern_len == nullptr)) return SEER_EINVAL;
    seer::draft::AppendArgs a{};
    a.tokens = tokens, a.seq_start = seq_start, a.seq_len = seq_len, a.seq_capacity = seq_capacity, a.req_seq = req_seq;
    a.emitted_tokens = emitted_tokens, a.n_emitted = n_emitted, a.pattern = pattern, a.pattern_len = pattern_len;
    a.status = status, a.pool_tokens = pool_tokens, a.T = T, a.n_seq = n_seq, a.p_max = pattern_lookup_max;
    hipLaunchKernelGGL(seer::draft::history_append_kernel, dim3(B), dim3(64), 0, static_cast<hipStream_t>(hip_stream), a);
    const hipError_t err = hipGetLastError();
    return err == hipSuccess ? SEER_OK : static_cast<int>(err);
}
