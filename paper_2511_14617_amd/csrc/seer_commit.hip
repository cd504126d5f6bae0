// seer_kv_commit: the step right after verification.
//
// A verify step scores T = gamma + 1 positions whose keys/values sit at the request's last T
// logical positions, slot s at n0 + s.  With several candidate paths (Section 3.4.2, multi-path
// drafting) one root path is accepted; the sequence must continue exactly as serial decoding
// would have produced it (Section 3.1, lossless), i.e. prefix + root + accepted draft tokens in
// path order.  So the rows of path[1..a] move to positions n0+1 .. n0+a, the length becomes
// n0 + 1 + a, and the step emits the a accepted draft tokens plus the bonus token (Section
// 3.4.1).  For a linear chain path[i] = i and nothing moves.
//
// One workgroup per request; per KV head it reads all rows to move into registers, waits for the
// whole workgroup, then writes them (a destination may be another row's source).  The amount of
// data is tiny (at most 63 rows of 256..1152 bytes per head), so this is a latency-sized kernel.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/seer_verify.h"
#include "seer_device.h"

namespace seer {

constexpr int kCommitThreads = 256;
constexpr int kCommitMaxPerThread = 18;   // 16-byte chunks a thread holds: 63 rows x 72 chunks / 256 threads

struct CommitArgs {
    unsigned char* k_pages;
    unsigned char* v_pages;          // nullptr: shared latent
    const int32_t* block_table;
    int32_t* ctx_len;
    const int32_t* accepted_len;
    const int32_t* accepted_path;
    const int32_t* draft_tokens;     // may be nullptr (then nothing is emitted)
    const int32_t* bonus_token;
    int32_t* emitted_tokens;
    int32_t* n_emitted;
    int32_t* status;                 // may be nullptr
    int T, Hkv, P, num_pages, max_pages;
    int k_chunks, v_chunks;          // 16-byte chunks per K row, per V row
};

__global__ __launch_bounds__(kCommitThreads) void kv_commit_kernel(CommitArgs a) {
    __shared__ int s_path[SEER_MAX_T];
    __shared__ int s_bad;
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int T = a.T;
    const int n = a.ctx_len[b];
    const int n0 = n - T;
    const int len = a.accepted_len[b];
    if (tid == 0) s_bad = 0;
    if (tid < T) s_path[tid] = a.accepted_path[static_cast<size_t>(b) * T + tid];
    __syncthreads();
    // a request whose inputs are out of range is left as it is and reported
    int bad = 0;
    if (n < T || (static_cast<int64_t>(n) + a.P - 1) / a.P > a.max_pages) bad |= 1;
    if (len < 0 || len > T - 1) bad |= 4;
    if (!bad && tid <= len) {
        const int node = s_path[tid];
        // a node is used as an index only once it is known to lie on an ascending path inside the T slots
        const bool node_ok = tid == 0 ? node == 0 : (node > s_path[tid - 1] && node > 0 && node < T);
        if (!node_ok) atomicOr(&s_bad, 4);
        if (tid >= 1 && node_ok) {
            const int32_t* table = a.block_table + static_cast<size_t>(b) * a.max_pages;
            const int p_src = table[(n0 + node) / a.P], p_dst = table[(n0 + tid) / a.P];
            if (p_src < 0 || p_src >= a.num_pages || p_dst < 0 || p_dst >= a.num_pages) atomicOr(&s_bad, 2);
        }
    }
    __syncthreads();
    bad |= s_bad;
    if (bad) {                       // uniform for the workgroup
        if (tid == 0 && a.status) atomicOr(a.status, bad);
        return;
    }

    const int32_t* table = a.block_table + static_cast<size_t>(b) * a.max_pages;
    const int per_tok = a.k_chunks + a.v_chunks;
    const int total = len * per_tok;
    for (int h = 0; h < a.Hkv; ++h) {
        u32x4 hold[kCommitMaxPerThread];
#pragma unroll
        for (int j = 0; j < kCommitMaxPerThread; ++j) {
            const int idx = tid + j * kCommitThreads;
            if (idx < total) {
                const int i = 1 + idx / per_tok, c = idx - (i - 1) * per_tok;
                const int pos = n0 + s_path[i];
                const size_t row = (static_cast<size_t>(table[pos / a.P]) * a.Hkv + h) * a.P + pos % a.P;
                const unsigned char* src = c < a.k_chunks ? a.k_pages + (row * a.k_chunks + c) * 16
                                                          : a.v_pages + (row * a.v_chunks + (c - a.k_chunks)) * 16;
                hold[j] = *reinterpret_cast<const u32x4*>(src);
            }
        }
        __syncthreads();             // every source row of this head has been read
#pragma unroll
        for (int j = 0; j < kCommitMaxPerThread; ++j) {
            const int idx = tid + j * kCommitThreads;
            if (idx < total) {
                const int i = 1 + idx / per_tok, c = idx - (i - 1) * per_tok;
                if (s_path[i] != i) {                  // already in place otherwise
                    const int pos = n0 + i;
                    const size_t row = (static_cast<size_t>(table[pos / a.P]) * a.Hkv + h) * a.P + pos % a.P;
                    unsigned char* dst = c < a.k_chunks ? a.k_pages + (row * a.k_chunks + c) * 16
                                                        : a.v_pages + (row * a.v_chunks + (c - a.k_chunks)) * 16;
                    *reinterpret_cast<u32x4*>(dst) = hold[j];
                }
            }
        }
    }
    if (tid == 0) a.ctx_len[b] = n0 + 1 + len;
    if (a.emitted_tokens && tid < T) {
        int tok = -1;
        if (tid < len) tok = a.draft_tokens[static_cast<size_t>(b) * T + s_path[tid + 1]];
        else if (tid == len) tok = a.bonus_token[b];
        a.emitted_tokens[static_cast<size_t>(b) * T + tid] = tok;
        if (tid == 0) a.n_emitted[b] = len + 1;
    }
}

}  // namespace seer

extern "C" int seer_kv_commit(const seer_attn_params* p, void* k_pages, void* v_pages, const int32_t* block_table,
                              int32_t* ctx_len, const int32_t* accepted_len, const int32_t* accepted_path,
                              const int32_t* draft_tokens, const int32_t* bonus_token, int32_t* emitted_tokens,
                              int32_t* n_emitted, int32_t* status, void* hip_stream) {
    if (!p) return SEER_EINVAL;
    if (p->B < 0 || p->num_pages < 1 || p->max_pages_per_seq < 1 || p->page_size < 1) return SEER_EINVAL;
    if (p->T < 1 || p->T > SEER_MAX_T || p->Hkv < 1 || p->Dqk < 1) return SEER_ESHAPE;
    const bool shared = p->kv_shared_latent != 0;
    if (!shared && p->Dv < 1) return SEER_ESHAPE;
    if (p->Dqk % 8 != 0 || (!shared && p->Dv % 8 != 0)) return SEER_ESHAPE;            // rows are moved in 16-byte chunks
    if (p->B == 0) return SEER_OK;
    if (!k_pages || (!shared && !v_pages) || !block_table || !ctx_len || !accepted_len || !accepted_path) return SEER_EINVAL;
    if (emitted_tokens && (!draft_tokens || !bonus_token || !n_emitted)) return SEER_EINVAL;
    if (reinterpret_cast<uintptr_t>(k_pages) % 16 != 0 || (!shared && reinterpret_cast<uintptr_t>(v_pages) % 16 != 0))
        return SEER_EALIGN;
    seer::CommitArgs a{};
    a.k_pages = static_cast<unsigned char*>(k_pages);
    a.v_pages = shared ? nullptr : static_cast<unsigned char*>(v_pages);
    a.block_table = block_table;
    a.ctx_len = ctx_len;
    a.accepted_len = accepted_len;
    a.accepted_path = accepted_path;
    a.draft_tokens = draft_tokens;
    a.bonus_token = bonus_token;
    a.emitted_tokens = emitted_tokens;
    a.n_emitted = n_emitted;
    a.status = status;
    a.T = p->T, a.Hkv = p->Hkv, a.P = p->page_size, a.num_pages = p->num_pages, a.max_pages = p->max_pages_per_seq;
    a.k_chunks = p->Dqk / 8;
    a.v_chunks = shared ? 0 : p->Dv / 8;
    if (static_cast<int64_t>(p->T - 1) * (a.k_chunks + a.v_chunks) >
        static_cast<int64_t>(seer::kCommitThreads) * seer::kCommitMaxPerThread)
        return SEER_EUNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipLaunchKernelGGL(seer::kv_commit_kernel, dim3(p->B), dim3(seer::kCommitThreads), 0, stream, a);
    const hipError_t err = hipGetLastError();
    return err == hipSuccess ? SEER_OK : static_cast<int>(err);
}
