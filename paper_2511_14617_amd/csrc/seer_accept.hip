// seer_accept: target token per verify slot (vocabulary argmax) and the longest
// accepted root path over the draft tree.
//
// The paper fixes what a verification step emits -- the accepted draft prefix
// plus one bonus token (Section 3.4.1; Table 2, whose acceptance lengths count
// the bonus token) -- and that with several candidate paths the longest
// accepted one counts (Section 3.4.2).  The scan below is the HBM-bound part:
// one pass over B*T*V fp32 logits.
//
// Kernel 1 (argmax_chunks): the rows are cut into chunks of 16 384 (sampled: 8192) floats so
//   that a launch has rows*chunks workgroups (thousands, against 256 CUs) no
//   matter how B*T and V split the work.  Each workgroup streams its chunk
//   with 16-byte loads, keeps (max, lowest index) per lane, reduces across the
//   wave with shuffles and across the 4 waves through LDS, and writes one
//   (value, index) pair.
// Kernel 2 (accept_walk): one wave per request.  Lane t merges the chunk pairs
//   of slot t in ascending chunk order (strict '>' keeps the lowest index),
//   publishes the slot's target token, then lane 0 walks the parent pointers in
//   slot order: ok[t] = ok[parent] && draft[t] == target[parent], depth = depth
//   of parent + 1, winner = deepest accepted slot, lowest slot on ties.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/seer_verify.h"
#include "seer_device.h"
#include "seer_sampling.h"

namespace seer {

constexpr int kArgmaxThreads = 256;
// Floats per workgroup: 16 x 16-byte loads per lane for the greedy scan, 8 for the sampled one (measured on
// V = 152 064: 16 384 instead of 8192 floats takes the greedy scan from 54 to 52 us for 576 rows and from 374 to
// 364 us for 4224 rows; the sampled scan, bound by its arithmetic, takes the same time with either).
constexpr int kChunkGreedy = 16384;
constexpr int kChunkSampled = 8192;

__host__ __device__ inline int accept_num_chunks(int V, int chunk) { return (V + chunk - 1) / chunk; }
// the workspace holds the finer of the two partitions
__host__ __device__ inline int accept_max_chunks(int V) { return accept_num_chunks(V, kChunkSampled); }

// (a, ia) beats (b, ib) iff a > b, or a == b and ia < ib.
__device__ __forceinline__ void take_better(float& v, int& i, float ov, int oi) {
    const bool better = (ov > v) || (ov == v && oi < i);
    v = better ? ov : v;
    i = better ? oi : i;
}

// kSampled: the maximum is taken over logits[v] / tau + G(seed, row, v) (seer_sampling.h) instead of
// the logits themselves; one generator call serves the four elements of a 16-byte load.
struct SampleArgs {
    float inv_tau;
    uint32_t seed_lo, seed_hi;
};

// Upper bound of logits[v] / tau + G_v without the two logarithms: with z = the number of leading one bits of the
// generator's word (of its upper 23 bits, which are all that G uses), 1 - u > 2^-(z+1), so G < (z + 1) ln 2.
// kGumbelBoundC = ln 2 plus 0.05 for the error of the fixed-polynomial logarithms and for the roundings of the
// three fused multiply-adds involved (checked for every one of the 2^23 words on the host; the roundings stay
// below the slack while |logit / tau| < 2^17, beyond which the caller takes the exact path).
constexpr float kLn2 = 0.693147182f;
constexpr float kGumbelBoundC = 0.693147182f + 0.05f;
constexpr float kGumbelBoundMaxLogit = 131072.f;
__device__ __forceinline__ float perturb_upper_bound(float logit, float inv_tau, uint32_t w) {
    const int z = __builtin_clz(~w | 0x1ffu);          // 0 .. 23
    return __builtin_fmaf(static_cast<float>(z), kLn2, __builtin_fmaf(logit, inv_tau, kGumbelBoundC));
}

template <bool kVec4, bool kSampled>
__global__ __launch_bounds__(kArgmaxThreads) void argmax_chunks(const float* __restrict__ logits, int V,
                                                                int n_chunks, float* __restrict__ part_val,
                                                                int* __restrict__ part_idx, SampleArgs sa) {
    constexpr int kChunk = kSampled ? kChunkSampled : kChunkGreedy;
    const int row = blockIdx.x / n_chunks;
    const int chunk = blockIdx.x - row * n_chunks;
    const int begin = chunk * kChunk;
    const int end = min(V, begin + kChunk);
    const float* __restrict__ base = logits + static_cast<size_t>(row) * V;

    float best = kNegInf;
    int best_i = begin;  // a row of -inf (or an all -inf chunk) resolves to its first index
    if constexpr (kVec4 && kSampled) {
        // The sampled scan is bound by its arithmetic (ten generator rounds and two polynomial logarithms per
        // logit), and almost all of the logarithms are spent on elements that cannot win: an element whose upper
        // bound lies strictly below a perturbed value that the workgroup has already seen is neither the maximum
        // nor tied with it.  Per 16-byte load a wave evaluates the generator and the bound; only if some lane's
        // bound reaches the best value seen so far does the wave compute the four exact values of every lane.
        // The result is that of the plain scan, bit for bit: only provable losers are skipped.
        constexpr int kIter = kChunk / (kArgmaxThreads * 4);
        constexpr int kWaves = kArgmaxThreads / kWave;
        __shared__ volatile float s_seen[kWaves];        // per wave: a perturbed value it has met (its maximum so far)
        if (threadIdx.x < kWaves) s_seen[threadIdx.x] = kNegInf;
        __syncthreads();
        const int wv = threadIdx.x / kWave;
        float seen = kNegInf;                            // wave-uniform
        f32x4 x[kIter];
#pragma unroll
        for (int it = 0; it < kIter; ++it) {
            const int i = begin + (it * kArgmaxThreads + threadIdx.x) * 4;
            x[it] = (i < end) ? __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(base + i))
                              : f32x4{kNegInf, kNegInf, kNegInf, kNegInf};
        }
#pragma unroll
        for (int it = 0; it < kIter; ++it) {
            const int i = begin + (it * kArgmaxThreads + threadIdx.x) * 4;
            const Philox4 r = philox4x32_10(static_cast<uint32_t>(i) >> 2, static_cast<uint32_t>(row), 0u, 0u,
                                            sa.seed_lo, sa.seed_hi);
            // what the other waves of the workgroup have met (a stale value is still a value that was met)
            float floor_v = seen;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) floor_v = fmaxf(floor_v, s_seen[w]);
            const float u0 = perturb_upper_bound(x[it].x, sa.inv_tau, r.w[0]);
            const float u1 = perturb_upper_bound(x[it].y, sa.inv_tau, r.w[1]);
            const float u2 = perturb_upper_bound(x[it].z, sa.inv_tau, r.w[2]);
            const float u3 = perturb_upper_bound(x[it].w, sa.inv_tau, r.w[3]);
            const float ub = fmaxf(fmaxf(u0, u1), fmaxf(u2, u3));
            const float mag = fmaxf(fmaxf(fabsf(x[it].x), fabsf(x[it].y)), fmaxf(fabsf(x[it].z), fabsf(x[it].w)));
            // (written so that a NaN anywhere, an infinity or a huge logit takes the exact path)
            const bool provably_below = i >= end || (ub < floor_v && mag * fabsf(sa.inv_tau) < kGumbelBoundMaxLogit);
            if (__any(!provably_below)) {
                if (i < end) {  // indices ascend within a lane: strict '>' keeps the lowest
                    const float y0 = perturb(x[it].x, sa.inv_tau, r.w[0]);
                    const float y1 = perturb(x[it].y, sa.inv_tau, r.w[1]);
                    const float y2 = perturb(x[it].z, sa.inv_tau, r.w[2]);
                    const float y3 = perturb(x[it].w, sa.inv_tau, r.w[3]);
                    if (y0 > best) { best = y0; best_i = i; }
                    if (y1 > best) { best = y1; best_i = i + 1; }
                    if (y2 > best) { best = y2; best_i = i + 2; }
                    if (y3 > best) { best = y3; best_i = i + 3; }
                }
                float m = best;
#pragma unroll
                for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, kWave));
                seen = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(m)));
                if ((threadIdx.x & (kWave - 1)) == 0) s_seen[wv] = seen;
            }
        }
    } else if constexpr (kVec4) {
        // V % 4 == 0 and a 16-byte aligned base: every row starts aligned.
        constexpr int kIter = kChunk / (kArgmaxThreads * 4);
        f32x4 x[kIter];
#pragma unroll
        for (int it = 0; it < kIter; ++it) {
            const int i = begin + (it * kArgmaxThreads + threadIdx.x) * 4;
            x[it] = (i < end) ? __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(base + i))
                              : f32x4{kNegInf, kNegInf, kNegInf, kNegInf};
        }
#pragma unroll
        for (int it = 0; it < kIter; ++it) {
            const int i = begin + (it * kArgmaxThreads + threadIdx.x) * 4;
            if (i < end) {  // indices ascend within a lane: strict '>' keeps the lowest
                if constexpr (kSampled) {
                    const Philox4 r = philox4x32_10(static_cast<uint32_t>(i) >> 2, static_cast<uint32_t>(row), 0u, 0u,
                                                    sa.seed_lo, sa.seed_hi);
                    x[it].x = perturb(x[it].x, sa.inv_tau, r.w[0]);
                    x[it].y = perturb(x[it].y, sa.inv_tau, r.w[1]);
                    x[it].z = perturb(x[it].z, sa.inv_tau, r.w[2]);
                    x[it].w = perturb(x[it].w, sa.inv_tau, r.w[3]);
                }
                if (x[it].x > best) { best = x[it].x; best_i = i; }
                if (x[it].y > best) { best = x[it].y; best_i = i + 1; }
                if (x[it].z > best) { best = x[it].z; best_i = i + 2; }
                if (x[it].w > best) { best = x[it].w; best_i = i + 3; }
            }
        }
    } else {
        for (int i = begin + threadIdx.x; i < end; i += kArgmaxThreads) {
            float x = base[i];
            if constexpr (kSampled) {
                const Philox4 r = philox4x32_10(static_cast<uint32_t>(i) >> 2, static_cast<uint32_t>(row), 0u, 0u,
                                                sa.seed_lo, sa.seed_hi);
                x = perturb(x, sa.inv_tau, r.w[i & 3]);
            }
            if (x > best) { best = x; best_i = i; }
        }
    }
    // A lane that met nothing above -inf still reports (-inf, begin); that pair can only
    // win when the whole chunk is -inf, and then `begin` is the right answer.

#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const float ov = __shfl_xor(best, o, kWave);
        const int oi = __shfl_xor(best_i, o, kWave);
        take_better(best, best_i, ov, oi);
    }
    __shared__ float s_val[kArgmaxThreads / kWave];
    __shared__ int s_idx[kArgmaxThreads / kWave];
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) {
        s_val[wave] = best;
        s_idx[wave] = best_i;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < kArgmaxThreads / kWave; ++w) take_better(best, best_i, s_val[w], s_idx[w]);
        part_val[blockIdx.x] = best;
        part_idx[blockIdx.x] = best_i;
    }
}

__global__ __launch_bounds__(kWave) void accept_walk(const float* __restrict__ part_val,
                                                     const int* __restrict__ part_idx, int n_chunks,
                                                     const int32_t* __restrict__ draft_tokens,
                                                     const int32_t* __restrict__ tree_parent, int T,
                                                     int32_t* __restrict__ accepted_len,
                                                     int32_t* __restrict__ accepted_path,
                                                     int32_t* __restrict__ bonus_token,
                                                     int32_t* __restrict__ target_argmax) {
    __shared__ int s_tgt[SEER_MAX_T];
    __shared__ int s_draft[SEER_MAX_T];
    __shared__ int s_par[SEER_MAX_T];
    __shared__ int s_depth[SEER_MAX_T];
    __shared__ int s_path[SEER_MAX_T];
    const int b = blockIdx.x;
    const int t = threadIdx.x;
    if (t < T) {
        const size_t row = static_cast<size_t>(b) * T + t;
        float best = part_val[row * n_chunks];
        int best_i = part_idx[row * n_chunks];
        for (int c = 1; c < n_chunks; ++c) {
            const float v = part_val[row * n_chunks + c];
            if (v > best) {  // chunks ascend: strict '>' keeps the lowest index
                best = v;
                best_i = part_idx[row * n_chunks + c];
            }
        }
        target_argmax[row] = best_i;
        s_tgt[t] = best_i;
        s_draft[t] = draft_tokens[row];
        int par = tree_parent ? tree_parent[row] : t - 1;
        if (t == 0) par = -1;
        if (par < 0 || par >= t) par = (t == 0) ? -1 : -2;  // anything else counts as a padded slot
        s_par[t] = par;
        s_path[t] = -1;
    }
    __syncthreads();
    if (t == 0) {
        uint64_t ok = 1;  // bit t: slot t accepted
        int win = 0;
        s_depth[0] = 0;
        for (int i = 1; i < T; ++i) {
            const int par = s_par[i];
            int depth = 0;
            if (par >= 0 && ((ok >> par) & 1) && s_draft[i] == s_tgt[par]) {
                ok |= (1ull << i);
                depth = s_depth[par] + 1;
                if (depth > s_depth[win]) win = i;
            }
            s_depth[i] = depth;
        }
        const int len = s_depth[win];
        accepted_len[b] = len;
        if (bonus_token) bonus_token[b] = s_tgt[win];
        int node = win;
        for (int i = len; i >= 0; --i) {
            s_path[i] = node;
            node = s_par[node];
        }
    }
    __syncthreads();
    if (t < T) accepted_path[static_cast<size_t>(b) * T + t] = s_path[t];
}

}  // namespace seer

extern "C" size_t seer_accept_workspace(int32_t B, int32_t T, int32_t V) {
    if (B < 1 || T < 1 || T > SEER_MAX_T || V < 1) return 0;
    const size_t pairs = static_cast<size_t>(B) * T * seer::accept_max_chunks(V);
    return pairs * (sizeof(float) + sizeof(int32_t));
}

namespace seer {

// Argument checks that need no device: what both entry-point families share.
static int check_accept_args(const float* logits, const int32_t* draft_tokens, int32_t B, int32_t T, int32_t V,
                             const int32_t* accepted_len, const int32_t* accepted_path, const int32_t* target_token) {
    if (B < 0 || V < 1) return SEER_EINVAL;
    if (T < 1 || T > SEER_MAX_T) return SEER_ESHAPE;
    if (B == 0) return SEER_OK;
    if (!logits || !draft_tokens || !accepted_len || !accepted_path || !target_token) return SEER_EINVAL;
    if (static_cast<int64_t>(B) * T * accept_max_chunks(V) > 0x7fffffffLL) return SEER_ESHAPE;
    if (reinterpret_cast<uintptr_t>(logits) % 4 != 0) return SEER_EALIGN;
    return SEER_OK;
}

// The two launches.  scratch holds `capacity` (value, index) pairs: capacity floats, then capacity ints;
// the caller has checked that B * T * n_chunks pairs fit.
static int launch_accept(const float* logits, const int32_t* draft_tokens, const int32_t* tree_parent, int32_t B,
                         int32_t T, int32_t V, bool sampled, SampleArgs sa, int32_t* accepted_len,
                         int32_t* accepted_path, int32_t* bonus_token, int32_t* target_token, void* scratch,
                         size_t capacity, hipStream_t stream) {
    const int n_chunks = accept_num_chunks(V, sampled ? kChunkSampled : kChunkGreedy);
    float* part_val = static_cast<float*>(scratch);
    int* part_idx = reinterpret_cast<int*>(part_val + capacity);
    const bool vec4 = (V % 4 == 0) && (reinterpret_cast<uintptr_t>(logits) % 16 == 0);
    const dim3 grid(static_cast<unsigned>(static_cast<size_t>(B) * T * n_chunks));
    const dim3 block(kArgmaxThreads);
    if (vec4 && sampled) hipLaunchKernelGGL((argmax_chunks<true, true>), grid, block, 0, stream, logits, V, n_chunks, part_val, part_idx, sa);
    else if (vec4) hipLaunchKernelGGL((argmax_chunks<true, false>), grid, block, 0, stream, logits, V, n_chunks, part_val, part_idx, sa);
    else if (sampled) hipLaunchKernelGGL((argmax_chunks<false, true>), grid, block, 0, stream, logits, V, n_chunks, part_val, part_idx, sa);
    else hipLaunchKernelGGL((argmax_chunks<false, false>), grid, block, 0, stream, logits, V, n_chunks, part_val, part_idx, sa);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return static_cast<int>(err);
    hipLaunchKernelGGL(accept_walk, dim3(B), dim3(kWave), 0, stream, part_val, part_idx, n_chunks, draft_tokens,
                       tree_parent, T, accepted_len, accepted_path, bonus_token, target_token);
    err = hipGetLastError();
    return err == hipSuccess ? SEER_OK : static_cast<int>(err);
}

static int run_accept(const float* logits, const int32_t* draft_tokens, const int32_t* tree_parent, int32_t B,
                      int32_t T, int32_t V, bool sampled, SampleArgs sa, int32_t* accepted_len,
                      int32_t* accepted_path, int32_t* bonus_token, int32_t* target_token, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
    const int rc = check_accept_args(logits, draft_tokens, B, T, V, accepted_len, accepted_path, target_token);
    if (rc != SEER_OK || B == 0) return rc;
    const size_t need = seer_accept_workspace(B, T, V);
    if (!workspace || workspace_bytes < need) return SEER_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) % 16 != 0) return SEER_EALIGN;
    const size_t capacity = static_cast<size_t>(B) * T * accept_max_chunks(V);     // pairs the workspace holds
    return launch_accept(logits, draft_tokens, tree_parent, B, T, V, sampled, sa, accepted_len, accepted_path,
                         bonus_token, target_token, workspace, capacity, static_cast<hipStream_t>(hip_stream));
}

}  // namespace seer

extern "C" int seer_accept(const float* logits, const int32_t* draft_tokens, const int32_t* tree_parent,
                           int32_t B, int32_t T, int32_t V, int32_t* accepted_len, int32_t* accepted_path,
                           int32_t* bonus_token, int32_t* target_argmax, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
    return seer::run_accept(logits, draft_tokens, tree_parent, B, T, V, false, seer::SampleArgs{1.f, 0u, 0u},
                            accepted_len, accepted_path, bonus_token, target_argmax, workspace, workspace_bytes,
                            hip_stream);
}

extern "C" int seer_accept_sampled(const float* logits, const int32_t* draft_tokens, const int32_t* tree_parent,
                                   int32_t B, int32_t T, int32_t V, float temperature, uint64_t seed,
                                   int32_t* accepted_len, int32_t* accepted_path, int32_t* bonus_token,
                                   int32_t* target_token, void* workspace, size_t workspace_bytes,
                                   void* hip_stream) {
    if (!(temperature > 0.f) || temperature > 3.0e38f) return SEER_EINVAL;   // positive and finite
    const seer::SampleArgs sa{1.0f / temperature, static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32)};
    return seer::run_accept(logits, draft_tokens, tree_parent, B, T, V, true, sa, accepted_len, accepted_path,
                            bonus_token, target_token, workspace, workspace_bytes, hip_stream);
}

// ---------------------------------------------------------------------------
// seer_accept_static: seer_accept for callers that cannot allocate.  The chunk results of the scan live in
// a fixed array in the library's own device image instead of a caller workspace.
// ---------------------------------------------------------------------------
namespace seer {

constexpr size_t kStaticPairs = size_t{SEER_ACCEPT_STATIC_MAX_PAIRS};      // (value, index) pairs
static __device__ __align__(256) unsigned char scratch[kStaticPairs * (sizeof(float) + sizeof(int32_t))];

// In host code `scratch` is only a stand-in for the symbol, not a device address; every GPU holds its own
// copy of the array at its own address, looked up once per device and kept here.
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_lock;
static void* g_scratch_ptr[kMaxDevices];

static int static_scratch(void** ptr) {
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return static_cast<int>(err);
    if (dev < 0 || dev >= kMaxDevices) return static_cast<int>(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return static_cast<int>(err);
        if (!p) return static_cast<int>(hipErrorInvalidSymbol);
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return SEER_OK;
}

}  // namespace seer

extern "C" int seer_accept_static(const float* logits, const int32_t* draft_tokens, const int32_t* tree_parent,
                                  int32_t B, int32_t T, int32_t V, int32_t* accepted_len, int32_t* accepted_path,
                                  int32_t* bonus_token, int32_t* target_argmax, void* hip_stream) {
    const int rc = seer::check_accept_args(logits, draft_tokens, B, T, V, accepted_len, accepted_path, target_argmax);
    if (rc != SEER_OK) return rc;
    const size_t pairs = static_cast<size_t>(B) * T * seer::accept_num_chunks(V, seer::kChunkGreedy);
    if (pairs > seer::kStaticPairs) return SEER_ELIMIT;
    void* ptr = nullptr;
    const int rs = seer::static_scratch(&ptr);      // also with B == 0: resolves the address, launches nothing
    if (rs != SEER_OK || B == 0) return rs;
    // Every pair the walk reads is written by this call's scan first, so nothing has to start at zero.
    return seer::launch_accept(logits, draft_tokens, tree_parent, B, T, V, false, seer::SampleArgs{1.f, 0u, 0u},
                               accepted_len, accepted_path, bonus_token, target_argmax, ptr, seer::kStaticPairs,
                               static_cast<hipStream_t>(hip_stream));
}
