// seer_mba_draft_lengths: the draft-length policy of the paper (Algorithm 1, Marginal-Benefit-Aware
// adaptive speculation, Section 3.4.2) on top of its throughput model (Section 3.4.1):
//   expected time per generated token  T_SD(B, gamma) = (1 - alpha) (D + T)(B, gamma) / (1 - alpha^(gamma+1)),
//   gamma* = argmin_gamma T_SD, total budget gamma* (B_h + B_l) draft tokens, handed out one token per
//   request of a class at a time to the class with the larger marginal benefit (high priority weighted
//   by lambda), each class capped at gamma_max.  The hand-out is written here as a merge of two
//   precomputed lists of weighted marginal gains; its result is the algorithm's.
// Host arithmetic only; the (D + T)(B, gamma) row comes from measured verify-step times.
// Below it, the kernel that collects the acceptance probabilities the policy reads (seer_acceptance_stats).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/seer_verify.h"

extern "C" int seer_mba_draft_lengths(int32_t B_h, int32_t B_l, const double* beta, int32_t n_beta,
                                      int32_t gamma_max, double lambda, const double* step_time,
                                      int32_t* gamma_h, int32_t* gamma_l, int32_t* gamma_star) {
    if (!beta || !step_time || !gamma_h || !gamma_l) return SEER_EINVAL;
    if (B_h < 1 || B_l < 0 || gamma_max < 0 || gamma_max > SEER_MAX_T - 1) return SEER_ESHAPE;
    if (n_beta < gamma_max + 1) return SEER_ESHAPE;          // the loop reads beta[gamma + 1]
    if (!(lambda >= 1.0)) return SEER_EINVAL;
    double sum = 0.0;
    for (int i = 0; i < n_beta; ++i) {
        if (!(beta[i] >= 0.0 && beta[i] <= 1.0)) return SEER_EINVAL;
        if (i < gamma_max) sum += beta[i];
    }
    for (int g = 0; g <= gamma_max; ++g)
        if (!(step_time[g] > 0.0)) return SEER_EINVAL;
    const double alpha = gamma_max > 0 ? sum / gamma_max : 0.0;
    // gamma* = argmin of the expected time per token (smaller gamma on ties)
    int best = 0;
    double best_t = 0.0;
    double pow_alpha = 1.0;                                   // alpha^gamma
    for (int g = 0; g <= gamma_max; ++g) {
        pow_alpha *= alpha;                                   // alpha^(g + 1)
        const double t = alpha >= 1.0 ? step_time[g] / (g + 1) : (1.0 - alpha) * step_time[g] / (1.0 - pow_alpha);
        if (g == 0 || t < best_t) {
            best = g;
            best_t = t;
        }
    }
    if (gamma_star) *gamma_star = best;
    const int64_t budget = static_cast<int64_t>(best) * (static_cast<int64_t>(B_h) + B_l);
    if (budget < B_h) {                                       // not even one draft token per high-priority request
        *gamma_h = 0;
        *gamma_l = 0;
        return SEER_OK;
    }
    // The allocation is a merge of two descending-by-construction price lists.  Raising a class from level g to
    // g + 1 costs one token per request of the class and buys size * (beta[g] - beta[g + 1]) expected tokens
    // (beta[0] = 1: the token already accepted); the low class's prices carry the factor lambda, so that the
    // high class wins a round only if its gain exceeds lambda times the other's.  Both lists are written out
    // once, then rounds are dealt until neither class can take one.
    struct Klass {
        int64_t size;                      // requests: the cost of one more level
        int level;                         // draft tokens per request so far
        double price[SEER_MAX_T + 1];      // price[g]: weighted gain of level g -> g + 1
        bool can_take(int64_t left, int cap) const { return size > 0 && level < cap && left >= size; }
    };
    Klass high{B_h, 1, {}}, low{B_l, 0, {}};                  // the budget check above paid the high class's first level
    for (int g = 0; g <= gamma_max; ++g) {
        const double drop = (g == 0 ? 1.0 : beta[g - 1]) - beta[g];
        high.price[g] = static_cast<double>(B_h) * drop;
        low.price[g] = lambda * (static_cast<double>(B_l) * drop);
    }
    int64_t left = budget - B_h;
    while (left > 0) {
        // the high class takes the round if it bids more AND can pay; otherwise the round falls to the low
        // class if that one can pay; otherwise the hand-out ends
        Klass* taker = nullptr;
        if (high.price[high.level] > low.price[low.level] && high.can_take(left, gamma_max)) taker = &high;
        else if (low.can_take(left, gamma_max)) taker = &low;
        if (!taker) break;
        taker->level += 1;
        left -= taker->size;
    }
    *gamma_h = high.level;
    *gamma_l = low.level;
    return SEER_OK;
}

// ------------------------------------------------------------------------------------------------
// seer_acceptance_stats: the online side of the policy (Section 3.4.2: Algorithm 1 runs on "online-collected
// acceptance rates", per draft position).  One wave per request looks at the step's draft tree and at the
// accepted path that seer_accept wrote and adds to three counters per position k (= depth under the root):
// offered (the tree has a node of depth k), tried (the path reached depth k - 1 and its node there has a child:
// a token of depth k was compared with the target's), accepted (accepted_len >= k).  Integer counts, so the
// result does not depend on the order of the atomics.  A workgroup gathers its requests' counts in LDS and adds
// them to the caller's array once.
// ------------------------------------------------------------------------------------------------
namespace seer {
namespace {

constexpr int kStatsThreads = 256;     // four waves: four requests at a time

__global__ __launch_bounds__(kStatsThreads) void acceptance_stats_kernel(const int32_t* accepted_len,
                                                                          const int32_t* accepted_path,
                                                                          const int32_t* tree_parent, int B, int T,
                                                                          unsigned long long* counts) {
    __shared__ unsigned int s_cnt[3][SEER_MAX_T];
    for (int i = threadIdx.x; i < 3 * SEER_MAX_T; i += kStatsThreads) (&s_cnt[0][0])[i] = 0u;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int waves = (kStatsThreads >> 6) * gridDim.x;
    for (int b = blockIdx.x * (kStatsThreads >> 6) + wave; b < B; b += waves) {
        // lane t = slot t: its parent, and its depth by walking up (parents precede children, so at most T - 1 steps)
        int p = -2;
        if (lane < T) p = lane == 0 ? -1 : (tree_parent ? tree_parent[static_cast<size_t>(b) * T + lane] : lane - 1);
        if (lane > 0 && !(p >= 0 && p < lane)) p = -2;               // a padded slot: no node
        int depth = lane == 0 ? 0 : -1;
        {
            int q = p, d = 1;
            bool walking = lane > 0 && lane < T && p >= 0;
            for (int step = 0; step < T; ++step) {                   // uniform trip count: the shuffles need every lane
                const int up = __shfl(p, q < 0 ? 0 : q, 64);         // parent of q
                if (walking) {
                    if (q == 0) depth = d, walking = false;
                    else if (up < 0) walking = false;                // an ancestor is no node
                    else q = up, ++d;
                }
            }
        }
        const bool node = depth >= 0 && lane < T;
        const int a = accepted_len[b];
        // the path must be a root path of this tree: slot path[i] is a node of depth i under path[i - 1]
        bool ok = a >= 0 && a <= T - 1;
        int mine = -1;                                               // lane i: path[i]
        if (ok && lane <= a) mine = accepted_path[static_cast<size_t>(b) * T + lane];
        const int before = __shfl_up(mine, 1, 64);
        bool good = true;
        if (ok && lane <= a) {
            if (lane == 0) good = mine == 0;
            else good = mine > 0 && mine < T;
        }
        const int mine_c = mine < 0 || mine >= T ? 0 : mine;
        const int d_of = __shfl(depth, mine_c, 64), p_of = __shfl(p, mine_c, 64);
        if (ok && lane >= 1 && lane <= a && good) good = d_of == lane && p_of == before;
        ok = ok && __ballot(!good) == 0;
        if (!ok) continue;                                           // uniform: a and the ballot are
        const int last = __shfl(mine, a, 64);                        // the node the path ends in
        const bool has_child = __ballot(node && lane > 0 && p == last) != 0;
        // lane k speaks for position k
        bool offered = false;
        for (int k = 0; k < T; ++k) {                                // (T ballots: a handful of microseconds per launch at most)
            const bool any = __ballot(node && depth == k) != 0;
            if (lane == k) offered = any;
        }
        if (lane < T) {
            if (offered) atomicAdd(&s_cnt[0][lane], 1u);
            if (lane <= a || (lane == a + 1 && has_child)) atomicAdd(&s_cnt[1][lane], 1u);
            if (lane <= a) atomicAdd(&s_cnt[2][lane], 1u);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 3 * SEER_MAX_T; i += kStatsThreads) {
        const int which = i / SEER_MAX_T, k = i - which * SEER_MAX_T;
        const unsigned int c = s_cnt[which][k];
        if (c && k < T) atomicAdd(&counts[static_cast<size_t>(which) * T + k], static_cast<unsigned long long>(c));
    }
}

}  // namespace
}  // namespace seer

extern "C" int seer_acceptance_stats(const int32_t* accepted_len, const int32_t* accepted_path, const int32_t* tree_parent,
                                     int32_t B, int32_t T, uint64_t* counts, void* hip_stream) {
    if (B < 0 || T < 1 || T > SEER_MAX_T) return SEER_ESHAPE;
    if (B == 0) return SEER_OK;
    if (!accepted_len || !accepted_path || !counts) return SEER_EINVAL;
    if (reinterpret_cast<uintptr_t>(counts) % 8 != 0 || reinterpret_cast<uintptr_t>(accepted_len) % 4 != 0 ||
        reinterpret_cast<uintptr_t>(accepted_path) % 4 != 0 || reinterpret_cast<uintptr_t>(tree_parent) % 4 != 0)
        return SEER_EALIGN;
    const int per_block = seer::kStatsThreads / 64;
    int blocks = (B + per_block - 1) / per_block;
    if (blocks > 64) blocks = 64;
    hipLaunchKernelGGL(seer::acceptance_stats_kernel, dim3(blocks), dim3(seer::kStatsThreads), 0,
                       static_cast<hipStream_t>(hip_stream), accepted_len, accepted_path, tree_parent, B, T,
                       reinterpret_cast<unsigned long long*>(counts));
    const hipError_t err = hipGetLastError();
    return err == hipSuccess ? SEER_OK : static_cast<int>(err);
}

extern "C" int seer_acceptance_beta(const uint64_t* counts, int32_t T, int32_t conditional, double prior,
                                    double* beta) {
    if (!counts || !beta) return SEER_EINVAL;
    if (T < 1 || T > SEER_MAX_T) return SEER_ESHAPE;
    if (!(prior >= 0.0 && prior <= 1.0)) return SEER_EINVAL;
    const uint64_t* den = counts + (conditional ? 1 : 0) * static_cast<size_t>(T);
    const uint64_t* num = counts + 2 * static_cast<size_t>(T);
    for (int k = 1; k < T; ++k) {
        if (num[k] > den[k]) return SEER_EINVAL;             // not counts of this library
        beta[k - 1] = den[k] > 0 ? static_cast<double>(num[k]) / static_cast<double>(den[k]) : prior;
    }
    return SEER_OK;
}
