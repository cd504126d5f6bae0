// seer_mba_draft_lengths: the draft-length policy of the paper (Algorithm 1, Marginal-Benefit-Aware
// adaptive speculation, Section 3.4.2) on top of its throughput model (Section 3.4.1):
//   expected time per generated token  T_SD(B, gamma) = (1 - alpha) (D + T)(B, gamma) / (1 - alpha^(gamma+1)),
//   gamma* = argmin_gamma T_SD, total budget gamma* (B_h + B_l) draft tokens, handed out one token per
//   request of a class at a time to the class with the larger marginal benefit (high priority weighted
//   by lambda), each class capped at gamma_max.  The hand-out is written here as a merge of two
//   precomputed lists of weighted marginal gains; its result is the algorithm's.
// Host arithmetic only; the (D + T)(B, gamma) row comes from measured verify-step times.
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
