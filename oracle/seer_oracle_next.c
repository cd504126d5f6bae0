/*
 * CPU oracle, second part: what follows and what generalises the verify step.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call it and it
 * shares no code, header, table or helper with the HIP sources.  Compiled with
 * -ffp-contract=off: the sampled path below decides an integer (an argmax) in
 * fp32, so every fp32 operation here is exactly the one written.
 *
 * 1. Committing the accepted path (oracle_kv_commit).
 *    A verify step scores T = gamma + 1 positions whose keys/values the caller
 *    has already written at the request's last T logical positions, slot s at
 *    position n0 + s.  With several candidate paths (Section 3.4.2,
 *    multi-path drafting) only one root path is accepted; since the result must
 *    equal serial decoding (Section 3.1, lossless), the sequence after the step
 *    is prefix + root + the accepted draft tokens, in path order.  So the
 *    key/value rows of path[1..a] move to positions n0+1 .. n0+a and the new
 *    length is n0 + 1 + a.  (The bonus token has no key/value yet: it is the
 *    next step's root.)  The step emits the a accepted draft tokens and the
 *    bonus token, a + 1 tokens (Section 3.4.1: accepted prefix plus bonus).
 *
 * 2. Sampled verification (oracle_argmax_sampled).
 *    The paper's workloads sample at temperature 1.0 and 0.8 (Section 4.1, setup
 *    table), and its drafts are deterministic token sequences from suffix
 *    trees, not distributions (Section 3.4).  Lossless verification of such a
 *    draft under sampling: draw the target model's token at every verify
 *    position and accept a draft token iff it equals the draw at its parent.
 *    A draw from softmax(logits / tau) is argmax_v (logits[v] / tau + G_v) with
 *    independent standard Gumbel G_v (the Gumbel-max identity), so the greedy
 *    acceptance rule applies unchanged to the perturbed logits.  To make the
 *    draw reproducible on any machine the noise is a pure function of
 *    (seed, row, v):
 *      - Philox4x32-10 (Salmon et al., "Parallel random numbers: as easy as 1,
 *        2, 3", SC'11) with counter (v / 4, row, 0, 0) and key (seed low, seed
 *        high); element v takes output word v % 4;
 *      - u = ((w >> 9) + 0.5) * 2^-23, in (0, 1), exact in fp32;
 *      - E = -log2(u) * ln2, G = -log2(E) * ln2, with log2 evaluated by the
 *        fixed fp32 polynomial below (fused multiply-adds only, so that two
 *        IEEE-754 machines get the same bits);
 *      - y_v = fma(logits[v], 1/tau, G_v) in fp32; token = lowest index
 *        attaining the maximum of y.
 *    The pins check the generator against the published known-answer vectors,
 *    the logarithm against libm, and the draws against softmax(logits / tau).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_OK = 0, ORACLE_ESHAPE = -1, ORACLE_ERANGE = -2, ORACLE_EPAGE = -3, ORACLE_EPARENT = -4, ORACLE_ENOMEM = -5 };

/* ---------------------------------------------------------------- commit -- */

/* Row of logical position j of request b, kv head h, in a pool with rows of D elements. */
static uint16_t *row_ptr(uint16_t *pool, const int32_t *table_row, int64_t j, int h, int Hkv, int P, int D) {
    const int64_t page = table_row[j / P];
    return pool + (((size_t)page * Hkv + h) * P + (size_t)(j % P)) * D;
}

int oracle_kv_commit(uint16_t *k_pages, uint16_t *v_pages, const int32_t *block_table, const int32_t *ctx_len,
                     const int32_t *accepted_len, const int32_t *accepted_path, int B, int T, int Hkv, int Dqk,
                     int Dv, int P, int num_pages, int max_pages, int32_t *ctx_len_out) {
    if (!k_pages || !block_table || !ctx_len || !accepted_len || !accepted_path || !ctx_len_out) return ORACLE_ESHAPE;
    if (B < 0 || T < 1 || Hkv < 1 || Dqk < 1 || P < 1 || num_pages < 1 || max_pages < 1) return ORACLE_ESHAPE;
    if (v_pages && Dv < 1) return ORACLE_ESHAPE;
    uint16_t *tmp = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)T * (size_t)(Dqk > Dv ? Dqk : Dv));
    if (!tmp) return ORACLE_ENOMEM;
    int rc = ORACLE_OK;
    for (int b = 0; b < B && rc == ORACLE_OK; ++b) {
        const int32_t *trow = block_table + (size_t)b * max_pages;
        const int64_t n = ctx_len[b], n0 = n - T;
        const int a = accepted_len[b];
        const int32_t *path = accepted_path + (size_t)b * T;
        if (n < T || (n + P - 1) / P > max_pages || a < 0 || a > T - 1) { rc = ORACLE_ERANGE; break; }
        if (path[0] != 0) { rc = ORACLE_EPARENT; break; }
        for (int i = 1; i <= a; ++i)
            if (path[i] <= path[i - 1] || path[i] >= T) rc = ORACLE_EPARENT;   /* parents precede children */
        for (int64_t j = n0; j < n; ++j)
            if (trow[j / P] < 0 || trow[j / P] >= num_pages) rc = ORACLE_EPAGE;
        if (rc != ORACLE_OK) break;
        for (int pool = 0; pool < 2; ++pool) {
            uint16_t *base = pool == 0 ? k_pages : v_pages;
            const int D = pool == 0 ? Dqk : Dv;
            if (!base) continue;                       /* shared latent: the values are part of the key rows */
            for (int h = 0; h < Hkv; ++h) {
                /* copy of the T draft rows as they are before the step, then the accepted ones in path order */
                for (int s = 0; s < T; ++s)
                    memcpy(tmp + (size_t)s * D, row_ptr(base, trow, n0 + s, h, Hkv, P, D), sizeof(uint16_t) * D);
                for (int i = 1; i <= a; ++i)
                    memcpy(row_ptr(base, trow, n0 + i, h, Hkv, P, D), tmp + (size_t)path[i] * D, sizeof(uint16_t) * D);
            }
        }
        ctx_len_out[b] = (int32_t)(n0 + 1 + a);
    }
    free(tmp);
    return rc;
}

/* Tokens a step emits: the accepted draft tokens in path order, then the bonus token. */
int oracle_emitted_tokens(const int32_t *draft, const int32_t *accepted_len, const int32_t *accepted_path,
                          const int32_t *bonus, int B, int T, int32_t *emitted, int32_t *n_emitted) {
    if (!draft || !accepted_len || !accepted_path || !bonus || !emitted || !n_emitted) return ORACLE_ESHAPE;
    for (int b = 0; b < B; ++b) {
        const int a = accepted_len[b];
        if (a < 0 || a > T - 1) return ORACLE_ERANGE;
        for (int i = 0; i < T; ++i) emitted[(size_t)b * T + i] = -1;
        for (int i = 1; i <= a; ++i) emitted[(size_t)b * T + i - 1] = draft[(size_t)b * T + accepted_path[(size_t)b * T + i]];
        emitted[(size_t)b * T + a] = bonus[b];
        n_emitted[b] = a + 1;
    }
    return ORACLE_OK;
}

/* -------------------------------------------------------------- sampling -- */

void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
        c0 = n0, c1 = n1, c2 = n2, c3 = n3;
        k0 += 0x9E3779B9u, k1 += 0xBB67AE85u;
    }
    out[0] = c0, out[1] = c1, out[2] = c2, out[3] = c3;
}

/* log2 of a positive normal float: exponent + polynomial on [sqrt(1/2), sqrt(2)), fused multiply-adds */
float oracle_log2_det(float x) {
    uint32_t bits;
    memcpy(&bits, &x, 4);
    int e = (int)(bits >> 23) - 127;
    bits = (bits & 0x007fffffu) | 0x3f800000u;
    float m;
    memcpy(&m, &bits, 4);
    if (m > 1.41421354f) {
        m = m * 0.5f;
        e += 1;
    }
    const float f = m - 1.0f;
    float p = 0.12614846229553223f;
    p = fmaf(p, f, -0.20742103457450867f);
    p = fmaf(p, f, 0.21566985547542572f);
    p = fmaf(p, f, -0.23892034590244293f);
    p = fmaf(p, f, 0.2879183292388916f);
    p = fmaf(p, f, -0.36070483922958374f);
    p = fmaf(p, f, 0.48091059923171997f);
    p = fmaf(p, f, -0.7213473320007324f);
    p = fmaf(p, f, 1.4426950216293335f);
    return fmaf(f, p, (float)e);
}

/* standard Gumbel deviate from one 32-bit word of the generator (its upper 23 bits) */
static float gumbel_of_word(uint32_t word) {
    const float u = ((float)(word >> 9) + 0.5f) * 1.1920928955078125e-07f;   /* 2^-23 */
    const float e = -oracle_log2_det(u) * 0.693147182f;
    return -(oracle_log2_det(e) * 0.693147182f);
}

float oracle_gumbel(uint64_t seed, uint32_t row, uint32_t v) {
    const uint32_t ctr[4] = {v >> 2, row, 0u, 0u}, key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t w[4];
    oracle_philox4x32_10(ctr, key, w);
    return gumbel_of_word(w[v & 3u]);
}

/* the same deviates for given generator words (tests sweep all 2^23 distinct inputs) */
void oracle_gumbel_of_words(const uint32_t *words, int64_t n, float *out) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = gumbel_of_word(words[i]);
}

int oracle_argmax_sampled(const float *logits, int64_t n_rows, int V, float temperature, uint64_t seed,
                          int32_t *target) {
    if (!logits || !target || n_rows < 0 || V < 1 || !(temperature > 0.0f)) return ORACLE_ESHAPE;
    const float inv_tau = 1.0f / temperature;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) {
        const float *row = logits + (size_t)r * V;
        float best = fmaf(row[0], inv_tau, oracle_gumbel(seed, (uint32_t)r, 0u));
        int32_t arg = 0;
        for (int v = 1; v < V; ++v) {
            const float y = fmaf(row[v], inv_tau, oracle_gumbel(seed, (uint32_t)r, (uint32_t)v));
            if (y > best) {
                best = y;
                arg = v;
            }
        }
        target[r] = arg;
    }
    return ORACLE_OK;
}
