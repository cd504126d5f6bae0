/*
 * CPU oracle for batched draft verification (speculative-decoding verify step).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  Nothing in the product path may call it and
 * it shares no code, header, table or helper with the HIP sources.
 *
 * What is computed, and which passage of the paper fixes it:
 *
 *  - Verification scores all draft tokens of a request in ONE pass of the
 *    target model instead of one pass per token (Section 2.2, "Draft" and
 *    "Verification" stages).  For attention this means: the T = gamma + 1
 *    verify positions of a request (the last accepted token plus gamma draft
 *    tokens) all attend to the request's cached context, and each additionally
 *    to those draft positions that precede it on its own draft path (a linear
 *    chain, or one of several candidate paths, Section 3.4.2 "multi-path").
 *    Each position's result must equal what serial decoding along its path
 *    would have produced (Section 3.1: the system is algorithmically
 *    lossless).  So the definition below is ordinary softmax attention of one
 *    query over "prefix + own root path", written densely in fp64.
 *
 *  - A step emits the accepted draft prefix plus one bonus token: with gamma
 *    drafts at most gamma + 1 tokens (Section 3.4.1, expected tokens per
 *    forward (1 - alpha^(gamma+1)) / (1 - alpha); Table 2 counts the bonus
 *    token in its acceptance lengths).  With several candidate paths the
 *    longest accepted one is taken (Section 3.4.2: multi-path drafting is used
 *    to lengthen acceptance).
 *
 *  The paper gives no page layout, mask encoding, tie rule or precision; the
 *  readings used here (listed in the design notes of the repository):
 *    * bf16 inputs are widened exactly; all arithmetic is fp64.
 *    * ctx_len[b] counts the T verify slots; slot s sits at logical position
 *      ctx_len[b] - T + s.  Query slot t sees every position below
 *      ctx_len[b] - T, and slot s iff bit s of tree_mask[b][t] is set
 *      (no mask given: s <= t, the causal chain).
 *    * target token of a slot = lowest index attaining the row maximum.
 *    * a node is accepted iff its parent is accepted and its token equals the
 *      parent's target token; the winner is the deepest accepted node, the
 *      lowest index among equally deep ones.
 *
 *  Every function is exact by definition (not an approximation), so the tests
 *  pin it with closed forms, reductions to textbook decode attention and brute
 *  force enumeration rather than with stored numbers.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_EARG (-1)   /* bad shape / null pointer                     */
#define ORACLE_ECTX (-2)   /* ctx_len < T or more pages than the table has */
#define ORACLE_EPAGE (-3)  /* block-table entry outside the pool           */
#define ORACLE_ETREE (-4)  /* parent not in [-2, t)                        */
#define ORACLE_ENOMEM (-5)

/* bf16 -> fp64: a bf16 is the upper half of an fp32 bit pattern. */
static double widen_bf16(uint16_t h) {
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

typedef struct {
    int B, T, Hq, Hkv, Dqk, Dv, P, num_pages, max_pages;
    double scale;
} shape_t;

static int check_shape(const shape_t *s) {
    if (s->B < 0 || s->T < 1 || s->T > 64 || s->Hq < 1 || s->Hkv < 1 || s->Hq % s->Hkv != 0 ||
        s->Dqk < 1 || s->Dv < 1 || s->P < 1 || s->num_pages < 1 || s->max_pages < 1)
        return ORACLE_EARG;
    return ORACLE_OK;
}

/* Step 1 of the definition: gather one request's K and V for one KV head into
 * dense fp64 arrays Kd[n][Dqk], Vd[n][Dv].  With a shared latent (v_pages ==
 * NULL) the value of a token is the first Dv components of its key. */
static int gather_head(const shape_t *s, const uint16_t *k_pages, const uint16_t *v_pages,
                       const int32_t *table_row, int n, int kvh, double *Kd, double *Vd) {
    for (int j = 0; j < n; ++j) {
        int lp = j / s->P, slot = j % s->P;
        if (lp >= s->max_pages) return ORACLE_ECTX;
        int32_t pg = table_row[lp];
        if (pg < 0 || pg >= s->num_pages) return ORACLE_EPAGE;
        size_t krow = (((size_t)pg * s->Hkv + kvh) * s->P + slot) * (size_t)s->Dqk;
        for (int d = 0; d < s->Dqk; ++d) Kd[(size_t)j * s->Dqk + d] = widen_bf16(k_pages[krow + d]);
        if (v_pages) {
            size_t vrow = (((size_t)pg * s->Hkv + kvh) * s->P + slot) * (size_t)s->Dv;
            for (int d = 0; d < s->Dv; ++d) Vd[(size_t)j * s->Dv + d] = widen_bf16(v_pages[vrow + d]);
        } else {
            for (int d = 0; d < s->Dv; ++d) Vd[(size_t)j * s->Dv + d] = Kd[(size_t)j * s->Dqk + d];
        }
    }
    return ORACLE_OK;
}

/* Steps 2 and 3: visibility, scores, softmax, weighted sum for ONE query row.
 * n = ctx_len, n0 = n - T, word = ancestor-or-self bits of the query's slot.
 * score[] is scratch of n doubles. */
static void attend_row(const shape_t *s, const uint16_t *qrow, const double *Kd, const double *Vd,
                       int n, int n0, uint64_t word, double *score, double *out) {
    double m = -INFINITY;
    for (int j = 0; j < n; ++j) {
        int visible = (j < n0) || ((word >> (unsigned)(j - n0)) & 1u);
        if (!visible) {
            score[j] = -INFINITY;
            continue;
        }
        double acc = 0.0;
        for (int d = 0; d < s->Dqk; ++d) acc += widen_bf16(qrow[d]) * Kd[(size_t)j * s->Dqk + d];
        score[j] = s->scale * acc;
        if (score[j] > m) m = score[j];
    }
    double Z = 0.0;
    for (int j = 0; j < n; ++j) {
        if (score[j] == -INFINITY) {
            score[j] = 0.0;
        } else {
            score[j] = exp(score[j] - m);
            Z += score[j];
        }
    }
    for (int d = 0; d < s->Dv; ++d) out[d] = 0.0;
    for (int j = 0; j < n; ++j) {
        if (score[j] == 0.0) continue;
        double p = score[j] / Z;
        for (int d = 0; d < s->Dv; ++d) out[d] += p * Vd[(size_t)j * s->Dv + d];
    }
}

static uint64_t mask_word(const uint64_t *tree_mask, int b, int t, int T) {
    if (tree_mask) return tree_mask[(size_t)b * T + t];
    /* causal chain: slots 0..t */
    return (t >= 63) ? ~(uint64_t)0 : (((uint64_t)1 << (t + 1)) - 1);
}

/* Full verify attention: out[B][T][Hq][Dv] in fp64. */
int oracle_verify_attention(double *out, const uint16_t *q, const uint16_t *k_pages,
                            const uint16_t *v_pages, const int32_t *block_table,
                            const int32_t *ctx_len, const uint64_t *tree_mask, int B, int T, int Hq,
                            int Hkv, int Dqk, int Dv, int P, int num_pages, int max_pages,
                            double scale) {
    shape_t s = {B, T, Hq, Hkv, Dqk, Dv, P, num_pages, max_pages, scale};
    int rc = check_shape(&s);
    if (rc) return rc;
    if (!out || !q || !k_pages || !block_table || !ctx_len) return ORACLE_EARG;
    if (!v_pages && Dv > Dqk) return ORACLE_EARG;
    const int G = Hq / Hkv;
    for (int b = 0; b < B; ++b) {
        const int n = ctx_len[b];
        if (n < T || (n + P - 1) / P > max_pages) return ORACLE_ECTX;
    }
    int status = ORACLE_OK;
    for (int b = 0; b < B; ++b) {
        const int n = ctx_len[b], n0 = n - T;
        for (int kvh = 0; kvh < Hkv; ++kvh) {
            double *Kd = (double *)malloc((size_t)n * Dqk * sizeof(double));
            double *Vd = (double *)malloc((size_t)n * Dv * sizeof(double));
            if (!Kd || !Vd) {
                free(Kd);
                free(Vd);
                return ORACLE_ENOMEM;
            }
            rc = gather_head(&s, k_pages, v_pages, block_table + (size_t)b * max_pages, n, kvh, Kd, Vd);
            if (rc) {
                free(Kd);
                free(Vd);
                return rc;
            }
#pragma omp parallel
            {
                double *score = (double *)malloc((size_t)n * sizeof(double));
#pragma omp for collapse(2) schedule(dynamic, 1)
                for (int t = 0; t < T; ++t) {
                    for (int g = 0; g < G; ++g) {
                        if (!score) {
#pragma omp atomic write
                            status = ORACLE_ENOMEM;
                            continue;
                        }
                        const int h = kvh * G + g;
                        const uint16_t *qrow = q + (((size_t)b * T + t) * Hq + h) * (size_t)Dqk;
                        double *o = out + (((size_t)b * T + t) * Hq + h) * (size_t)Dv;
                        attend_row(&s, qrow, Kd, Vd, n, n0, mask_word(tree_mask, b, t, T), score, o);
                    }
                }
                free(score);
            }
            free(Kd);
            free(Vd);
            if (status) return status;
        }
    }
    return ORACLE_OK;
}

/* The same definition for a chosen list of output rows: rows[i] = (b, t, h),
 * out[i][Dv].  Used to check a few outputs of workloads too large to run whole. */
int oracle_verify_attention_rows(double *out, const int32_t *rows, int n_rows, const uint16_t *q,
                                 const uint16_t *k_pages, const uint16_t *v_pages,
                                 const int32_t *block_table, const int32_t *ctx_len,
                                 const uint64_t *tree_mask, int B, int T, int Hq, int Hkv, int Dqk,
                                 int Dv, int P, int num_pages, int max_pages, double scale) {
    shape_t s = {B, T, Hq, Hkv, Dqk, Dv, P, num_pages, max_pages, scale};
    int rc = check_shape(&s);
    if (rc) return rc;
    if (!out || !rows || !q || !k_pages || !block_table || !ctx_len || n_rows < 0) return ORACLE_EARG;
    if (!v_pages && Dv > Dqk) return ORACLE_EARG;
    const int G = Hq / Hkv;
    for (int i = 0; i < n_rows; ++i) {
        int b = rows[3 * i], t = rows[3 * i + 1], h = rows[3 * i + 2];
        if (b < 0 || b >= B || t < 0 || t >= T || h < 0 || h >= Hq) return ORACLE_EARG;
        const int n = ctx_len[b];
        if (n < T || (n + P - 1) / P > max_pages) return ORACLE_ECTX;
    }
    int status = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n_rows; ++i) {
        int b = rows[3 * i], t = rows[3 * i + 1], h = rows[3 * i + 2];
        const int n = ctx_len[b], n0 = n - T;
        double *Kd = (double *)malloc((size_t)n * Dqk * sizeof(double));
        double *Vd = (double *)malloc((size_t)n * Dv * sizeof(double));
        double *score = (double *)malloc((size_t)n * sizeof(double));
        int r = (Kd && Vd && score) ? ORACLE_OK : ORACLE_ENOMEM;
        if (!r) r = gather_head(&s, k_pages, v_pages, block_table + (size_t)b * max_pages, n, h / G, Kd, Vd);
        if (!r) {
            const uint16_t *qrow = q + (((size_t)b * T + t) * Hq + h) * (size_t)Dqk;
            attend_row(&s, qrow, Kd, Vd, n, n0, mask_word(tree_mask, b, t, T), score, out + (size_t)i * Dv);
        } else {
#pragma omp atomic write
            status = r;
        }
        free(Kd);
        free(Vd);
        free(score);
    }
    return status;
}

/* Step 4: target token of each row = lowest index attaining the row maximum.
 * Plain comparison of fp32 values (+0 equals -0); inputs are NaN-free. */
int oracle_argmax(const float *logits, int64_t n_rows, int V, int32_t *target) {
    if (!logits || !target || V < 1 || n_rows < 0) return ORACLE_EARG;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) {
        const float *row = logits + (size_t)r * V;
        int best = 0;
        float bv = row[0];
        for (int v = 1; v < V; ++v) {
            if (row[v] > bv) {
                bv = row[v];
                best = v;
            }
        }
        target[r] = best;
    }
    return ORACLE_OK;
}

/* Step 5: acceptance over the parent-pointer tree, from the slots' target
 * tokens.  parent == NULL means the chain parent[t] = t - 1.
 * accepted_len[b]  = number of accepted DRAFT tokens (depth of the winner);
 * accepted_path[b] = slot ids root..winner, then -1;  bonus[b] = target of the winner. */
int oracle_accept(const int32_t *target, const int32_t *draft, const int32_t *parent, int B, int T,
                  int32_t *accepted_len, int32_t *accepted_path, int32_t *bonus) {
    if (!target || !draft || !accepted_len || !accepted_path || B < 0 || T < 1 || T > 64)
        return ORACLE_EARG;
    for (int b = 0; b < B; ++b) {
        int ok[64], depth[64], par[64];
        for (int t = 0; t < T; ++t) {
            par[t] = parent ? parent[(size_t)b * T + t] : t - 1;
            if (t == 0) par[t] = -1;
            if (par[t] < -2 || par[t] >= t) return ORACLE_ETREE;
        }
        ok[0] = 1;
        depth[0] = 0;
        int win = 0;
        for (int t = 1; t < T; ++t) {
            ok[t] = 0;
            depth[t] = 0;
            if (par[t] < 0) continue; /* padded slot */
            if (ok[par[t]] && draft[(size_t)b * T + t] == target[(size_t)b * T + par[t]]) {
                ok[t] = 1;
                depth[t] = depth[par[t]] + 1;
                if (depth[t] > depth[win]) win = t; /* strict: lowest index among equals */
            }
        }
        accepted_len[b] = depth[win];
        for (int t = 0; t < T; ++t) accepted_path[(size_t)b * T + t] = -1;
        for (int node = win, i = depth[win]; node >= 0; node = par[node], --i)
            accepted_path[(size_t)b * T + i] = node;
        if (bonus) bonus[b] = target[(size_t)b * T + win];
    }
    return ORACLE_OK;
}

int oracle_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
