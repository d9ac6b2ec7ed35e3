/*
 * CPU oracle for the batched speculative-verification step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, single-threaded
 * definition the GPU path is checked against.  It shares no code, header,
 * table or helper with the HIP library, and the product never calls it.
 * Only the tests, the smoke check and the benchmark's CPU-baseline leg may
 * load it.
 *
 * Everything floating point is computed in double.  There is no tiling, no
 * online rescaling and no reordering beyond what the definitions state.
 *
 * What it follows (paper = arXiv 2406.14066):
 *   - Section 2.2: a draft proposes k tokens; the target evaluates k+1
 *     conditional distributions in parallel; a prefix of m tokens is kept
 *     and position m+1 is always drawn from the target, so a step emits
 *     m+1 tokens, 1 <= m+1 <= k+1, with the target's own distribution.
 *   - Section 4 (overview of a generation step): scoring is one forward
 *     pass over the k+1 positions; acceptance is rejection sampling, and
 *     the emitted sequence is the validated draft tokens plus one bonus
 *     token that either corrects the first wrong draft token or extends a
 *     fully accepted draft.
 *   - Eq. 1: goodput counts generated (accepted + bonus) tokens.
 *   - Eq. 4: expected generated length (1 - a^(k+1)) / (1 - a).
 * The rejection rule itself is the one of the speculative-sampling method
 * the paper cites for its acceptance phase: accept draft token x with
 * probability min(1, p(x)/q(x)); on the first rejection draw the correction
 * from the normalised positive part of p - q; after k acceptances draw the
 * bonus from the last target distribution.
 *
 * Parity status: every function below is pinned by tests that do not go
 * through this file's own formulas (known-answer vectors of the published
 * Philox generator, brute-force dense attention, library attention, closed
 * forms and chi-square tests); nothing here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_K_MAX 8
#define ORACLE_NEAR_TIE 1e-6

/* ------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon et al., "Parallel random numbers: as easy as  */
/* 1, 2, 3").  Written from the published round function: two 32x32    */
/* -> 64 multiplies, a word permutation with key xor, and a Weyl key   */
/* schedule; ten rounds.                                                */
/* ------------------------------------------------------------------ */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod_a = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t prod_b = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(prod_b >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)prod_b;
        uint32_t n2 = (uint32_t)(prod_a >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)prod_a;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Counter layout of the step's random numbers (a choice of this build; the
 * paper only says "rejection sampling"):
 *   key     = (seed low 32, seed high 32)
 *   counter = (index, request b, step low 32, (step bits 32..55) << 8 | stream)
 *   stream 0: accept test of draft position i  -> index = i, output word 0
 *   stream 1: race variate of vocabulary id v  -> index = v >> 2, word v & 3
 */
static uint32_t philox_word(uint64_t seed, uint64_t step, uint32_t stream,
                            uint32_t b, uint32_t index, int word)
{
    uint32_t ctr[4], key[2], out[4];
    ctr[0] = index;
    ctr[1] = b;
    ctr[2] = (uint32_t)(step & 0xFFFFFFFFu);
    ctr[3] = (uint32_t)(((step >> 32) & 0xFFFFFFu) << 8) | (stream & 0xFFu);
    key[0] = (uint32_t)(seed & 0xFFFFFFFFu);
    key[1] = (uint32_t)(seed >> 32);
    oracle_philox4x32_10(ctr, key, out);
    return out[word];
}

/* u in [0,1): top 24 bits of the word times 2^-24. */
double oracle_u_accept(uint64_t seed, uint64_t step, int32_t b, int32_t i)
{
    uint32_t w = philox_word(seed, step, 0u, (uint32_t)b, (uint32_t)i, 0);
    return (double)(w >> 8) * (1.0 / 16777216.0);
}

/* U' in (0,1]: (top 24 bits + 1) times 2^-24, so -log(U') is finite and >= 0. */
double oracle_u_race(uint64_t seed, uint64_t step, int32_t b, int32_t v)
{
    uint32_t w = philox_word(seed, step, 1u, (uint32_t)b, (uint32_t)v >> 2, v & 3);
    return (double)((w >> 8) + 1u) * (1.0 / 16777216.0);
}

/* ------------------------------------------------------------------ */
/* Element access.  dtype 0 = IEEE fp32, dtype 1 = bfloat16 (the top   */
/* 16 bits of an fp32), both converted to double exactly.              */
/* ------------------------------------------------------------------ */
static double load_elem(const void *base, size_t index, int dtype)
{
    if (dtype == 0) {
        return (double)((const float *)base)[index];
    } else {
        uint32_t bits = (uint32_t)((const uint16_t *)base)[index] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
}

/* ------------------------------------------------------------------ */
/* Lookahead attention (Section 2.2: position n+i is conditioned on    */
/* x_1..x_{n+i-1}; Section 4: one scoring pass over k+1 positions).    */
/*                                                                      */
/* Request b has q_b = cu_q_len[b+1]-cu_q_len[b] query positions and    */
/* kv_len[b] cached tokens, the last q_b of which are the positions     */
/* being scored.  Query j sits at absolute position kv_len-q_b+j and    */
/* sees keys 0..that position.  Logical token t of request b lives in   */
/* physical page block_table[b][t / bs], slot t % bs.  Pages are        */
/* token-major: [num_blocks][Hkv][bs][d].  Query head h uses KV head    */
/* h / (Hq/Hkv).  Output [T][Hq][d] fp32.                               */
/* Returns 0, or -1 on a malformed argument.                            */
/* ------------------------------------------------------------------ */
int oracle_verify_attn(int32_t B, int32_t Hq, int32_t Hkv, int32_t d, int32_t bs,
                       int32_t num_blocks, int32_t max_blocks_per_req, int32_t dtype,
                       const void *q, const void *k_cache, const void *v_cache,
                       const int32_t *block_table, const int32_t *kv_len,
                       const int32_t *cu_q_len, double scale, float *out)
{
    if (B < 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || bs <= 0 || Hq % Hkv != 0) return -1;
    if (scale == 0.0) scale = 1.0 / sqrt((double)d);
    const int group = Hq / Hkv;
    int32_t max_len = 0;
    for (int b = 0; b < B; ++b) if (kv_len[b] > max_len) max_len = kv_len[b];
    double *score = (double *)malloc(sizeof(double) * (size_t)(max_len > 0 ? max_len : 1));
    double *acc = (double *)malloc(sizeof(double) * (size_t)d);
    if (!score || !acc) { free(score); free(acc); return -1; }

    for (int b = 0; b < B; ++b) {
        const int q_b = cu_q_len[b + 1] - cu_q_len[b];
        const int len = kv_len[b];
        if (q_b < 1 || len < q_b || (len + bs - 1) / bs > max_blocks_per_req) { free(score); free(acc); return -1; }
        for (int j = 0; j < q_b; ++j) {
            const int row = cu_q_len[b] + j;
            const int last_visible = len - q_b + j;
            for (int h = 0; h < Hq; ++h) {
                const int kvh = h / group;
                const size_t q_off = ((size_t)row * Hq + h) * d;
                /* scores and their maximum */
                double s_max = -INFINITY;
                for (int t = 0; t <= last_visible; ++t) {
                    const int32_t page = block_table[(size_t)b * max_blocks_per_req + t / bs];
                    if (page < 0 || page >= num_blocks) { free(score); free(acc); return -1; }
                    const size_t kv_off = (((size_t)page * Hkv + kvh) * bs + (t % bs)) * d;
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c)
                        dot += load_elem(q, q_off + c, dtype) * load_elem(k_cache, kv_off + c, dtype);
                    score[t] = dot * scale;
                    if (score[t] > s_max) s_max = score[t];
                }
                /* softmax weights, then the weighted sum of values */
                double denom = 0.0;
                for (int t = 0; t <= last_visible; ++t) {
                    score[t] = exp(score[t] - s_max);
                    denom += score[t];
                }
                for (int c = 0; c < d; ++c) acc[c] = 0.0;
                for (int t = 0; t <= last_visible; ++t) {
                    const int32_t page = block_table[(size_t)b * max_blocks_per_req + t / bs];
                    const size_t kv_off = (((size_t)page * Hkv + kvh) * bs + (t % bs)) * d;
                    const double w = score[t] / denom;
                    for (int c = 0; c < d; ++c)
                        acc[c] += w * load_elem(v_cache, kv_off + c, dtype);
                }
                for (int c = 0; c < d; ++c) out[q_off + c] = (float)acc[c];
            }
        }
    }
    free(score);
    free(acc);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Softmax of one fp32 logit row in double: prob[v] = e^(x_v - max) /  */
/* sum.                                                                 */
/* ------------------------------------------------------------------ */
void oracle_softmax_row(const float *logits, int32_t V, double *prob)
{
    double x_max = -INFINITY;
    for (int v = 0; v < V; ++v) if ((double)logits[v] > x_max) x_max = (double)logits[v];
    double denom = 0.0;
    for (int v = 0; v < V; ++v) { prob[v] = exp((double)logits[v] - x_max); denom += prob[v]; }
    for (int v = 0; v < V; ++v) prob[v] /= denom;
}

/* Probability that a draft token drawn from softmax(draft row) passes the
 * accept test against softmax(target row): sum_v min(p_v, q_v).  Used to
 * characterise synthetic inputs and in the statistical pins. */
double oracle_accept_probability(const float *target_row, const float *draft_row, int32_t V)
{
    double *p = (double *)malloc(sizeof(double) * (size_t)V);
    double *q = (double *)malloc(sizeof(double) * (size_t)V);
    oracle_softmax_row(target_row, V, p);
    oracle_softmax_row(draft_row, V, q);
    double total = 0.0;
    for (int v = 0; v < V; ++v) total += p[v] < q[v] ? p[v] : q[v];
    free(p); free(q);
    return total;
}

/* ------------------------------------------------------------------ */
/* Rejection sampling with bonus/correction token (Section 4's          */
/* acceptance phase; Section 2.2's m and m+1).                          */
/*                                                                      */
/* Request b owns target rows cu_q_len[b] .. cu_q_len[b]+k_b (k_b+1     */
/* rows) and draft rows cu_q_len[b]-b .. +k_b-1 (k_b rows); draft row i */
/* produced draft token x_i and target row i scores it.                 */
/*                                                                      */
/* Per request:                                                         */
/*  1. for i = 0..k_b-1 in order: p = softmax(target row i),            */
/*     q = softmax(draft row i), ratio = p[x_i]/q[x_i], u = accept      */
/*     uniform (b,i); accept iff u < ratio (p[x]=0 rejects, q[x]=0 with */
/*     p[x]>0 accepts); stop at the first rejection -> m_b.             */
/*  2. weights r: if m_b < k_b, r_v = max(0, p_v - q_v) of row m_b (if  */
/*     that is identically zero, r = p); else r = softmax(target row    */
/*     k_b).                                                            */
/*  3. next token = argmax_v r_v / e_v, e_v = -log(race uniform (b,v)): */
/*     the first arrival of independent exponential clocks with rates   */
/*     r_v, i.e. a draw with probability proportional to r_v.  r_v = 0  */
/*     never wins; equal scores go to the lowest v.                     */
/*  4. counters (accumulated): [0] proposed sum k_b, [1] accepted sum   */
/*     m_b, [2] attempted sum min(m_b+1,k_b) (accept tests evaluated),  */
/*     [3] emitted sum (m_b+1), [4] evaluated accept tests with         */
/*     |u - ratio| < 1e-6, [5] requests, [6],[7] untouched.             */
/*                                                                      */
/* Diagnostics (each may be NULL):                                      */
/*   dec_u, dec_ratio [T-B]: u and p/q of every evaluated accept test   */
/*     (NaN where the chain had already stopped).                       */
/*   race_margin [B]: the smallest relative perturbation of the p and q */
/*     entries that could change the race winner:                       */
/*       min over v != best of (s_best - s_v) / (w_best + w_v),         */
/*     s = r/e, w = (p+q)/e for a correction row, w = p/e for a bonus   */
/*     row.  A small value marks a decision that finite precision may   */
/*     legitimately take either way.                                    */
/*   out_tokens [B][K_MAX+1]: accepted draft tokens, then the next      */
/*     token, then -1 padding.                                          */
/* Returns 0, or -1 on a malformed argument.                            */
/* ------------------------------------------------------------------ */
int oracle_reject_sample(int32_t B, int32_t V, const float *target_logits,
                         const float *draft_logits, const int32_t *draft_tokens,
                         const int32_t *cu_q_len, uint64_t seed, uint64_t step,
                         int32_t *accepted_len, int32_t *next_token, int32_t *out_tokens,
                         int64_t *counters, double *dec_u, double *dec_ratio,
                         double *race_margin)
{
    if (B < 0 || V <= 0) return -1;
    double *p = (double *)malloc(sizeof(double) * (size_t)V);
    double *q = (double *)malloc(sizeof(double) * (size_t)V);
    double *r = (double *)malloc(sizeof(double) * (size_t)V);
    if (!p || !q || !r) { free(p); free(q); free(r); return -1; }

    for (int b = 0; b < B; ++b) {
        const int k_b = cu_q_len[b + 1] - cu_q_len[b] - 1;
        if (k_b < 0 || k_b > ORACLE_K_MAX) { free(p); free(q); free(r); return -1; }
        const size_t t_row0 = (size_t)cu_q_len[b];
        const size_t d_row0 = (size_t)cu_q_len[b] - (size_t)b;

        if (dec_u) for (int i = 0; i < k_b; ++i) { dec_u[d_row0 + i] = NAN; dec_ratio[d_row0 + i] = NAN; }

        /* step 1: the accept chain */
        int m = 0;
        int near_ties = 0;
        for (int i = 0; i < k_b; ++i) {
            const int32_t x = draft_tokens[d_row0 + i];
            if (x < 0 || x >= V) { free(p); free(q); free(r); return -1; }
            oracle_softmax_row(target_logits + (t_row0 + i) * V, V, p);
            oracle_softmax_row(draft_logits + (d_row0 + i) * V, V, q);
            double ratio;
            if (p[x] == 0.0) ratio = 0.0;
            else if (q[x] == 0.0) ratio = INFINITY;
            else ratio = p[x] / q[x];
            const double u = oracle_u_accept(seed, step, b, i);
            if (dec_u) { dec_u[d_row0 + i] = u; dec_ratio[d_row0 + i] = ratio; }
            if (fabs(u - ratio) < ORACLE_NEAR_TIE) ++near_ties;
            if (u < ratio) ++m; else break;
        }

        /* step 2: weights of the next token */
        int correction = (m < k_b);
        if (correction) {
            /* p and q still hold row m (the chain stopped there) */
            double total = 0.0;
            for (int v = 0; v < V; ++v) { r[v] = p[v] > q[v] ? p[v] - q[v] : 0.0; total += r[v]; }
            if (total == 0.0) { for (int v = 0; v < V; ++v) r[v] = p[v]; correction = 0; }
        } else {
            oracle_softmax_row(target_logits + (t_row0 + k_b) * V, V, p);
            for (int v = 0; v < V; ++v) r[v] = p[v];
        }

        /* step 3: exponential race */
        int best = -1;
        double best_score = -1.0;
        for (int v = 0; v < V; ++v) {
            if (r[v] <= 0.0) continue;
            const double e = -log(oracle_u_race(seed, step, b, v));
            const double s = (e == 0.0) ? INFINITY : r[v] / e;
            if (s > best_score) { best_score = s; best = v; }
        }
        if (best < 0) { free(p); free(q); free(r); return -1; }  /* unreachable: r sums to > 0 */

        if (race_margin) {
            double margin = INFINITY;
            const double e_best = -log(oracle_u_race(seed, step, b, best));
            const double w_best = (correction ? p[best] + q[best] : p[best]) / e_best;
            for (int v = 0; v < V; ++v) {
                if (v == best) continue;
                const double e = -log(oracle_u_race(seed, step, b, v));
                /* signed score: a loser with p < q needs its p - q perturbed past 0 before it can win */
                const double s = (correction ? p[v] - q[v] : p[v]) / e;
                const double w = (correction ? p[v] + q[v] : p[v]) / e;
                double g;
                if (isinf(best_score)) g = isinf(s) ? 0.0 : INFINITY;
                else if (w_best + w == 0.0) g = INFINITY;
                else g = (best_score - s) / (w_best + w);
                if (g < margin) margin = g;
            }
            race_margin[b] = margin;
        }

        accepted_len[b] = m;
        next_token[b] = best;
        if (out_tokens) {
            int32_t *row = out_tokens + (size_t)b * (ORACLE_K_MAX + 1);
            for (int i = 0; i <= ORACLE_K_MAX; ++i) row[i] = -1;
            for (int i = 0; i < m; ++i) row[i] = draft_tokens[d_row0 + i];
            row[m] = best;
        }
        if (counters) {
            counters[0] += k_b;
            counters[1] += m;
            counters[2] += (m + 1 < k_b) ? m + 1 : k_b;
            counters[3] += m + 1;
            counters[4] += near_ties;
            counters[5] += 1;
        }
    }
    free(p); free(q); free(r);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Greedy acceptance (Section 2.2, "Speculative Decoding": a greedy      */
/* sampling method keeps draft token i iff it is the token that         */
/* maximises the target distribution of its position, accepts the       */
/* leading run of such tokens, and takes the next token from the target  */
/* distribution that follows the last accepted one; with greedy          */
/* sampling that is its most likely token).  No random numbers, no       */
/* draft logits.  Equal maxima: the lowest token id is "the" maximiser.  */
/* The arg-max is taken on the raw fp32 logits (softmax is monotone).    */
/* counters as in oracle_reject_sample (near ties: none, slot 4 += 0).   */
/* ------------------------------------------------------------------ */
int oracle_reject_greedy(int32_t B, int32_t V, const float *target_logits,
                         const int32_t *draft_tokens, const int32_t *cu_q_len,
                         int32_t *accepted_len, int32_t *next_token, int32_t *out_tokens,
                         int64_t *counters)
{
    if (B < 0 || V <= 0) return -1;
    for (int b = 0; b < B; ++b) {
        const int k_b = cu_q_len[b + 1] - cu_q_len[b] - 1;
        if (k_b < 0 || k_b > ORACLE_K_MAX) return -1;
        const size_t t_row0 = (size_t)cu_q_len[b];
        const size_t d_row0 = (size_t)cu_q_len[b] - (size_t)b;
        int m = 0;
        int best = -1;
        for (int i = 0; i <= k_b; ++i) {
            const float *row = target_logits + (t_row0 + i) * V;
            best = 0;
            for (int v = 1; v < V; ++v)
                if (row[v] > row[best]) best = v;
            if (i == k_b) break;                         /* bonus position: nothing to compare */
            const int32_t x = draft_tokens[d_row0 + i];
            if (x < 0 || x >= V) return -1;
            if (x != best) break;                        /* first mismatch: `best` is the correction */
            ++m;
        }
        accepted_len[b] = m;
        next_token[b] = best;
        if (out_tokens) {
            int32_t *row = out_tokens + (size_t)b * (ORACLE_K_MAX + 1);
            for (int i = 0; i <= ORACLE_K_MAX; ++i) row[i] = -1;
            for (int i = 0; i < m; ++i) row[i] = draft_tokens[d_row0 + i];
            row[m] = best;
        }
        if (counters) {
            counters[0] += k_b;
            counters[1] += m;
            counters[2] += (m + 1 < k_b) ? m + 1 : k_b;
            counters[3] += m + 1;
            counters[5] += 1;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Stochastic acceptance for a proposer that gives tokens but no         */
/* distribution (Section 2.2: draft-model free speculation; Section 7:   */
/* prompt lookup and single-candidate heads).  The draft distribution    */
/* of position i is then the point mass on the proposed token x_i, and   */
/* the rule of oracle_reject_sample reads: accept iff u < p_i(x_i); at   */
/* the first rejection draw from norm(max(0, p - onehot(x))), which is   */
/* p with x removed; if all are accepted draw the bonus from p_k.        */
/* Uniforms, race and outputs as in oracle_reject_sample; dec_ratio      */
/* holds p_i(x_i).                                                       */
/* ------------------------------------------------------------------ */
int oracle_reject_onehot(int32_t B, int32_t V, const float *target_logits,
                         const int32_t *draft_tokens, const int32_t *cu_q_len,
                         uint64_t seed, uint64_t step,
                         int32_t *accepted_len, int32_t *next_token, int32_t *out_tokens,
                         int64_t *counters, double *dec_u, double *dec_ratio,
                         double *race_margin)
{
    if (B < 0 || V <= 0) return -1;
    double *p = (double *)malloc(sizeof(double) * (size_t)V);
    double *r = (double *)malloc(sizeof(double) * (size_t)V);
    if (!p || !r) { free(p); free(r); return -1; }
    for (int b = 0; b < B; ++b) {
        const int k_b = cu_q_len[b + 1] - cu_q_len[b] - 1;
        if (k_b < 0 || k_b > ORACLE_K_MAX) { free(p); free(r); return -1; }
        const size_t t_row0 = (size_t)cu_q_len[b];
        const size_t d_row0 = (size_t)cu_q_len[b] - (size_t)b;
        if (dec_u) for (int i = 0; i < k_b; ++i) { dec_u[d_row0 + i] = NAN; dec_ratio[d_row0 + i] = NAN; }

        int m = 0, near_ties = 0;
        int32_t rejected = -1;
        for (int i = 0; i < k_b; ++i) {
            const int32_t x = draft_tokens[d_row0 + i];
            if (x < 0 || x >= V) { free(p); free(r); return -1; }
            oracle_softmax_row(target_logits + (t_row0 + i) * V, V, p);
            const double ratio = p[x];                     /* q(x) = 1 */
            const double u = oracle_u_accept(seed, step, b, i);
            if (dec_u) { dec_u[d_row0 + i] = u; dec_ratio[d_row0 + i] = ratio; }
            if (fabs(u - ratio) < ORACLE_NEAR_TIE) ++near_ties;
            if (u < ratio) ++m; else { rejected = x; break; }
        }
        if (m == k_b) oracle_softmax_row(target_logits + (t_row0 + k_b) * V, V, p);
        double total = 0.0;
        for (int v = 0; v < V; ++v) { r[v] = (v == rejected) ? 0.0 : p[v]; total += r[v]; }
        if (total == 0.0) for (int v = 0; v < V; ++v) r[v] = p[v];   /* p was the point mass on x (then u < 1 accepts: unreachable) */

        int best = -1;
        double best_score = -1.0;
        for (int v = 0; v < V; ++v) {
            if (r[v] <= 0.0) continue;
            const double e = -log(oracle_u_race(seed, step, b, v));
            const double s = (e == 0.0) ? INFINITY : r[v] / e;
            if (s > best_score) { best_score = s; best = v; }
        }
        if (best < 0) { free(p); free(r); return -1; }
        if (race_margin) {
            double margin = INFINITY;
            const double w_best = best_score;
            for (int v = 0; v < V; ++v) {
                if (v == best || r[v] <= 0.0) continue;
                const double e = -log(oracle_u_race(seed, step, b, v));
                const double s = (e == 0.0) ? INFINITY : r[v] / e;
                double g;
                if (isinf(best_score)) g = isinf(s) ? 0.0 : INFINITY;
                else g = (best_score - s) / (w_best + s);
                if (g < margin) margin = g;
            }
            race_margin[b] = margin;
        }

        accepted_len[b] = m;
        next_token[b] = best;
        if (out_tokens) {
            int32_t *row = out_tokens + (size_t)b * (ORACLE_K_MAX + 1);
            for (int i = 0; i <= ORACLE_K_MAX; ++i) row[i] = -1;
            for (int i = 0; i < m; ++i) row[i] = draft_tokens[d_row0 + i];
            row[m] = best;
        }
        if (counters) {
            counters[0] += k_b;
            counters[1] += m;
            counters[2] += (m + 1 < k_b) ? m + 1 : k_b;
            counters[3] += m + 1;
            counters[4] += near_ties;
            counters[5] += 1;
        }
    }
    free(p); free(r);
    return 0;
}

/* ------------------------------------------------------------------ */
/* The steps either side of the path (Section 5.1, "KV Cache of Bonus    */
/* Tokens"): before scoring, the K and V rows of this step's q_len        */
/* query positions are written into the paged cache at token positions   */
/* kv_len - q_len .. kv_len - 1; after acceptance the cache logically     */
/* keeps the first query position and the m accepted draft tokens, so    */
/* the rejected tail is dropped: new_kv_len = kv_len - (k - m).  The      */
/* draft model's own cache then lacks one token (the emitted one) after   */
/* a rejection, and two after full acceptance (the last draft token,      */
/* whose entry was never generated, and the bonus token).                 */
/*                                                                        */
/* Element (page, kvh, slot s, dim c) of one (page, KV head) sits at      */
/*   layout 0 (token-major)  s * d + c                                    */
/*   layout 1 (matrix-operand tiles, bf16, 16-token pages)                */
/*       K: (c / 8) * 128 + s * 8 + c % 8                                 */
/*       V: ((((c/32) * 4 + s/4) * 16 + c%16) * 2 + (c/16)%2) * 4 + s%4   */
/* in units of elements from the start of that (page, KV head), which     */
/* holds bs * d elements; (page, kvh) starts at (page*Hkv + kvh)*bs*d.    */
/* ------------------------------------------------------------------ */
static size_t oracle_kv_offset(int layout, int is_v, int bs, int d, int s, int c)
{
    if (layout == 0) return (size_t)s * d + c;
    (void)bs;
    if (!is_v) return (size_t)(c / 8) * 128 + (size_t)s * 8 + c % 8;
    return ((((size_t)(c / 32) * 4 + s / 4) * 16 + c % 16) * 2 + (c / 16) % 2) * 4 + s % 4;
}

int oracle_kv_append(int32_t B, int32_t Hkv, int32_t d, int32_t bs, int32_t num_blocks,
                     int32_t max_blocks, int32_t dtype, int32_t layout,
                     const void *new_k, const void *new_v, void *k_cache, void *v_cache,
                     const int32_t *block_table, const int32_t *kv_len, const int32_t *cu_q_len)
{
    if (layout != 0 && (layout != 1 || bs != 16 || dtype != 1 || d % 32 != 0)) return -1;
    const size_t esz = dtype == 1 ? 2 : 4;
    for (int b = 0; b < B; ++b) {
        const int q_len = cu_q_len[b + 1] - cu_q_len[b];
        if (q_len < 1 || kv_len[b] < q_len) return -1;
        for (int j = 0; j < q_len; ++j) {
            const int pos = kv_len[b] - q_len + j;
            if (pos / bs >= max_blocks) return -1;
            const int page = block_table[(size_t)b * max_blocks + pos / bs];
            if (page < 0 || page >= num_blocks) return -1;
            const int s = pos % bs;
            for (int h = 0; h < Hkv; ++h) {
                const size_t head = ((size_t)page * Hkv + h) * (size_t)bs * d;
                const size_t src = (((size_t)cu_q_len[b] + j) * Hkv + h) * d;
                for (int c = 0; c < d; ++c) {
                    memcpy((char *)k_cache + (head + oracle_kv_offset(layout, 0, bs, d, s, c)) * esz,
                           (const char *)new_k + (src + c) * esz, esz);
                    memcpy((char *)v_cache + (head + oracle_kv_offset(layout, 1, bs, d, s, c)) * esz,
                           (const char *)new_v + (src + c) * esz, esz);
                }
            }
        }
    }
    return 0;
}

void oracle_kv_after_accept(int32_t B, const int32_t *kv_len, const int32_t *cu_q_len,
                            const int32_t *accepted_len, int32_t *new_kv_len, int32_t *draft_next_len)
{
    for (int b = 0; b < B; ++b) {
        const int k = cu_q_len[b + 1] - cu_q_len[b] - 1;
        const int m = accepted_len[b];
        new_kv_len[b] = kv_len[b] - (k - m);
        draft_next_len[b] = (k > 0 && m == k) ? 2 : 1;
    }
}

/* Eq. 4: expected generated length per request, bonus token included. */
double oracle_expected_generated_len(double alpha, int32_t k)
{
    if (alpha == 1.0) return (double)(k + 1);
    return (1.0 - pow(alpha, (double)(k + 1))) / (1.0 - alpha);
}
