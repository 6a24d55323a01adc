/*
 * rollout_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, fp64 CPU statement of what the rollout hot path computes, used
 * only to check the GPU library and to be timed beside it as a baseline.  It
 * shares no source, header, table or helper with the GPU library and is never
 * called by it.
 *
 * The paper (Section 2.1, "RLHF Training") says which quantities exist in the
 * experience-generation step of PPO stage 3 -- the actor generates responses
 * token by token, and actor and reference inferences over the generated
 * sequences feed a penalty on policy deviation -- but prints no formula for
 * any of them.  Each function below is therefore the textbook definition
 * written out:
 *
 *   oracle_decode_attention   softmax(scale * q.K^T) V for one query token per
 *                             sequence over a paged key/value cache
 *   oracle_token_logprobs_kl  log-softmax of the actor logits gathered at the
 *                             sampled token, and KL(actor || reference) over
 *                             the whole vocabulary
 *   oracle_token_rewards      the reference model's log-probability of the
 *                             token and the KL-penalised per-token reward
 *   oracle_prefill_attention  causal attention of a block of new tokens per
 *                             sequence over the same paged cache
 *   oracle_sample_tokens      next-token sampling from softmax(logits / T) by
 *                             Gumbel-max over counter-based (Philox) uniforms
 *   oracle_sample_tokens_topk the same draw restricted to the k largest logits
 *                             of each row
 *
 * Inputs arrive in their storage precision (IEEE binary16, bfloat16 or
 * binary32) and are widened exactly to double; every sum, exponential and
 * logarithm is in double.  Loops run in logical order with a separate pass for
 * the maximum: no tiling, no online rescaling, no fused algebra.  OpenMP only
 * distributes independent outputs over host threads.
 *
 * Every function here is pinned by tests that do not go through this file's
 * own formulas (closed forms, brute force, library routines, invariants).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1, ORACLE_F32 = 2 };

/* IEEE 754 binary16 -> double, from the format definition: 1 sign bit, 5
 * exponent bits (bias 15), 10 fraction bits; exponent 0 is subnormal, 31 is
 * inf/NaN. */
static double widen_f16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(f | 0x400), e - 25);
    return sign ? -v : v;
}

/* bfloat16 is the upper half of a binary32. */
static double widen_bf16(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double load_elem(const void *base, size_t idx, int dtype)
{
    switch (dtype) {
    case ORACLE_F16:
        return widen_f16(((const uint16_t *)base)[idx]);
    case ORACLE_BF16:
        return widen_bf16(((const uint16_t *)base)[idx]);
    default:
        return (double)((const float *)base)[idx];
    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Single-token decode attention over a paged cache (Section 2.1: the actor
 * generating a response one token at a time; the definition is the standard
 * scaled dot-product attention with one query row).
 *
 *   q          [B][Hq][D]                      storage dtype
 *   k_pages    [n_pages][Hkv][P][D]            storage dtype, plain token-major pages
 *   v_pages    same shape
 *   page_table [B][max_pages]  physical page of logical page i of sequence b
 *   seq_lens   [B]             cached tokens, the current one included
 *   out        [B][Hq][D]      double
 *
 * Query head hq reads KV head hq / (Hq / Hkv).  Token j of sequence b lives at
 * page page_table[b][j / P], slot j % P.  For each (b, hq):
 *   s_j = scale * sum_d q_d K_jd ;  m = max_j s_j ;  w_j = exp(s_j - m)
 *   out = (sum_j w_j V_j) / (sum_j w_j)
 * A sequence of length 0 yields zeros.  weights_out, if not NULL, receives the
 * normalised weights w_j / sum w for (b, hq) in a [B][Hq][max_pages*P] array
 * (entries past the length are left untouched); tests use it for the
 * rows-sum-to-one pin.
 */
int oracle_decode_attention(const void *q, const void *k_pages, const void *v_pages,
                            const int32_t *page_table, const int32_t *seq_lens,
                            double *out, double *weights_out,
                            int B, int Hq, int Hkv, int D, int P, int max_pages,
                            int dtype, double scale)
{
    if (!q || !k_pages || !v_pages || !page_table || !seq_lens || !out)
        return -1;
    if (B < 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || P <= 0 || max_pages < 0 || Hq % Hkv)
        return -1;
    const int G = Hq / Hkv;
    const size_t page_elems = (size_t)Hkv * P * D;
    int bad = 0;

#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int hq = 0; hq < Hq; ++hq) {
            const int L = seq_lens[b];
            const int hkv = hq / G;
            double *o = out + ((size_t)b * Hq + hq) * D;
            for (int d = 0; d < D; ++d)
                o[d] = 0.0;
            if (L < 0 || L > max_pages * P) {
#pragma omp atomic write
                bad = 1;
                continue;
            }
            if (L == 0)
                continue;
            const size_t qbase = ((size_t)b * Hq + hq) * D;

            /* pass 1: the largest score */
            double m = -INFINITY;
            for (int j = 0; j < L; ++j) {
                const size_t page = (size_t)page_table[(size_t)b * max_pages + j / P];
                const size_t row = page * page_elems + ((size_t)hkv * P + j % P) * D;
                double s = 0.0;
                for (int d = 0; d < D; ++d)
                    s += load_elem(q, qbase + d, dtype) * load_elem(k_pages, row + d, dtype);
                s *= scale;
                if (s > m)
                    m = s;
            }
            /* pass 2: weights, their sum, and the weighted sum of value rows */
            double denom = 0.0;
            for (int j = 0; j < L; ++j) {
                const size_t page = (size_t)page_table[(size_t)b * max_pages + j / P];
                const size_t row = page * page_elems + ((size_t)hkv * P + j % P) * D;
                double s = 0.0;
                for (int d = 0; d < D; ++d)
                    s += load_elem(q, qbase + d, dtype) * load_elem(k_pages, row + d, dtype);
                s *= scale;
                const double w = exp(s - m);
                denom += w;
                for (int d = 0; d < D; ++d)
                    o[d] += w * load_elem(v_pages, row + d, dtype);
                if (weights_out)
                    weights_out[((size_t)b * Hq + hq) * ((size_t)max_pages * P) + j] = w;
            }
            for (int d = 0; d < D; ++d)
                o[d] /= denom;
            if (weights_out)
                for (int j = 0; j < L; ++j)
                    weights_out[((size_t)b * Hq + hq) * ((size_t)max_pages * P) + j] /= denom;
        }
    }
    return bad ? -1 : 0;
}

/*
 * Per-position log-probability of the sampled token under the actor, and the
 * KL divergence of the actor's next-token distribution from the reference
 * model's (Section 2.1: the reference model restrains the policy; the actor is
 * trained with its deviation from that policy penalised).  Natural logarithms.
 *
 *   actor, ref  [N][stride] rows, first V entries of each row used; storage dtype
 *   tokens      [N]
 *   logp, kl    [N] double
 *
 * For row i:
 *   lse_a = m_a + log sum_v exp(a_v - m_a),  m_a = max_v a_v     (same for r)
 *   logp  = a_tok - lse_a
 *   kl    = sum_v p_v * ((a_v - lse_a) - (r_v - lse_r)),  p_v = exp(a_v - lse_a)
 * The KL is summed term by term from its definition.  A term with p_v == 0
 * counts as 0 (so an actor logit of -inf never produces 0 * inf).
 * tokens[i] < 0 or >= V marks a padded position: logp = kl = 0 for it.
 */
/* One row of the definitions above: log p_actor(tok), log p_ref(tok), KL. */
static void score_row(const void *actor, const void *ref, size_t base, int V, int dtype, int32_t tok,
                      double *logp_actor, double *logp_ref, double *kl)
{
    double ma = -INFINITY, mr = -INFINITY;
    for (int v = 0; v < V; ++v) {
        const double a = load_elem(actor, base + v, dtype);
        const double r = load_elem(ref, base + v, dtype);
        if (a > ma)
            ma = a;
        if (r > mr)
            mr = r;
    }
    double sa = 0.0, sr = 0.0;
    for (int v = 0; v < V; ++v) {
        sa += exp(load_elem(actor, base + v, dtype) - ma);
        sr += exp(load_elem(ref, base + v, dtype) - mr);
    }
    const double lse_a = ma + log(sa);
    const double lse_r = mr + log(sr);

    double acc = 0.0;
    for (int v = 0; v < V; ++v) {
        const double la = load_elem(actor, base + v, dtype) - lse_a; /* log p_v */
        const double lr = load_elem(ref, base + v, dtype) - lse_r;   /* log q_v */
        const double p = exp(la);
        if (p > 0.0)
            acc += p * (la - lr);
    }
    *logp_actor = load_elem(actor, base + (size_t)tok, dtype) - lse_a;
    *logp_ref = load_elem(ref, base + (size_t)tok, dtype) - lse_r;
    *kl = acc;
}

int oracle_token_logprobs_kl(const void *actor, const void *ref, const int32_t *tokens,
                             double *logp, double *kl,
                             int64_t N, int V, int64_t stride, int dtype)
{
    if (!actor || !ref || !tokens || !logp || !kl || N < 0 || V <= 0)
        return -1;
    if (stride == 0)
        stride = V;
    if (stride < V)
        return -1;

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        const int32_t tok = tokens[i];
        if (tok < 0 || tok >= V) {
            logp[i] = 0.0;
            kl[i] = 0.0;
            continue;
        }
        const size_t base = (size_t)i * (size_t)stride;
        double unused;
        score_row(actor, ref, base, V, dtype, tok, &logp[i], &unused, &kl[i]);
    }
    return 0;
}

/*
 * Per-token reward shaping on top of the same row quantities (Section 2.1: the
 * reference model keeps the reward from diverging; the reward model's score is
 * the sequence return).  For row i with sampled token tok:
 *   ref_logp = r_tok - lse_r
 *   penalty  = KL(actor || ref) of the row            if sampled_penalty == 0
 *            = log p_actor(tok) - log p_ref(tok)      if sampled_penalty != 0
 *   reward   = -kl_coef * penalty + terminal[i]       (terminal may be NULL = 0)
 * Padded positions (tok outside [0, V)) get 0 in both outputs.
 */
int oracle_token_rewards(const void *actor, const void *ref, const int32_t *tokens,
                         const double *terminal, double *ref_logp, double *reward,
                         int64_t N, int V, int64_t stride, int dtype,
                         double kl_coef, int sampled_penalty)
{
    if (!actor || !ref || !tokens || !ref_logp || !reward || N < 0 || V <= 0)
        return -1;
    if (stride == 0)
        stride = V;
    if (stride < V)
        return -1;

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        const int32_t tok = tokens[i];
        if (tok < 0 || tok >= V) {
            ref_logp[i] = 0.0;
            reward[i] = 0.0;
            continue;
        }
        double lpa, lpr, kl;
        score_row(actor, ref, (size_t)i * (size_t)stride, V, dtype, tok, &lpa, &lpr, &kl);
        const double penalty = sampled_penalty ? lpa - lpr : kl;
        ref_logp[i] = lpr;
        reward[i] = -kl_coef * penalty + (terminal ? terminal[i] : 0.0);
    }
    return 0;
}

/*
 * Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
 * as 1, 2, 3", SC'11), written from the published definition: ten rounds of
 *   (c0,c1,c2,c3) <- (hi(M1*c2) ^ c1 ^ k0, lo(M1*c2), hi(M0*c0) ^ c3 ^ k1, lo(M0*c0))
 * with the key advanced by the Weyl constants between rounds.
 */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = M0 * c0, p1 = M1 * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The uniform on (0,1) that vocabulary entry v of row i gets: the top 23 bits of
 * word v%4 of Philox(counter = (v/4, i, offset low, offset high), key = seed),
 * centred in their cell.  23 bits because (k + 1/2) / 2^23 is then exact in
 * binary32, the precision the sampled decision is taken in on the GPU. */
static double sampling_uniform(int64_t row, int v, uint64_t seed, uint64_t offset)
{
    const uint32_t ctr[4] = {(uint32_t)(v / 4), (uint32_t)row, (uint32_t)offset, (uint32_t)(offset >> 32)};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t r[4];
    oracle_philox4x32_10(ctr, key, r);
    return ((double)(r[v % 4] >> 9) + 0.5) * (1.0 / 8388608.0);
}

/*
 * Sampling the next token from the actor's logits (Section 2.1, experience
 * generation by the actor).  With temperature T > 0 the token is drawn from
 * softmax(logits / T) by the Gumbel-max construction:
 *     token = argmax_v ( logits_v / T + G_v ),   G_v = -ln(-ln u_v)
 * with u_v the counter-based uniforms above; T == 0 means greedy argmax.  Ties
 * go to the lowest index.  logp = log softmax(logits / T)[token] (T = 1 for
 * greedy).  perturbed_out, if not NULL, receives every logits_v / T + G_v
 * ([N][V]), which lets a test accept any token whose perturbed score is within
 * rounding of the maximum.
 */
int oracle_sample_tokens(const void *logits, int32_t *tokens, double *logp, double *perturbed_out,
                         int64_t N, int V, int64_t stride, int dtype,
                         double temperature, uint64_t seed, uint64_t offset)
{
    if (!logits || !tokens || !logp || N < 0 || V <= 0 || temperature < 0.0)
        return -1;
    if (stride == 0)
        stride = V;
    if (stride < V)
        return -1;
    const double inv_t = temperature > 0.0 ? 1.0 / temperature : 1.0;

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        const size_t base = (size_t)i * (size_t)stride;
        int best = 0;
        double best_z = -INFINITY, m = -INFINITY;
        for (int v = 0; v < V; ++v) {
            const double y = load_elem(logits, base + v, dtype) * inv_t;
            double z = y;
            if (temperature > 0.0)
                z += -log(-log(sampling_uniform(i, v, seed, offset)));
            if (perturbed_out)
                perturbed_out[(size_t)i * V + v] = z;
            if (z > best_z) {
                best_z = z;
                best = v;
            }
            if (y > m)
                m = y;
        }
        double s = 0.0;
        for (int v = 0; v < V; ++v)
            s += exp(load_elem(logits, base + v, dtype) * inv_t - m);
        tokens[i] = best;
        logp[i] = load_elem(logits, base + (size_t)best, dtype) * inv_t - (m + log(s));
    }
    return 0;
}

static int descending(const void *a, const void *b)
{
    const double x = *(const double *)a, y = *(const double *)b;
    return (x < y) - (x > y);
}

/*
 * Top-k sampling: the draw of oracle_sample_tokens restricted to the k largest
 * logits of the row.  The paper only says that the actor generates responses
 * (Section 2.1); this is the usual filter of generation code: with tau the
 * k-th largest logit of the row (multiplicity counted), every entry below tau
 * is removed, every entry equal to tau stays (so more than k entries survive
 * when the k-th value is tied), and the token is drawn from softmax(logits / T)
 * over the survivors with the SAME noise per vocabulary entry as the
 * unrestricted draw:
 *     C = { v : logits_v >= tau },  token = argmax_{v in C} ( logits_v / T + G_v )
 * T == 0 is greedy.  logp = log of the survivors' renormalised softmax at the
 * token.  k >= V keeps everything.  threshold_out, if not NULL, receives tau;
 * count_out the number of survivors; perturbed_out as in oracle_sample_tokens,
 * with -inf for removed entries.
 */
int oracle_sample_tokens_topk(const void *logits, int32_t *tokens, double *logp, double *perturbed_out,
                              double *threshold_out, int32_t *count_out, int64_t N, int V, int64_t stride,
                              int dtype, double temperature, int top_k, uint64_t seed, uint64_t offset)
{
    if (!logits || !tokens || !logp || N < 0 || V <= 0 || temperature < 0.0 || top_k < 1)
        return -1;
    if (stride == 0)
        stride = V;
    if (stride < V)
        return -1;
    const double inv_t = temperature > 0.0 ? 1.0 / temperature : 1.0;
    const int k = top_k < V ? top_k : V;
    int failed = 0;

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        const size_t base = (size_t)i * (size_t)stride;
        double *sorted = (double *)malloc((size_t)V * sizeof(double));
        if (!sorted) {
#pragma omp atomic write
            failed = 1;
            continue;
        }
        for (int v = 0; v < V; ++v)
            sorted[v] = load_elem(logits, base + v, dtype);
        qsort(sorted, (size_t)V, sizeof(double), descending);
        const double tau = sorted[k - 1];
        free(sorted);

        int best = -1, count = 0;
        double best_z = -INFINITY, m = -INFINITY;
        for (int v = 0; v < V; ++v) {
            const double a = load_elem(logits, base + v, dtype);
            const int kept = a >= tau;
            double z = -INFINITY;
            if (kept) {
                const double y = a * inv_t;
                z = y;
                if (temperature > 0.0)
                    z += -log(-log(sampling_uniform(i, v, seed, offset)));
                ++count;
                if (best < 0 || z > best_z) {
                    best_z = z;
                    best = v;
                }
                if (y > m)
                    m = y;
            }
            if (perturbed_out)
                perturbed_out[(size_t)i * V + v] = z;
        }
        double s = 0.0;
        for (int v = 0; v < V; ++v) {
            const double a = load_elem(logits, base + v, dtype);
            if (a >= tau)
                s += exp(a * inv_t - m);
        }
        tokens[i] = best;
        logp[i] = load_elem(logits, base + (size_t)best, dtype) * inv_t - (m + log(s));
        if (threshold_out)
            threshold_out[i] = tau;
        if (count_out)
            count_out[i] = count;
    }
    return failed ? -2 : 0;
}

/*
 * Causal attention for a block of new tokens per sequence ("prefill": the
 * prompt, or a chunk of it, entering the cache before generation starts;
 * Section 2.1, generation by the actor starts from the prompts).  The keys and
 * values of the new tokens are already in the paged cache.  Sequence b brings
 * n_b = cu_q[b+1] - cu_q[b] query rows; they are the LAST n_b tokens of its
 * L_b = seq_lens[b] cached tokens, so query row i sits at logical position
 * p = L_b - n_b + i and attends to keys 0 .. p (itself included):
 *   s_j = scale * <q_i, K_j>,  out_i = sum_{j<=p} softmax(s)_j V_j .
 *
 *   q    [cu_q[B]][Hq][D] packed rows, storage dtype
 *   out  [cu_q[B]][Hq][D] double
 * Pages, page table and head mapping as in oracle_decode_attention.
 */
int oracle_prefill_attention(const void *q, const int32_t *cu_q, const void *k_pages, const void *v_pages,
                             const int32_t *page_table, const int32_t *seq_lens, double *out,
                             int B, int Hq, int Hkv, int D, int P, int max_pages, int dtype, double scale)
{
    if (!q || !cu_q || !k_pages || !v_pages || !page_table || !seq_lens || !out)
        return -1;
    if (B < 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || P <= 0 || max_pages < 0 || Hq % Hkv)
        return -1;
    const int G = Hq / Hkv;
    const size_t page_elems = (size_t)Hkv * P * D;
    for (int b = 0; b < B; ++b) {
        const int n = cu_q[b + 1] - cu_q[b];
        if (n < 0 || n > seq_lens[b] || seq_lens[b] > max_pages * P)
            return -1;
    }
    for (int b = 0; b < B; ++b) {
        const int n = cu_q[b + 1] - cu_q[b];
        const int first = seq_lens[b] - n;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
        for (int i = 0; i < n; ++i) {
            for (int hq = 0; hq < Hq; ++hq) {
                const int p = first + i;          /* last key this query may see */
                const int hkv = hq / G;
                const size_t qbase = (((size_t)cu_q[b] + i) * Hq + hq) * D;
                double *o = out + qbase;
                double m = -INFINITY;
                for (int j = 0; j <= p; ++j) {
                    const size_t page = (size_t)page_table[(size_t)b * max_pages + j / P];
                    const size_t row = page * page_elems + ((size_t)hkv * P + j % P) * D;
                    double s = 0.0;
                    for (int d = 0; d < D; ++d)
                        s += load_elem(q, qbase + d, dtype) * load_elem(k_pages, row + d, dtype);
                    s *= scale;
                    if (s > m)
                        m = s;
                }
                double denom = 0.0;
                for (int d = 0; d < D; ++d)
                    o[d] = 0.0;
                for (int j = 0; j <= p; ++j) {
                    const size_t page = (size_t)page_table[(size_t)b * max_pages + j / P];
                    const size_t row = page * page_elems + ((size_t)hkv * P + j % P) * D;
                    double s = 0.0;
                    for (int d = 0; d < D; ++d)
                        s += load_elem(q, qbase + d, dtype) * load_elem(k_pages, row + d, dtype);
                    const double w = exp(s * scale - m);
                    denom += w;
                    for (int d = 0; d < D; ++d)
                        o[d] += w * load_elem(v_pages, row + d, dtype);
                }
                for (int d = 0; d < D; ++d)
                    o[d] /= denom;
            }
        }
    }
    return 0;
}
