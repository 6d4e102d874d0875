/*
 * CPU oracle for the per-token core of the UloRL objective (arxiv 2507.19766).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of what
 * the GPU library computes.  It shares no code, header, table or helper with the
 * HIP path and must never be linked, imported or called by the product path; only
 * tests, the smoke check and the benchmark's reported CPU baseline use it.
 *
 * Everything is evaluated in double precision, directly from the definitions:
 *   - softmax of the policy over the vocabulary (ratio numerator of Eq. 6; the
 *     p_t^j inside the DMMPT objective of Sec. 3.2.2),
 *   - per-token entropy, the inner vocabulary sum of the H-bar definition in
 *     Sec. 3.2.2 with the sign of an entropy (H = -sum p ln p),
 *   - SAIS / POIS importance ratio (Sec. 3.1.2, Eq. "sais" and the POIS paragraph),
 *   - the clipped surrogate (Eq. 1 / Eq. 7 with eps_low, eps_high),
 *   - the MPT set (Eq. "MPTS", Sec. 3.2.1) and the dynamic mask I_msk with its
 *     per-response entropy gate (Sec. 3.2.2),
 *   - the token-mean reduction 1 / sum_i |o_i| of the DMMPT objective,
 *   - the gradient of loss = -J with respect to the logits (chain rule; the mask
 *     is a constant, the paper adds no extra optimisation objective),
 * and, around that core: the group advantages (Eq. 4, the sampling constraint of
 * Eq. 7, the overlong rule of Sec. 3.5), per-segment diagnostics, and the pool
 * update of the segment-rollout loop (Algorithm 1, Sec. 3.1.1).
 *
 * Every function is pinned by tests to something other than itself (closed forms,
 * hand-worked cases, invariants, autograd / finite differences, conservation over
 * whole runs); none of the paper's printed numbers constrains the loss itself, so
 * parity against published values is unpinned.
 *
 * No blocking, no online rescaling, no fusion: each quantity is a loop over its
 * definition.  OpenMP is used over independent rows only; all sums that cross
 * rows (per-response entropy, the loss) are sequential in index order.
 *
 * Storage codes for logits: 0 = float32, 1 = bfloat16 (raw uint16), 2 = float64.
 * Both narrow types convert to double exactly, so the oracle consumes exactly
 * the values the GPU sees.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F64 = 2 };
enum { ORC_IS_SAIS = 0, ORC_IS_POIS = 1 };
enum { ORC_GATE_PER_RESPONSE = 0, ORC_GATE_GLOBAL = 1, ORC_GATE_ALWAYS = 2, ORC_GATE_NEVER = 3 };

static double bf16_bits_to_double(uint16_t h)
{
    uint32_t w = ((uint32_t)h) << 16; /* bfloat16 is the upper half of a binary32 */
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

static double logit_at(const void *base, int storage, int64_t idx)
{
    switch (storage) {
    case ORC_F32: return (double)((const float *)base)[idx];
    case ORC_BF16: return bf16_bits_to_double(((const uint16_t *)base)[idx]);
    default: return ((const double *)base)[idx];
    }
}

/*
 * Softmax statistics of each row (independent rows).
 *   lse[t]  = ln sum_j exp(z[t,j])                 (evaluated with the usual max shift)
 *   logp[t] = z[t, y[t]] - lse[t]                  log pi_theta(o_t | .)      (Eq. 6 numerator)
 *   H[t]    = - sum_j q_j ln q_j,  q_j = exp(z[t,j] - lse[t]),  ln q_j = z[t,j] - lse[t]
 *                                                  (Sec. 3.2.2, inner sum of H-bar; natural log)
 * Returns 0, or -1 on a token id outside [0, V).
 */
int ulorl_oracle_row_stats(const void *logits, int storage, int64_t n_rows, int64_t V,
                           int64_t row_stride, const int32_t *token_ids, double *lse,
                           double *logp, double *entropy)
{
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t t = 0; t < n_rows; ++t) {
        const int64_t off = t * row_stride;
        double m = -INFINITY;
        for (int64_t j = 0; j < V; ++j) {
            double z = logit_at(logits, storage, off + j);
            if (z > m) m = z;
        }
        double S = 0.0;
        for (int64_t j = 0; j < V; ++j) S += exp(logit_at(logits, storage, off + j) - m);
        const double l = m + log(S);
        double h = 0.0;
        for (int64_t j = 0; j < V; ++j) {
            const double lnq = logit_at(logits, storage, off + j) - l;
            const double q = exp(lnq);
            if (q > 0.0) h -= q * lnq;
        }
        lse[t] = l;
        entropy[t] = h;
        const int64_t y = token_ids[t];
        if (y < 0 || y >= V) {
            bad |= 1;
            logp[t] = NAN;
        } else {
            logp[t] = logit_at(logits, storage, off + y) - l;
        }
    }
    return bad ? -1 : 0;
}

/*
 * Everything that is O(1) per token, given the per-row log-prob and entropy.
 *
 * Per response i (cu[i] <= t < cu[i+1]):
 *   Hbar[i] = mean_t H[t]  over ALL tokens of the response          (Sec. 3.2.2)
 *   gate[i] = Hbar[i] < sigma (strict)                               (Sec. 3.2.2, I_msk case 1)
 *     gate modes: per response (the equation), global (token-mean entropy of the whole
 *     call, the reading of the prose, which speaks of the model's entropy as a whole), always (static masking
 *     experiment of Sec. 3.2.1), never (plain DAPO objective, Eq. 7).
 * Per token:
 *   seg[t]  = f(t): explicit id if given, else offset-in-response div seg_len   (Sec. 3.1.2)
 *   MPT     = (A[t] > 0) and (p[t] >= tau), p = exp(logp)            (Eq. MPTS; reward 1 <=> A > 0)
 *   I[t]    = gate and MPT
 *   r       = exp(logp - old_logp) [SAIS]  |  1 [POIS, d r / d logp = 1]
 *   s       = min(r A, clip(r, 1-eps_low, 1+eps_high) A)
 *   loss    = -(1/D) sum_t (1 - I[t]) s[t],  D = sum_i |o_i| = N unless overridden
 *   g[t]    = d loss / d logp[t] = -(1/D) (1 - I[t]) [r A <= clip(r) A] r A
 *
 * counters[0] = number of masked tokens (I = 1)
 * counters[1] = number of tokens whose clipped branch is the strict minimum (no gradient)
 * counters[2] = number of tokens with A > 0
 * Any output pointer except loss may be NULL.  Returns 0, or -2 on malformed cu_seqlens.
 */
int ulorl_oracle_token_terms(int64_t N, const double *logp, const double *entropy,
                             const int32_t *cu_seqlens, int32_t R, const int32_t *segment_ids,
                             int32_t seg_len, const double *old_logp, const double *advantages,
                             double eps_low, double eps_high, double tau, double sigma,
                             int is_mode, int gate_mode, double denominator,
                             double *loss, double *resp_entropy, uint8_t *resp_gate,
                             int32_t *seg_out, uint8_t *mask, double *ratio, double *surrogate,
                             double *gcoef, int64_t *counters)
{
    if (cu_seqlens[0] != 0 || cu_seqlens[R] != N) return -2;
    for (int32_t i = 0; i < R; ++i)
        if (cu_seqlens[i + 1] < cu_seqlens[i]) return -2;

    const double D = denominator > 0.0 ? denominator : (double)N;

    /* token-mean entropy over the whole call, for the global gate */
    double Hall = 0.0;
    for (int64_t t = 0; t < N; ++t) Hall += entropy[t];
    const double Hglobal = N > 0 ? Hall / (double)N : 0.0;

    double acc = 0.0;
    int64_t n_masked = 0, n_clipped = 0, n_pos = 0;
    for (int32_t i = 0; i < R; ++i) {
        const int64_t b = cu_seqlens[i], e = cu_seqlens[i + 1];
        double hs = 0.0;
        for (int64_t t = b; t < e; ++t) hs += entropy[t];
        const double hbar = e > b ? hs / (double)(e - b) : 0.0;
        int gate;
        switch (gate_mode) {
        case ORC_GATE_PER_RESPONSE: gate = (e > b) && (hbar < sigma); break;
        case ORC_GATE_GLOBAL: gate = Hglobal < sigma; break;
        case ORC_GATE_ALWAYS: gate = 1; break;
        default: gate = 0; break;
        }
        if (resp_entropy) resp_entropy[i] = hbar;
        if (resp_gate) resp_gate[i] = (uint8_t)gate;

        for (int64_t t = b; t < e; ++t) {
            const int32_t seg = segment_ids ? segment_ids[t]
                                            : (seg_len > 0 ? (int32_t)((t - b) / seg_len) : 0);
            const double A = advantages[t];
            const double p = exp(logp[t]);
            const int positive = A > 0.0;
            const int mpt = positive && (p >= tau);
            const int I = gate && mpt;
            const double r = (is_mode == ORC_IS_POIS) ? 1.0 : exp(logp[t] - old_logp[t]);
            double c = r;
            if (c < 1.0 - eps_low) c = 1.0 - eps_low;
            if (c > 1.0 + eps_high) c = 1.0 + eps_high;
            const double u = r * A, v = c * A;
            const int active = u <= v; /* the unclipped branch attains the min: gradient flows */
            const double s = active ? u : v;
            const double keep = I ? 0.0 : 1.0;
            acc += keep * s;
            if (seg_out) seg_out[t] = seg;
            if (mask) mask[t] = (uint8_t)I;
            if (ratio) ratio[t] = r;
            if (surrogate) surrogate[t] = s;
            if (gcoef) gcoef[t] = I ? 0.0 : (active ? -(r * A) / D : 0.0);
            n_masked += I;
            n_clipped += !active;
            n_pos += positive;
        }
    }
    *loss = -acc / D;
    if (counters) {
        counters[0] = n_masked;
        counters[1] = n_clipped;
        counters[2] = n_pos;
    }
    return 0;
}

/*
 * Gradient of the loss with respect to the logits of selected rows:
 *   dz[k, j] = grad_out * g[t] * ( [j == y[t]] - q_{t,j} ),  t = rows[k] (or k if rows == NULL),
 *   q_{t,j} = exp(z[t,j] - lse[t]).
 * Output is dense double [n_sel, V].
 */
int ulorl_oracle_dlogits(const void *logits, int storage, int64_t V, int64_t row_stride,
                         const int32_t *token_ids, const double *lse, const double *gcoef,
                         double grad_out, const int64_t *rows, int64_t n_sel, double *dz)
{
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < n_sel; ++k) {
        const int64_t t = rows ? rows[k] : k;
        const int64_t off = t * row_stride;
        const double w = grad_out * gcoef[t];
        const int64_t y = token_ids[t];
        double *out = dz + k * V;
        for (int64_t j = 0; j < V; ++j) {
            const double q = exp(logit_at(logits, storage, off + j) - lse[t]);
            out[j] = w * ((j == y ? 1.0 : 0.0) - q);
        }
    }
    return 0;
}

/* Number of OpenMP threads the row loops will use (reported by the CPU baseline). */
int ulorl_oracle_threads(void)
{
    int n = 1;
#pragma omp parallel
    {
#pragma omp single
#ifdef _OPENMP
        n = omp_get_num_threads();
#endif
    }
    return n;
}

/*
 * Advantage preparation, the step just before the token loss (Sec. 2.2 Eq. 4, Eq. 7 constraint,
 * Sec. 3.3, Sec. 3.5).  Responses come in consecutive groups of G (one group per prompt).
 *   effective reward   r_i = truncated_i ? 0 : reward_i          overlong samples count as wrong
 *   group statistics   mean_g, std_g over the G effective rewards (population std, or the
 *                      unbiased one if `unbiased`)
 *   dynamic sampling   a group is kept iff 0 < #{r_i > 0} < G      (Eq. 7 constraint)
 *   advantage          A_i = keep_g ? (r_i - mean_g) / (std_g + eps) : 0      (Eq. 4)
 *   broadcast          token_adv[t] = A_i for every token t of response i
 * kept_tokens = number of tokens in kept groups (the 1 / sum |o_i| of the filtered batch).
 * Returns 0, -2 on malformed cu_seqlens, -3 if R is not a multiple of G.
 */
int ulorl_oracle_advantages(int32_t R, int32_t G, const double *rewards, const uint8_t *truncated,
                            const int32_t *cu_seqlens, int64_t N, double eps, int unbiased,
                            double *resp_adv, uint8_t *group_keep, double *token_adv,
                            int64_t *kept_tokens)
{
    if (G <= 0 || R % G != 0) return -3;
    if (cu_seqlens[0] != 0 || cu_seqlens[R] != N) return -2;
    for (int32_t i = 0; i < R; ++i)
        if (cu_seqlens[i + 1] < cu_seqlens[i]) return -2;
    int64_t kept = 0;
    for (int32_t g0 = 0; g0 < R; g0 += G) {
        double sum = 0.0;
        int correct = 0;
        for (int32_t i = g0; i < g0 + G; ++i) {
            const double r = (truncated && truncated[i]) ? 0.0 : rewards[i];
            sum += r;
            correct += r > 0.0;
        }
        const double mean = sum / G;
        double ss = 0.0;
        for (int32_t i = g0; i < g0 + G; ++i) {
            const double r = (truncated && truncated[i]) ? 0.0 : rewards[i];
            ss += (r - mean) * (r - mean);
        }
        const double denom = unbiased ? (G > 1 ? G - 1 : 1) : G;
        const double sd = sqrt(ss / denom);
        const int keep = correct > 0 && correct < G;
        if (group_keep) group_keep[g0 / G] = (uint8_t)keep;
        for (int32_t i = g0; i < g0 + G; ++i) {
            const double r = (truncated && truncated[i]) ? 0.0 : rewards[i];
            const double a = keep ? (r - mean) / (sd + eps) : 0.0;
            if (resp_adv) resp_adv[i] = a;
            for (int64_t t = cu_seqlens[i]; t < cu_seqlens[i + 1]; ++t) token_adv[t] = a;
            if (keep) kept += cu_seqlens[i + 1] - cu_seqlens[i];
        }
    }
    if (kept_tokens) *kept_tokens = kept;
    return 0;
}

/*
 * Training-dynamics diagnostics per segment id (the quantities behind the paper's SAIS / POIS
 * comparison, Sec. 3.1.2, and its entropy curves, Sec. 3.2): for every segment id k < K
 *   count[k]      tokens whose segment id is k
 *   ratio_sum[k]  sum of importance ratios          ratio_max[k]  largest ratio
 *   clipped[k]    tokens on the clipped, gradient-free branch of the min
 *   kl_sum[k]     sum of (old_logp - logp): the sampled estimate of KL(pi_old || pi_theta)
 *   ent_sum[k]    sum of token entropies            masked[k]     tokens removed by the MPT mask
 * Tokens with a segment id outside [0, K) are counted in *out_of_range and otherwise ignored.
 */
int ulorl_oracle_segment_diagnostics(int64_t N, int32_t K, const int32_t *seg, const double *ratio,
                                     const double *logp, const double *old_logp, const double *entropy,
                                     const uint8_t *mask, const double *advantages, double eps_low,
                                     double eps_high, int64_t *count, double *ratio_sum,
                                     double *ratio_max, int64_t *clipped, double *kl_sum,
                                     double *ent_sum, int64_t *masked, int64_t *out_of_range)
{
    for (int32_t k = 0; k < K; ++k) {
        count[k] = 0; ratio_sum[k] = 0.0; ratio_max[k] = 0.0; clipped[k] = 0;
        kl_sum[k] = 0.0; ent_sum[k] = 0.0; masked[k] = 0;
    }
    int64_t oor = 0;
    for (int64_t t = 0; t < N; ++t) {
        const int32_t k = seg[t];
        if (k < 0 || k >= K) { ++oor; continue; }
        const double r = ratio[t], A = advantages[t];
        double c = r;
        if (c < 1.0 - eps_low) c = 1.0 - eps_low;
        if (c > 1.0 + eps_high) c = 1.0 + eps_high;
        count[k] += 1;
        ratio_sum[k] += r;
        if (r > ratio_max[k]) ratio_max[k] = r;
        clipped[k] += !(r * A <= c * A);
        kl_sum[k] += old_logp ? old_logp[t] - logp[t] : 0.0;
        ent_sum[k] += entropy[t];
        masked[k] += mask[t] != 0;
    }
    *out_of_range = oor;
    return 0;
}

/*
 * One rollout step of the segment-rollout loop (Algorithm 1, Sec. 3.1.1).  Every sample in
 * flight (carried over from the unfinished pool, or a new prompt with prev_len = 0) has just
 * been decoded for at most seg_len further tokens.  The three ways a decode can end decide
 * where the sample goes:
 *   the end-of-sequence token was produced          -> state 1, experience pool
 *   the global maximum length max_len is reached     -> state 2 (truncated), experience pool
 *   the segment is full and max_len is not reached   -> state 0, unfinished pool
 * An end-of-sequence token that lands exactly on the global maximum counts as a normal end.
 * A step that stops short of seg_len without either reason, or decodes more than the segment or
 * the global maximum allow, is inconsistent: it is reported in counts[4] and the sample is kept
 * in the unfinished pool (lengths clamped into range).
 *
 * Outputs (sample order is preserved inside each pool):
 *   state[B], total_len[B] = prev_len + new_len, segments[B] = segments the sample spans so far
 *   unfinished_idx[0 .. counts[0])   indices of the samples to decode further
 *   experience_idx[0 .. counts[1])   indices of the samples that go to training
 *   exp_cu_seqlens[0 .. counts[1]]   prefix sums of their total lengths (packed-batch boundaries)
 *   exp_truncated[0 .. counts[1])    1 where the sample was cut at max_len (its reward counts as 0, Sec. 3.5)
 *   counts[5]: unfinished, experience, truncated, experience tokens, inconsistent samples
 * Returns non-zero for seg_len <= 0, max_len <= 0 or B < 0.
 */
int ulorl_oracle_pool_step(int32_t B, const int32_t *prev_len, const int32_t *new_len,
                           const uint8_t *hit_eos, int32_t seg_len, int32_t max_len, uint8_t *state,
                           int32_t *total_len, int32_t *segments, int32_t *unfinished_idx,
                           int32_t *experience_idx, int64_t *exp_cu_seqlens, uint8_t *exp_truncated,
                           int64_t *counts)
{
    if (B < 0 || seg_len <= 0 || max_len <= 0) return 1;
    int64_t n_unf = 0, n_exp = 0, n_trunc = 0, tokens = 0, n_bad = 0;
    exp_cu_seqlens[0] = 0;
    for (int32_t i = 0; i < B; ++i) {
        int64_t p = prev_len[i], n = new_len[i];
        int bad = 0;
        if (p < 0 || p >= max_len) { bad = 1; p = p < 0 ? 0 : max_len - 1; }
        int64_t room = max_len - p;
        if (room > seg_len) room = seg_len;
        if (n < 0 || n > room) { bad = 1; n = n < 0 ? 0 : room; }
        const int64_t t = p + n;
        const int eos = hit_eos[i] != 0 && n > 0;
        if (hit_eos[i] != 0 && n == 0) bad = 1;             /* an end token is itself a decoded token */
        int st;
        if (bad) st = 0;
        else if (eos) st = 1;
        else if (t >= max_len) st = 2;
        else if (n == seg_len) st = 0;
        else { st = 0; bad = 1; }                             /* stopped early for no reason */
        state[i] = (uint8_t)st;
        total_len[i] = (int32_t)t;
        segments[i] = (int32_t)(t == 0 ? 0 : (t + seg_len - 1) / seg_len);
        n_bad += bad;
        if (st == 0) {
            unfinished_idx[n_unf++] = i;
        } else {
            experience_idx[n_exp] = i;
            exp_truncated[n_exp] = (uint8_t)(st == 2);
            tokens += t;
            exp_cu_seqlens[n_exp + 1] = tokens;
            n_trunc += st == 2;
            ++n_exp;
        }
    }
    counts[0] = n_unf; counts[1] = n_exp; counts[2] = n_trunc; counts[3] = tokens; counts[4] = n_bad;
    return 0;
}
