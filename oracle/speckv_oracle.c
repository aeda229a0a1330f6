/*
 * speckv_oracle.c -- slow, plain, float64 CPU oracle for the speculative-decoding
 * verify-and-select stage of SpecKV.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It exists so that the HIP library can be
 * checked against something that is obviously right.  Only tests/, the smoke
 * check and the benchmark's cpu_baseline leg may load it.  It shares no code,
 * header, table or helper with the HIP path.
 *
 * What it computes, and where the paper defines it:
 *   - per-position draft entropy  H(q_i) = -sum_v q_i(v) log2 q_i(v)   (Section 4.2, first bullet)
 *   - per-position draft confidence  max_v q_i(v)                      (Section 4.2, second bullet)
 *   - step aggregates: mean entropy, mean confidence, max entropy,
 *     min confidence over the gamma drafted positions                  (Section 4.2, all four bullets)
 *   - verification position by position until the first rejection,
 *     k accepted tokens plus one more token from the target, rate k/gamma (Section 3.1)
 *     with the lossless accept test min(1, p/q) of the speculative-sampling
 *     works the paper builds on (Section 2.1): accept iff u*q(t) < p(t);
 *     on rejection draw from max(0, p-q) normalised, after gamma accepts
 *     draw the bonus token from the last target distribution;
 *     and the greedy rule of Section 3.1 itself (target top-1 must equal the drafted token)
 *   - controller: context vector -> one hidden layer of ReLU units -> one
 *     predicted acceptance rate per candidate gamma in {2,4,6,8};
 *     score = rate*gamma + 1 (Eq. 1); pick the argmax (Section 4.3); also as f([x, gamma])
 *     evaluated per candidate and without a hidden layer (Section 4.3, Table 3)
 *   - the draft side's token proposal that precedes a step (Section 3.1): inverse CDF of q_i
 *
 * Notation: q = draft distribution, p = target distribution (the paper's
 * Section 4.2 writes the draft distribution as p_i; here p is always the target).
 * Positions are 0-based: draft rows i = 0..gamma-1, target rows i = 0..gamma.
 *
 * Everything is evaluated in double precision, in vocabulary order, one
 * sequence after the other.  "#pragma omp parallel for" over sequences only
 * changes which core handles a sequence, never the arithmetic inside one.
 *
 * Random numbers: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11), own
 * implementation, key = (seed low word, seed high word),
 * counter = (global sequence index, position, step, stream).
 *   word 0 of block (b, i, step, 0) -> accept uniform  u  = (w0 >> 8) * 2^-24
 *   word 1 of block (b, n, step, 0) -> resample uniform u' =  w1 * 2^-32
 *   word 0 of block (b, i, step, 1) -> proposal uniform        w0 * 2^-32
 *
 * Parity pins for every function here live in tests/test_oracle_*.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define SKO_F32 0
#define SKO_F16 1
#define SKO_BF16 2

#define SKO_FLAG_NONFINITE 1u  /* a row of the sequence holds NaN or +inf, or no finite logit */
#define SKO_FLAG_BAD_TOKEN 2u  /* a drafted token id of the sequence is outside [0, V) */
#define SKO_FLAG_FALLBACK 4u   /* residual mass below SKO_RESID_FLOOR or not finite: drew from p_n instead */

/* The residual max(0, p_n - q_n) has mass R = total-variation distance of p_n and q_n.  The paper
 * (Section 3.1) only says the rejected position receives the target's correction; the lossless
 * scheme of Section 2.1's references normalises the residual by R and is silent about R = 0, which
 * happens when a position is rejected although p_n = q_n (a drafted token that neither row can
 * emit).  Reading taken: when R < 1e-6 the two distributions are the same to within 1e-6 and the
 * correction is drawn from p_n itself.  A threshold rather than "R == 0" so that the decision does
 * not hang on rounding noise; the output law moves by less than P(reject) * R < 1e-6. */
#define SKO_RESID_FLOOR 1e-6

static const int SKO_GAMMAS[4] = {2, 4, 6, 8}; /* candidate set, Section 4.1 / 4.3 */

/* ------------------------------------------------------------------------- */
/* Philox4x32-10                                                              */
/* ------------------------------------------------------------------------- */
void sko_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t prod1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(prod0 >> 32), lo0 = (uint32_t)prod0;
        uint32_t hi1 = (uint32_t)(prod1 >> 32), lo1 = (uint32_t)prod1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

static void step_block(uint64_t seed, uint32_t seq, uint32_t pos, uint32_t step, uint32_t w[4])
{
    uint32_t ctr[4] = {seq, pos, step, 0u};
    uint32_t key[2] = {(uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32)};
    sko_philox4x32_10(ctr, key, w);
}

/* ------------------------------------------------------------------------- */
/* Stored logit -> double, exactly                                            */
/* ------------------------------------------------------------------------- */
static double half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int mant = h & 0x3ff;
    double v;
    if (expo == 0)
        v = ldexp((double)mant, -24); /* zero and subnormals */
    else if (expo == 31)
        v = mant ? NAN : INFINITY;
    else
        v = ldexp((double)(mant | 0x400), expo - 25);
    return sign ? -v : v;
}

static double bf16_to_double(uint16_t h)
{
    uint32_t bits = (uint32_t)h << 16; /* bfloat16 is the top half of a binary32 */
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

double sko_load_logit(const void *base, int dtype, int64_t index)
{
    switch (dtype) {
    case SKO_F32: return (double)((const float *)base)[index];
    case SKO_F16: return half_to_double(((const uint16_t *)base)[index]);
    case SKO_BF16: return bf16_to_double(((const uint16_t *)base)[index]);
    default: return NAN;
    }
}

/* ------------------------------------------------------------------------- */
/* Softmax of one vocabulary row, its entropy (bits), max prob, argmax        */
/* ------------------------------------------------------------------------- */
/* prob[V] receives softmax(x).  Returns 1 if the row holds NaN or +inf.      */
int sko_row_softmax(const void *logits, int dtype, int64_t row, int V, double *prob,
                    double *H_bits, double *conf, int32_t *argmax)
{
    const int64_t base = row * (int64_t)V;
    int bad = 0;
    double m = -INFINITY;
    int32_t am = 0;
    for (int v = 0; v < V; ++v) {
        double x = sko_load_logit(logits, dtype, base + v);
        if (isnan(x) || x == INFINITY) bad = 1;
        if (x > m) { m = x; am = v; } /* strict: lowest index wins ties */
    }
    double S = 0.0;
    for (int v = 0; v < V; ++v) {
        double x = sko_load_logit(logits, dtype, base + v);
        prob[v] = exp(x - m); /* exp(-inf) = 0: a masked token has probability 0 */
        S += prob[v];
    }
    double H = 0.0, c = 0.0;
    for (int v = 0; v < V; ++v) {
        prob[v] /= S;
        if (prob[v] > 0.0) H -= prob[v] * log2(prob[v]); /* 0 log 0 = 0 */
        if (prob[v] > c) c = prob[v];
    }
    if (H_bits) *H_bits = H;
    if (conf) *conf = c;
    if (argmax) *argmax = am;
    return bad;
}

/* ------------------------------------------------------------------------- */
/* Signals of every draft row and the four step aggregates (Section 4.2)     */
/* ------------------------------------------------------------------------- */
/* draft: packed rows, sequence b owns rows row_off[b] .. row_off[b]+gamma[b]-1.
 * H, conf, argmax: one entry per draft row.  agg: [B][4] = mean H, mean c, max H, min c. */
int sko_signals(const void *draft, int dtype, int B, int V, const int32_t *gamma,
                const int64_t *row_off, double *H, double *conf, int32_t *argmax, double *agg)
{
    int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        double *prob = (double *)malloc(sizeof(double) * (size_t)V);
        if (!prob) {
#pragma omp atomic write
            status = 1;
            continue;
        }
        const int g = gamma[b];
        double sumH = 0.0, sumC = 0.0, maxH = -INFINITY, minC = INFINITY;
        for (int i = 0; i < g; ++i) {
            const int64_t r = row_off[b] + i;
            double h, c;
            int32_t am;
            sko_row_softmax(draft, dtype, r, V, prob, &h, &c, &am);
            H[r] = h; conf[r] = c;
            if (argmax) argmax[r] = am;
            sumH += h; sumC += c;
            if (h > maxH) maxH = h;
            if (c < minC) minC = c;
        }
        agg[4 * b + 0] = sumH / g;
        agg[4 * b + 1] = sumC / g;
        agg[4 * b + 2] = maxH;
        agg[4 * b + 3] = minC;
        free(prob);
    }
    return status;
}

/* ------------------------------------------------------------------------- */
/* Residual distribution and inverse-CDF draw, exported so tests can look in */
/* ------------------------------------------------------------------------- */
/* r(v) = max(0, p(v) - q(v)); q == NULL means the bonus case r = p.  Returns R = sum r. */
double sko_residual(const double *p, const double *q, int V, double *r)
{
    double R = 0.0;
    for (int v = 0; v < V; ++v) {
        double d = q ? p[v] - q[v] : p[v];
        r[v] = d > 0.0 ? d : 0.0;
        R += r[v];
    }
    return R;
}

/* Smallest v whose running sum of r exceeds tau; if rounding leaves none, the
 * largest v with r(v) > 0.  margin = distance from tau to the nearer edge of the
 * chosen token's CDF interval. */
int32_t sko_inverse_cdf(const double *r, int V, double tau, double *margin)
{
    double C = 0.0;
    int32_t last_pos = -1;
    for (int v = 0; v < V; ++v) {
        double prev = C;
        C += r[v];
        if (r[v] > 0.0) last_pos = v;
        if (C > tau) {
            if (margin) *margin = fmin(tau - prev, C - tau);
            return v;
        }
    }
    if (margin) *margin = 0.0;
    return last_pos;
}

/* ------------------------------------------------------------------------- */
/* Verification of every sequence (Section 3.1)                               */
/* ------------------------------------------------------------------------- */
/* target: packed rows, sequence b owns rows row_off[b]+b .. row_off[b]+b+gamma[b].
 * tokens: [B][gamma_max+1].  Optional outputs may be NULL.
 * resid_mass: [B] the mass R of max(0, p_n - q_n) (of p_gamma in the bonus case) as first computed,
 * i.e. before the fall-back to p_n that R < SKO_RESID_FLOOR triggers.
 * dbg: [B][gamma_max][3] = (u_i, q_i(t_i), p_i(t_i)) for the positions that were tested. */
int sko_verify(const void *draft, const void *target, int dtype, int B, int V,
               const int32_t *gamma, const int64_t *row_off, const int32_t *draft_tokens,
               uint64_t seed, uint32_t step, uint32_t seq_base, int gamma_max,
               int32_t *n_accepted, int32_t *tokens, int32_t *num_tokens, double *accept_rate,
               uint32_t *row_flags, double *marg_acc, double *marg_cdf, double *resid_mass, double *dbg)
{
    int status = 0;
    const int W = gamma_max + 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        double *q = (double *)malloc(sizeof(double) * (size_t)V);
        double *p = (double *)malloc(sizeof(double) * (size_t)V);
        double *r = (double *)malloc(sizeof(double) * (size_t)V);
        if (!q || !p || !r) {
#pragma omp atomic write
            status = 1;
            free(q); free(p); free(r);
            continue;
        }
        const int g = gamma[b];
        const int64_t drow = row_off[b], trow = row_off[b] + b;
        uint32_t flags = 0;
        double macc = INFINITY;

        /* flag scan over every row and every drafted token the sequence owns (the accept
         * loop below may stop early) */
        for (int i = 0; i < g; ++i) {
            int finite = 0;
            for (int v = 0; v < V; ++v) {
                double x = sko_load_logit(draft, dtype, (drow + i) * (int64_t)V + v);
                if (isnan(x) || x == INFINITY) flags |= SKO_FLAG_NONFINITE;
                if (isfinite(x)) finite = 1;
            }
            if (!finite) flags |= SKO_FLAG_NONFINITE;
            const int32_t t = draft_tokens[drow + i];
            if (t < 0 || t >= V) flags |= SKO_FLAG_BAD_TOKEN;
        }
        for (int i = 0; i <= g; ++i) {
            int finite = 0;
            for (int v = 0; v < V; ++v) {
                double x = sko_load_logit(target, dtype, (trow + i) * (int64_t)V + v);
                if (isnan(x) || x == INFINITY) flags |= SKO_FLAG_NONFINITE;
                if (isfinite(x)) finite = 1;
            }
            if (!finite) flags |= SKO_FLAG_NONFINITE;
        }

        /* sequential accept / reject */
        int n = 0;
        while (n < g) {
            const int i = n;
            uint32_t w[4];
            step_block(seed, seq_base + (uint32_t)b, (uint32_t)i, step, w);
            const double u = (double)(w[0] >> 8) * 0x1.0p-24;
            sko_row_softmax(draft, dtype, drow + i, V, q, NULL, NULL, NULL);
            sko_row_softmax(target, dtype, trow + i, V, p, NULL, NULL, NULL);
            const int32_t t = draft_tokens[drow + i];
            double qt = 0.0, pt = 0.0;
            if (t >= 0 && t < V) { qt = q[t]; pt = p[t]; } /* a bad id has probability 0 on both sides */
            if (dbg) {
                double *d = dbg + ((size_t)b * gamma_max + i) * 3;
                d[0] = u; d[1] = qt; d[2] = pt;
            }
            const double gap = fabs(u * qt - pt);
            if (gap < macc) macc = gap;
            if (u * qt < pt) ++n; /* accept with probability min(1, p/q) */
            else break;
        }

        /* the one extra token: correction (n < gamma) or bonus (n == gamma) */
        uint32_t w[4];
        step_block(seed, seq_base + (uint32_t)b, (uint32_t)n, step, w);
        const double u2 = (double)w[1] * 0x1.0p-32;
        double R;
        if (n < g) {
            R = sko_residual(p, q, V, r); /* p, q still hold position n */
        } else {
            sko_row_softmax(target, dtype, trow + g, V, p, NULL, NULL, NULL);
            R = sko_residual(p, NULL, V, r);
        }
        if (resid_mass) resid_mass[b] = R;
        if (!(R >= SKO_RESID_FLOOR) || !isfinite(R)) {
            flags |= SKO_FLAG_FALLBACK;
            R = sko_residual(p, NULL, V, r);
        }
        double mcdf = 0.0;
        int32_t y = sko_inverse_cdf(r, V, u2 * R, &mcdf);
        if (y < 0) y = 0; /* only reachable when the row is all NaN; keeps the id in range */

        n_accepted[b] = n;
        num_tokens[b] = n + 1;
        for (int j = 0; j < W; ++j) tokens[(size_t)b * W + j] = -1;
        for (int j = 0; j < n; ++j) tokens[(size_t)b * W + j] = draft_tokens[drow + j];
        tokens[(size_t)b * W + n] = y;
        if (accept_rate) accept_rate[b] = (double)n / (double)g;
        if (row_flags) row_flags[b] = flags;
        if (marg_acc) marg_acc[b] = macc;
        if (marg_cdf) marg_cdf[b] = mcdf;
        free(q); free(p); free(r);
    }
    return status;
}

/* ------------------------------------------------------------------------- */
/* Token proposal on the draft side (the step before verification, Section 3.1) */
/* ------------------------------------------------------------------------- */
/* The draft model proposes the gamma tokens of a step (Section 3.1); the paper does not say how a
 * token is drawn from q_i.  Reading taken: t_i is the smallest v whose cumulative probability, in
 * vocabulary order, exceeds u, with u = w0 * 2^-32 of the Philox block whose counter is
 * (sequence, position, step, 1) -- the fourth counter word 1 keeps these draws apart from the
 * ones verification makes for the same sequence, position and step.
 * draft: packed rows as in sko_signals; row (b, i) is drawn for position pos0 + i.
 * tokens, prob (q_i(t_i)), flags (SKO_FLAG_NONFINITE per row), margin (distance from u to the
 * nearer edge of the chosen token's CDF interval): one entry per draft row; optional ones may be NULL. */
int sko_sample_draft(const void *draft, int dtype, int B, int V, const int32_t *gamma,
                     const int64_t *row_off, uint64_t seed, uint32_t step, uint32_t seq_base,
                     uint32_t pos0, int32_t *tokens, double *prob, uint32_t *flags, double *margin)
{
    int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        double *q = (double *)malloc(sizeof(double) * (size_t)V);
        if (!q) {
#pragma omp atomic write
            status = 1;
            continue;
        }
        for (int i = 0; i < gamma[b]; ++i) {
            const int64_t r = row_off[b] + i;
            uint32_t f = 0;
            int finite = 0;
            for (int v = 0; v < V; ++v) {
                double x = sko_load_logit(draft, dtype, r * (int64_t)V + v);
                if (isnan(x) || x == INFINITY) f |= SKO_FLAG_NONFINITE;
                if (isfinite(x)) finite = 1;
            }
            if (!finite) f |= SKO_FLAG_NONFINITE;
            sko_row_softmax(draft, dtype, r, V, q, NULL, NULL, NULL);
            uint32_t ctr[4] = {seq_base + (uint32_t)b, pos0 + (uint32_t)i, step, 1u};
            uint32_t key[2] = {(uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32)};
            uint32_t w[4];
            sko_philox4x32_10(ctr, key, w);
            const double u = (double)w[0] * 0x1.0p-32;
            double total = 0.0;
            for (int v = 0; v < V; ++v) total += q[v];
            double m = 0.0;
            int32_t y = sko_inverse_cdf(q, V, u * total, &m);
            if (y < 0) y = 0; /* only reachable when the row is all NaN; keeps the id in range */
            tokens[r] = y;
            if (prob) prob[r] = q[y];
            if (flags) flags[r] = f;
            if (margin) margin[r] = m;
        }
        free(q);
    }
    return status;
}

/* ------------------------------------------------------------------------- */
/* Greedy verification: the accept rule exactly as Section 3.1 words it        */
/* ------------------------------------------------------------------------- */
/* Position i is accepted iff the target's top prediction at i (argmax of the target row, lowest
 * index on ties) equals the drafted token t_i.  At the first mismatch the target's prediction
 * replaces the draft token; after gamma accepts the extra token is the target's top prediction
 * at position gamma.  No draft logits and no random numbers are involved. */
int sko_verify_greedy(const void *target, int dtype, int B, int V, const int32_t *gamma,
                      const int64_t *row_off, const int32_t *draft_tokens, int gamma_max,
                      int32_t *n_accepted, int32_t *tokens, int32_t *num_tokens, double *accept_rate,
                      uint32_t *row_flags)
{
    const int W = gamma_max + 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const int g = gamma[b];
        const int64_t drow = row_off[b], trow = row_off[b] + b;
        uint32_t flags = 0;
        int32_t top[64]; /* gamma_max + 1 <= 17 */
        for (int i = 0; i <= g; ++i) {
            double m = -INFINITY;
            int32_t am = 0;
            int finite = 0;
            for (int v = 0; v < V; ++v) {
                double x = sko_load_logit(target, dtype, (trow + i) * (int64_t)V + v);
                if (isnan(x) || x == INFINITY) flags |= SKO_FLAG_NONFINITE;
                if (isfinite(x)) finite = 1;
                if (x > m) { m = x; am = v; }
            }
            if (!finite) flags |= SKO_FLAG_NONFINITE;
            top[i] = am;
        }
        for (int i = 0; i < g; ++i) {
            const int32_t t = draft_tokens[drow + i];
            if (t < 0 || t >= V) flags |= SKO_FLAG_BAD_TOKEN;
        }
        int n = 0;
        while (n < g && draft_tokens[drow + n] == top[n]) ++n;
        n_accepted[b] = n;
        num_tokens[b] = n + 1;
        for (int j = 0; j < W; ++j) tokens[(size_t)b * W + j] = -1;
        for (int j = 0; j < n; ++j) tokens[(size_t)b * W + j] = draft_tokens[drow + j];
        tokens[(size_t)b * W + n] = top[n];
        if (accept_rate) accept_rate[b] = (double)n / (double)g;
        if (row_flags) row_flags[b] = flags;
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Controller (Section 4.3, Eq. 1)                                            */
/* ------------------------------------------------------------------------- */
/* mode 0: x = [H_0, c_0, onehot3(comp)]            (5 inputs: position-0 signals)
 * mode 1: x = [meanH, meanC, maxH, minC, onehot3]  (7 inputs: the context vector of Section 4.3)
 *
 * The predictor f of Section 4.3 estimates the acceptance rate of each candidate Gamma_j in
 * (2, 4, 6, 8); Eq. 1 turns it into score_j = f_j * Gamma_j + 1 and the largest score wins
 * (lowest j on ties).  Two ways to evaluate f, each with or without a hidden layer:
 *   form 0 ("vector"): one network with four outputs, f_j = output j.
 *       n_hidden >= 1: h = relu(W1 x + b1), f = W2 h + b2; W1 [n_hidden][n_in], W2 [4][n_hidden], b2 [4]
 *       n_hidden == 0: f = W2 x + b2 (linear);             W2 [4][n_in], b2 [4]
 *   form 1 ("scalar", the way Section 4.3 writes it): f_j = f([x, Gamma_j]), evaluated four times.
 *       n_hidden >= 1: h = relu(W1 [x, Gamma_j] + b1), f_j = W2 h + b2; W1 [n_hidden][n_in + 1],
 *                      W2 [1][n_hidden], b2 [1]   (Table 3's MLP rows)
 *       n_hidden == 0: f_j = W2 [x, Gamma_j] + b2;  W2 [1][n_in + 1], b2 [1]   (Table 3's Ridge row)
 * All weights row-major binary32.  gap[b] = best score minus second-best score. */
int sko_select_gamma_form(int form, int mode, int n_hidden, const float *W1, const float *b1,
                          const float *W2, const float *b2, const double *H, const double *conf,
                          const double *agg, const int64_t *row_off, const uint8_t *comp, int B,
                          int32_t *gamma_next, double *scores, double *gap)
{
    const int n_in = mode == 0 ? 5 : 7;
    if (n_hidden < 0 || n_hidden > 1024 || (form != 0 && form != 1)) return 1;
    for (int b = 0; b < B; ++b) {
        double x[8];
        int k = 0;
        if (mode == 0) {
            x[k++] = H[row_off[b]];
            x[k++] = conf[row_off[b]];
        } else {
            for (int j = 0; j < 4; ++j) x[k++] = agg[4 * b + j];
        }
        for (int c = 0; c < 3; ++c) x[k++] = comp[b] == c ? 1.0 : 0.0;
        double f[4];
        if (form == 0) {
            double hid[1024];
            for (int j = 0; j < n_hidden; ++j) {
                double a = (double)b1[j];
                for (int i = 0; i < n_in; ++i) a += (double)W1[j * n_in + i] * x[i];
                hid[j] = a > 0.0 ? a : 0.0;
            }
            for (int o = 0; o < 4; ++o) {
                double a = (double)b2[o];
                if (n_hidden > 0)
                    for (int j = 0; j < n_hidden; ++j) a += (double)W2[o * n_hidden + j] * hid[j];
                else
                    for (int i = 0; i < n_in; ++i) a += (double)W2[o * n_in + i] * x[i];
                f[o] = a;
            }
        } else {
            const int n1 = n_in + 1;
            for (int o = 0; o < 4; ++o) {
                x[n_in] = (double)SKO_GAMMAS[o];
                double a = (double)b2[0];
                if (n_hidden > 0) {
                    for (int j = 0; j < n_hidden; ++j) {
                        double u = (double)b1[j];
                        for (int i = 0; i < n1; ++i) u += (double)W1[j * n1 + i] * x[i];
                        a += (double)W2[j] * (u > 0.0 ? u : 0.0);
                    }
                } else {
                    for (int i = 0; i < n1; ++i) a += (double)W2[i] * x[i];
                }
                f[o] = a;
            }
        }
        double sc[4];
        for (int o = 0; o < 4; ++o) sc[o] = f[o] * (double)SKO_GAMMAS[o] + 1.0; /* Eq. 1 */
        int best = 0;
        for (int o = 1; o < 4; ++o)
            if (sc[o] > sc[best]) best = o; /* strict: lowest index wins ties */
        double second = -INFINITY;
        for (int o = 0; o < 4; ++o)
            if (o != best && sc[o] > second) second = sc[o];
        gamma_next[b] = SKO_GAMMAS[best];
        if (scores)
            for (int o = 0; o < 4; ++o) scores[4 * b + o] = sc[o];
        if (gap) gap[b] = sc[best] - second;
    }
    return 0;
}

/* The four-output network with a hidden layer (the form the benchmark configurations use). */
int sko_select_gamma(int mode, int n_hidden, const float *W1, const float *b1, const float *W2,
                     const float *b2, const double *H, const double *conf, const double *agg,
                     const int64_t *row_off, const uint8_t *comp, int B, int32_t *gamma_next,
                     double *scores, double *gap)
{
    if (n_hidden < 1) return 1;
    return sko_select_gamma_form(0, mode, n_hidden, W1, b1, W2, b2, H, conf, agg, row_off, comp, B,
                                 gamma_next, scores, gap);
}
