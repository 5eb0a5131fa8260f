/*
 * CPU oracle for the lookahead-step attention and the greedy verification
 * reduction of Lookahead Decoding (arXiv 2402.02057).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, fp64 statement of
 * what the hot path computes, written from the paper, and it shares no code,
 * header, table or helper with the HIP library.  Only the tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it; the product path
 * never does.
 *
 * What is pinned (see tests/test_oracle_*.py): the mask against a
 * parent-pointer (ancestor) formulation, the position-chain invariant, the
 * closed-form count of visible pairs and the worked example of Sec. 3.3;
 * the attention arithmetic against textbook causal attention run on each
 * row's own token chain, against a library softmax-attention for the
 * one-token decode special case, and against isolation / permutation
 * invariants; the verification reduction against exhaustive enumeration on
 * tiny vocabularies, a library argmax, and the paper's Algorithm 3; the
 * end-of-step reduction (accepted token list, best candidate, new window
 * tokens) against the same exhaustive enumeration written from the words of
 * Sec. 3.2, a literal walk through Algorithm 3 on a prefix-deterministic toy
 * model (whose output must also equal plain greedy decoding), and a library
 * argmax; sampling verification (Algorithm 4) against the exact law of its
 * decision tree computed independently in the test (which is also checked
 * to give every emitted token the model's own distribution: Theorem A of
 * App. B), hand-computed accept/reject regions, the zero-temperature limit
 * (greedy verification) and a library softmax + inverse-CDF search.
 *
 * Row / key order of one step (same for q, step_k, step_v, out):
 *   r = 0                               the current input token, relative position 0
 *   r = 1 + l*W + j                     lookahead level l (0 = oldest of the N-1
 *                                       kept Jacobi iterates), column j; relative
 *                                       position 1 + l + j           (Sec. 3.1)
 *   r = 1 + W*(N-1) + g*(N-1) + k       candidate n-gram g, its k-th token after
 *                                       the shared first token; position 1 + k
 *                                                                    (Sec. 3.2)
 * T = 1 + (W + G)*(N - 1).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { TOK_CURRENT = 0, TOK_LOOKAHEAD = 1, TOK_CANDIDATE = 2 };

typedef struct {
    int branch; /* TOK_* */
    int level;  /* lookahead: level l; candidate: index g of the n-gram */
    int offset; /* lookahead: column j; candidate: token index k */
    int pos;    /* position relative to the current token */
} token_t;

int la_oracle_num_rows(int W, int N, int G) { return 1 + (W + G) * (N - 1); }

static token_t token_of(int r, int W, int N, int G)
{
    token_t t;
    (void)G;
    if (r == 0) {
        t.branch = TOK_CURRENT; t.level = 0; t.offset = 0; t.pos = 0;
    } else if (r < 1 + W * (N - 1)) {
        int x = r - 1;
        t.branch = TOK_LOOKAHEAD; t.level = x / W; t.offset = x % W;
        t.pos = 1 + t.level + t.offset;
    } else {
        int x = r - 1 - W * (N - 1);
        t.branch = TOK_CANDIDATE; t.level = x / (N - 1); t.offset = x % (N - 1);
        t.pos = 1 + t.offset;
    }
    return t;
}

/* Relative position of step row r (the digit printed on each token in Fig. 2(b)). */
int la_oracle_position(int r, int W, int N, int G) { return token_of(r, W, N, G).pos; }

/*
 * May step row r attend to step key c?  (Sec. 3.3, Fig. 2(b); the conditioning
 * sets of Algorithm 2.)
 *  - every row sees the current token;
 *  - a lookahead row (l, j) is conditioned on its own column at the levels up
 *    to its own, and on the oldest level up to its own column: that is its
 *    Jacobi trajectory followed back to the current token;
 *  - a candidate row (g, k) sees the earlier tokens of the same candidate;
 *  - the two branches do not see each other, nor do different candidates.
 */
int la_oracle_visible(int r, int c, int W, int N, int G)
{
    token_t tr = token_of(r, W, N, G), tc = token_of(c, W, N, G);
    if (tc.branch == TOK_CURRENT) return 1;
    if (tc.branch == TOK_LOOKAHEAD) {
        if (tr.branch != TOK_LOOKAHEAD) return 0;
        if (tc.level == 0 && tc.offset <= tr.offset) return 1;
        if (tc.offset == tr.offset && tc.level <= tr.level) return 1;
        return 0;
    }
    /* tc is a candidate token */
    if (tr.branch != TOK_CANDIDATE) return 0;
    return tc.level == tr.level && tc.offset <= tr.offset;
}

/* mask[r*T + c] = 1 iff step row r may attend to step key c. */
void la_oracle_step_mask(int W, int N, int G, uint8_t *mask)
{
    int T = la_oracle_num_rows(W, N, G);
    for (int r = 0; r < T; ++r)
        for (int c = 0; c < T; ++c)
            mask[(size_t)r * T + c] = (uint8_t)la_oracle_visible(r, c, W, N, G);
}

static double bf16_bits_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/*
 * The 8-bit float of a quantised KV cache: the OCP "E4M3" format in its finite-only form (one sign
 * bit, four exponent bits with bias 7, three mantissa bits).  Exponent field 0 holds the subnormals
 * m/8 * 2^-6; there are no infinities, and S.1111.111 is the only NaN, so the largest value is
 * 1.75 * 2^8 = 448.  (An extension of the step to a quantised cache: the paper computes in 16 bits.)
 */
static double fp8_e4m3_to_double(uint8_t c)
{
    const int sign = c >> 7, e = (c >> 3) & 15, m = c & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m / 8.0, -6);
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

void la_oracle_fp8_e4m3_decode(const uint8_t *codes, size_t n, double *out)
{
    for (size_t i = 0; i < n; ++i) out[i] = fp8_e4m3_to_double(codes[i]);
}

int la_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* How many threads the loops over heads may use from now on (timing the oracle on one core). */
void la_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/*
 * out = softmax(mask(q k^T / sqrt(head_dim))) v, per head (Sec. 2, "Causal
 * Attention in Decoder Models", with the mask of Sec. 3.3).  Keys of a row are
 * the P prefix keys of its KV head (all visible) followed by the T step keys
 * (visible per la_oracle_visible).  Query head h reads KV head h / (heads /
 * kv_heads).  All inputs are bf16 bit patterns, arithmetic is fp64.
 *
 *   q       [T][heads][head_dim]
 *   k_cache [kv_heads][P][head_dim]   v_cache likewise
 *   step_k  [T][kv_heads][head_dim]   step_v likewise
 *   out     [T][heads][head_dim]      fp64
 * Returns 0, or -1 for an impossible shape.
 */
/* One key or value element as fp64: a bf16 bit pattern, or (quantised cache) an 8-bit float times
 * the scale of its KV head. */
static double kv_element(const void *base, size_t index, int fp8, double scale)
{
    if (fp8) return fp8_e4m3_to_double(((const uint8_t *)base)[index]) * scale;
    return bf16_bits_to_double(((const uint16_t *)base)[index]);
}

static int step_attention_dense(const uint16_t *q, const void *k_cache, const void *v_cache,
                                const void *step_k, const void *step_v, int fp8, const float *k_scale,
                                const float *v_scale, int P, int W, int N, int G, int heads,
                                int kv_heads, int head_dim, double *out)
{
    if (P < 0 || W < 0 || G < 0 || N < 2 || heads < 1 || kv_heads < 1 || head_dim < 1) return -1;
    if (heads % kv_heads != 0) return -1;
    const int T = la_oracle_num_rows(W, N, G);
    const int group = heads / kv_heads;
    const int d = head_dim;
    const size_t L = (size_t)P + (size_t)T; /* keys per row */
    const double scale = 1.0 / sqrt((double)d);

    /* the explicit boolean mask over [T][P + T] */
    uint8_t *mask = (uint8_t *)malloc((size_t)T * L);
    if (!mask) return -1;
    for (int r = 0; r < T; ++r) {
        for (int p = 0; p < P; ++p) mask[(size_t)r * L + p] = 1;
        for (int c = 0; c < T; ++c)
            mask[(size_t)r * L + P + c] = (uint8_t)la_oracle_visible(r, c, W, N, G);
    }

    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < heads; ++h) {
        const int kvh = h / group;
        double *K = (double *)malloc(L * d * sizeof(double));
        double *V = (double *)malloc(L * d * sizeof(double));
        double *S = (double *)malloc((size_t)T * L * sizeof(double));
        double *qr = (double *)malloc((size_t)d * sizeof(double));
        if (!K || !V || !S || !qr) {
            failed = 1;
            free(K); free(V); free(S); free(qr);
            continue;
        }
        /* keys and values of this head, prefix then step tokens, as fp64 */
        const double ksc = fp8 ? (double)k_scale[kvh] : 1.0, vsc = fp8 ? (double)v_scale[kvh] : 1.0;
        for (int p = 0; p < P; ++p)
            for (int e = 0; e < d; ++e) {
                size_t src = ((size_t)kvh * P + p) * d + e;
                K[(size_t)p * d + e] = kv_element(k_cache, src, fp8, ksc);
                V[(size_t)p * d + e] = kv_element(v_cache, src, fp8, vsc);
            }
        for (int c = 0; c < T; ++c)
            for (int e = 0; e < d; ++e) {
                size_t src = ((size_t)c * kv_heads + kvh) * d + e;
                K[((size_t)P + c) * d + e] = kv_element(step_k, src, fp8, ksc);
                V[((size_t)P + c) * d + e] = kv_element(step_v, src, fp8, vsc);
            }
        /* dense scores */
        for (int r = 0; r < T; ++r) {
            for (int e = 0; e < d; ++e)
                qr[e] = bf16_bits_to_double(q[((size_t)r * heads + h) * d + e]);
            for (size_t c = 0; c < L; ++c) {
                double s = 0.0;
                for (int e = 0; e < d; ++e) s += qr[e] * K[c * d + e];
                S[(size_t)r * L + c] = s * scale;
            }
        }
        /* masked softmax and the weighted sum of values */
        for (int r = 0; r < T; ++r) {
            const uint8_t *mr = mask + (size_t)r * L;
            double *sr = S + (size_t)r * L;
            double m = -INFINITY;
            for (size_t c = 0; c < L; ++c)
                if (mr[c] && sr[c] > m) m = sr[c];
            double denom = 0.0;
            for (size_t c = 0; c < L; ++c) {
                sr[c] = mr[c] ? exp(sr[c] - m) : 0.0;
                denom += sr[c];
            }
            double *o = out + ((size_t)r * heads + h) * d;
            for (int e = 0; e < d; ++e) o[e] = 0.0;
            for (size_t c = 0; c < L; ++c) {
                if (!mr[c]) continue;
                double w = sr[c] / denom;
                for (int e = 0; e < d; ++e) o[e] += w * V[c * d + e];
            }
        }
        free(K); free(V); free(S); free(qr);
    }
    free(mask);
    return failed ? -1 : 0;
}

int la_oracle_step_attention(const uint16_t *q, const uint16_t *k_cache, const uint16_t *v_cache,
                             const uint16_t *step_k, const uint16_t *step_v, int P, int W, int N,
                             int G, int heads, int kv_heads, int head_dim, double *out)
{
    return step_attention_dense(q, k_cache, v_cache, step_k, step_v, 0, NULL, NULL, P, W, N, G, heads,
                                kv_heads, head_dim, out);
}

/*
 * The same step over a quantised KV cache: k_cache, v_cache, step_k and step_v hold 8-bit floats
 * (E4M3, see fp8_e4m3_to_double) in the layouts above, and an element of KV head h stands for its
 * decoded value times k_scale[h] (keys) or v_scale[h] (values).  The step's own keys and values are
 * quantised like the cache, so that a token committed later is read back exactly as its step saw it.
 * q stays bf16; everything is decoded to fp64 and goes through the dense definition unchanged.
 * Returns 0, or -1 for an impossible shape or a missing scale array.
 */
int la_oracle_step_attention_fp8kv(const uint16_t *q, const uint8_t *k_cache, const uint8_t *v_cache,
                                   const uint8_t *step_k, const uint8_t *step_v, const float *k_scale,
                                   const float *v_scale, int P, int W, int N, int G, int heads,
                                   int kv_heads, int head_dim, double *out)
{
    if (!k_scale || !v_scale) return -1;
    return step_attention_dense(q, k_cache, v_cache, step_k, step_v, 1, k_scale, v_scale, P, W, N, G,
                                heads, kv_heads, head_dim, out);
}

/*
 * Greedy verification reduction (Sec. 2, the guess-and-verify paragraph: accept while the
 * model's greedy choice equals the draft token, stop at the first mismatch;
 * Algorithm 3 applies it to G candidates at once).
 *
 *   logits      [G][N-1][V] fp32; row (g,k) is the model output that judges
 *               cand_tokens[g][k]
 *   cand_tokens [G][N-1]
 *   accepted    [G][N-1]  out: argmax of every row, lowest index on ties
 *   accept_len  [G]       out: number of leading k with accepted == cand_tokens
 */
int la_oracle_verify(const float *logits, const int32_t *cand_tokens, int G, int N, int V,
                     int32_t *accept_len, int32_t *accepted)
{
    if (G < 0 || N < 2 || V < 1) return -1;
    const int n1 = N - 1;
    for (int g = 0; g < G; ++g) {
        for (int k = 0; k < n1; ++k) {
            const float *row = logits + ((size_t)g * n1 + k) * V;
            int best = 0;
            for (int v = 1; v < V; ++v)
                if (row[v] > row[best]) best = v;
            accepted[g * n1 + k] = best;
        }
        int len = 0;
        while (len < n1 && accepted[g * n1 + len] == cand_tokens[g * n1 + len]) ++len;
        accept_len[g] = len;
    }
    return 0;
}

/*
 * The end of a greedy lookahead step in one call (Algorithm 3 in full, and the new window
 * tokens of Algorithm 2's lookahead branch).  Plain definition, scalar loops.
 *
 *   logits_cur   [V]          model output at the current token: judges slot 0 of every candidate
 *   logits_look  [W][V]       outputs at the W newest lookahead tokens (one per column)
 *   logits_cand  [G][N-1][V]  row (g,k): output at candidate g's token k; judges slot k+1, and
 *                             row (g,N-2) gives the bonus token when all N-1 slots were accepted
 *   cand_tokens  [G][N-1]
 * out:
 *   accept_len[g]  leading slots s with argmax(judge(g,s)) == cand_tokens[g][s]
 *   best           lowest g with the largest accept_len (-1 if G == 0); L = that length
 *   out_tokens     cand_tokens[best][0..L-1], then argmax(judge(best, L)): the correction
 *                  token (L < N-1) or the bonus token (L == N-1); n_out = L + 1
 *   new_window[j]  argmax of logits_look[j]
 * argmax = lowest index of the maximum.
 */
static int argmax_row(const float *row, int V)
{
    int best = 0;
    for (int v = 1; v < V; ++v)
        if (row[v] > row[best]) best = v;
    return best;
}

int la_oracle_verify_step(const float *logits_cur, const float *logits_look, const float *logits_cand,
                          const int32_t *cand_tokens, int W, int N, int G, int V, int32_t *out_tokens,
                          int32_t *n_out, int32_t *best, int32_t *new_window, int32_t *accept_len)
{
    if (W < 0 || G < 0 || N < 2 || V < 1) return -1;
    const int n1 = N - 1;
    for (int j = 0; j < W; ++j) new_window[j] = argmax_row(logits_look + (size_t)j * V, V);
    const int cur_token = argmax_row(logits_cur, V);
    int best_g = -1, best_len = 0;
    for (int g = 0; g < G; ++g) {
        int len = 0;
        while (len < n1) {
            const int judged = len == 0 ? cur_token
                                        : argmax_row(logits_cand + ((size_t)g * n1 + (len - 1)) * V, V);
            if (judged != cand_tokens[g * n1 + len]) break;
            ++len;
        }
        accept_len[g] = len;
        if (best_g < 0 || len > best_len) {
            best_g = g;
            best_len = len;
        }
    }
    *best = best_g;
    for (int s = 0; s < best_len; ++s) out_tokens[s] = cand_tokens[best_g * n1 + s];
    out_tokens[best_len] = best_len == 0 ? cur_token
                                         : argmax_row(logits_cand + ((size_t)best_g * n1 + (best_len - 1)) * V, V);
    *n_out = best_len + 1;
    return 0;
}

/*
 * Sampling verification (Algorithm 4), step by step in the algorithm's order, fp64.
 *
 *   logits_cur   [V]          model output at the current token (the first of the N
 *                             distributions of every candidate)
 *   logits_cand  [G][N-1][V]  row (g,k): output at candidate g's token k (distribution k+2)
 *   cand_tokens  [G][N-1]
 *   u_test       [N-1][G]     the uniform draws of the accept tests: u_test[i][j] is the one
 *                             drawn for the j-th candidate examined at position i
 *   u_final                   the draw that samples the last token
 *   temperature > 0           distributions are softmax(logits / temperature)
 *
 * At each position the surviving candidates are examined in order; candidate token s is
 * accepted if the draw is below P(s), where P starts as the model's distribution at this
 * position (all survivors share the accepted prefix, the first survivor's row is used) and,
 * after every rejection, has the rejected token's probability set to zero and is renormalised.
 * After an acceptance only the later candidates with the same token survive.  If no candidate
 * is accepted, one token is sampled from the residual P and the walk stops; after N-1
 * acceptances one token is sampled from the first survivor's N-th distribution.
 *
 * Readings: the test "r <= P(s)" is taken as r < P(s) for r in [0,1) (same probability; a
 * token of probability zero is never accepted); sampling is by inverse CDF in index order:
 * the first v whose cumulative probability exceeds u.  G == 0: one token sampled from the
 * current token's distribution.  A candidate token outside 0 .. V-1 (a padding id) is examined
 * like any other - its draw is spent - and has probability zero.
 */
static void softmax_row(const float *row, int V, double inv_t, double *P)
{
    double m = (double)row[0] * inv_t;
    for (int v = 1; v < V; ++v)
        if ((double)row[v] * inv_t > m) m = (double)row[v] * inv_t;
    double z = 0.0;
    for (int v = 0; v < V; ++v) {
        P[v] = exp((double)row[v] * inv_t - m);
        z += P[v];
    }
    for (int v = 0; v < V; ++v) P[v] /= z;
}

static int sample_inverse_cdf(const double *P, int V, double u)
{
    double c = 0.0;
    int last_positive = 0;
    for (int v = 0; v < V; ++v) {
        if (P[v] > 0.0) last_positive = v;
        c += P[v];
        if (c > u) return v;
    }
    return last_positive;  /* rounding left the total a hair below u */
}

int la_oracle_verify_sample(const float *logits_cur, const float *logits_cand, const int32_t *cand_tokens,
                            const float *u_test, float u_final, float temperature, int N, int G, int V,
                            int32_t *out_tokens, int32_t *n_out)
{
    if (G < 0 || N < 2 || V < 1 || !(temperature > 0.0f)) return -1;
    const int n1 = N - 1;
    const double inv_t = 1.0 / (double)temperature;
    double *P = (double *)malloc((size_t)V * sizeof(double));
    int *alive = (int *)malloc((size_t)(G > 0 ? G : 1) * sizeof(int));
    if (!P || !alive) { free(P); free(alive); return -2; }
    int n_alive = G, len = 0;
    for (int g = 0; g < G; ++g) alive[g] = g;

    for (int i = 0; i < n1 && n_alive > 0; ++i) {
        /* the i-th distribution of the first survivor */
        const int g0 = alive[0];
        softmax_row(i == 0 ? logits_cur : logits_cand + ((size_t)g0 * n1 + (i - 1)) * V, V, inv_t, P);
        int accepted = 0;
        for (int j = 0; j < n_alive; ++j) {
            const int s = cand_tokens[alive[j] * n1 + i];
            const double r = (double)u_test[i * G + j];
            /* a token outside the vocabulary has probability zero under every distribution over
             * it: the draw is spent, the token is not accepted and there is nothing to rule out */
            if (s < 0 || s >= V) continue;
            if (r < P[s]) {
                out_tokens[len++] = s;
                accepted = 1;
                int m = 0;
                for (int k = j; k < n_alive; ++k)
                    if (cand_tokens[alive[k] * n1 + i] == s) alive[m++] = alive[k];
                n_alive = m;
                break;
            }
            /* rejected: this token is ruled out, renormalise */
            P[s] = 0.0;
            double z = 0.0;
            for (int v = 0; v < V; ++v) z += P[v];
            for (int v = 0; v < V; ++v) P[v] /= z;
        }
        if (!accepted) {
            out_tokens[len++] = sample_inverse_cdf(P, V, (double)u_final);
            *n_out = len;
            free(P); free(alive);
            return 0;
        }
    }
    /* every position accepted (or no candidates at all): one more token from the model */
    softmax_row(len == 0 ? logits_cur : logits_cand + ((size_t)alive[0] * n1 + (len - 1)) * V, V, inv_t, P);
    out_tokens[len++] = sample_inverse_cdf(P, V, (double)u_final);
    *n_out = len;
    free(P); free(alive);
    return 0;
}

