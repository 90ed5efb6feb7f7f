/*
 * ssd_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, single-threaded CPU statement of what the SSD compressed
 * decode-attention path computes (arxiv 2510.18716).  It exists so that the
 * GPU library can be checked against something written straight from the
 * paper.  It shares no code, header, table or helper with the GPU library
 * and is never called by it.  Only the tests, the smoke check and the
 * benchmark's "cpu_baseline" leg may use it.
 *
 * Everything accumulates in double; inputs and outputs are float arrays
 * (a bf16 workload is handed over already widened to float, which is exact).
 * There is no blocking, fusion or reordering: rows are visited in ascending
 * token position, exactly as the definitions below state.
 *
 * Contents (paper passage each part follows):
 *   O1  dense softmax attention of one query over a list of rows
 *       -- the full-cache baseline of Sec. 4.1 and the "AttentionScores"
 *          step of Algorithm 1.
 *   O2  the sparsity metric s_{l,h} (display formula in Sec. 3.3,
 *       "Spatial Sparsity Analysis") and the threshold rule, Eq. (3).
 *   O3  top-M selection by accumulated score ("IndicesOfTopM", Algorithm 1).
 *   O5  accumulated scores of a prompt processed at once under causal
 *       attention (prefill branch of Algorithm 2).
 *   O6  classifier-free guidance of the two distributions of a prompt,
 *       Eq. (1) of Sec. 3.1.
 *   O7  rotary position embedding of a query / key row.  Not from the paper
 *       (which is silent on the model's position encoding): the definition
 *       of Su et al., "RoFormer", in the two element pairings in use.  It
 *       serves the variant of the fused step that rotates q and k on the way
 *       in.
 *   O4  the per-head cache policy of Algorithm 1 with the additions the text
 *       of Sec. 3.3 makes (initial sink token for spatial heads, reserved
 *       recent window R for semantic heads) and the deferred-compression
 *       cadence of Algorithm 2 (row buffer, overflow error), including
 *       Algorithm 2's treatment of spatial heads (cached window as of the
 *       last compression, plus the row buffer).
 *
 * Readings of points the paper leaves open (identical on the GPU side):
 *   - softmax scale is a caller-supplied number (1/sqrt(d) by default);
 *   - the new token is appended first, then attended to (it sees itself),
 *     and the probabilities of that same softmax are what is accumulated;
 *   - W counts the current token; S initial positions are always kept by a
 *     spatial head; R newest tokens of a semantic head are never evicted and
 *     are not candidates; an evicted token never returns and its score is
 *     dropped; ties in the top-M go to the lower position; fewer than M
 *     candidates keeps all of them;
 *   - the metric's sums run over visual rows only (row t-1 is the query's
 *     own), a step with t <= w contributes ratio 0, a zero denominator
 *     contributes ratio 0.
 *
 * Pins: see tests/test_oracle_*.py (closed forms, library softmax/SDPA,
 * brute force, the exact-rational worked case under tests/golden/).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ O1 -- */

/*
 * Softmax attention of query q[d] over the rows listed in rows[0..n_rows)
 * of K[., d], V[., d] (row-major, row index = token position).
 *   z_j = scale * sum_i q_i K[rows[j]][i]
 *   p_j = exp(z_j - max z) / sum_j exp(z_j - max z)
 *   o   = sum_j p_j V[rows[j]]
 * o_out[d] (float), p32_out[n_rows] (float, may be NULL), p64_out[n_rows]
 * (double, may be NULL).  n_rows == 0 gives o = 0.  Returns 0.
 */
int ssd_oracle_attend(const float *q, const float *K, const float *V, int d,
                      const int32_t *rows, int n_rows, double scale,
                      float *o_out, float *p32_out, double *p64_out)
{
    int i, j;
    double *z, *acc, mx, sum;
    if (n_rows <= 0) {
        for (i = 0; i < d; ++i) o_out[i] = 0.0f;
        return 0;
    }
    z = (double *)malloc(sizeof(double) * (size_t)n_rows);
    acc = (double *)calloc((size_t)d, sizeof(double));
    for (j = 0; j < n_rows; ++j) {
        const float *k = K + (size_t)rows[j] * (size_t)d;
        double dot = 0.0;
        for (i = 0; i < d; ++i) dot += (double)q[i] * (double)k[i];
        z[j] = scale * dot;
    }
    mx = z[0];
    for (j = 1; j < n_rows; ++j) if (z[j] > mx) mx = z[j];
    sum = 0.0;
    for (j = 0; j < n_rows; ++j) { z[j] = exp(z[j] - mx); sum += z[j]; }
    for (j = 0; j < n_rows; ++j) {
        const float *v = V + (size_t)rows[j] * (size_t)d;
        double p = z[j] / sum;
        if (p32_out) p32_out[j] = (float)p;
        if (p64_out) p64_out[j] = p;
        for (i = 0; i < d; ++i) acc[i] += p * (double)v[i];
    }
    for (i = 0; i < d; ++i) o_out[i] = (float)acc[i];
    free(z);
    free(acc);
    return 0;
}

/* Dense attention over rows 0..n-1 (the full-cache baseline). */
int ssd_oracle_dense_attend(const float *q, const float *K, const float *V,
                            int d, int n, double scale, float *o_out,
                            float *p32_out, double *p64_out)
{
    int j, rc;
    int32_t *rows = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    for (j = 0; j < n; ++j) rows[j] = j;
    rc = ssd_oracle_attend(q, K, V, d, rows, n, scale, o_out, p32_out, p64_out);
    free(rows);
    return rc;
}

/* ------------------------------------------------------------------ O2 -- */

/*
 * One term of the sparsity metric.  p[0..n0+t) is the attention distribution
 * of the t-th visual token (t >= 1) over the n0 prompt rows followed by the t
 * visual rows generated so far (its own row last).  With visual rows indexed
 * i = 0..t-1:
 *   tot = sum_{i=0}^{t-1}   p[n0+i]
 *   far = sum_{i=0}^{t-1-w} p[n0+i]      (empty when t <= w)
 */
void ssd_oracle_far_tot(const double *p, int n0, int t, int w, double *far,
                        double *tot)
{
    int i;
    double f = 0.0, s = 0.0;
    for (i = 0; i <= t - 1; ++i) s += p[n0 + i];
    for (i = 0; i <= t - 1 - w; ++i) f += p[n0 + i];
    *far = f;
    *tot = s;
}

/*
 * far/tot of every visual step of one (sequence, head): q, K, V are
 * [n0+T, d]; step t = 1..T uses query row n0+t-1 over rows 0..n0+t-1.
 * far_out[T], tot_out[T] as float (what a profiling run hands to the
 * classification reduction).
 */
void ssd_oracle_profile_unit(const float *q, const float *K, const float *V,
                             int d, int n0, int T, int w, double scale,
                             float *far_out, float *tot_out)
{
    int t;
    float *o = (float *)malloc(sizeof(float) * (size_t)d);
    double *p = (double *)malloc(sizeof(double) * (size_t)(n0 + T));
    for (t = 1; t <= T; ++t) {
        double far, tot;
        int n = n0 + t;
        ssd_oracle_dense_attend(q + (size_t)(n - 1) * (size_t)d, K, V, d, n,
                                scale, o, NULL, p);
        ssd_oracle_far_tot(p, n0, t, w, &far, &tot);
        far_out[t - 1] = (float)far;
        tot_out[t - 1] = (float)tot;
    }
    free(o);
    free(p);
}

/*
 * s[l][h] = (1/P) sum_p (1/T) sum_t far/tot over far, tot laid out
 * [L, P, H, T]; type[l][h] = 1 (Semantic) iff s > tau, else 0 (Spatial).
 */
void ssd_oracle_classify(const float *far, const float *tot, int L, int P,
                         int H, int T, double tau, double *s_out,
                         uint8_t *type_out)
{
    int l, p, h, t;
    for (l = 0; l < L; ++l) {
        for (h = 0; h < H; ++h) {
            double acc = 0.0;
            for (p = 0; p < P; ++p) {
                const size_t base = (((size_t)l * P + p) * H + h) * (size_t)T;
                double inner = 0.0;
                for (t = 0; t < T; ++t) {
                    double den = (double)tot[base + t];
                    double num = (double)far[base + t];
                    inner += (den > 0.0) ? num / den : 0.0;
                }
                acc += inner / (double)T;
            }
            acc /= (double)P;
            s_out[(size_t)l * H + h] = acc;
            type_out[(size_t)l * H + h] = (acc > tau) ? 1 : 0;
        }
    }
}

/* ---------------------------------------------------------- prefill scores -- */

/*
 * Accumulated attention scores of a prompt of n tokens under causal attention
 * (the prefill branch of Algorithm 2: "Accumulate semantic attention scores"
 * when the whole prompt is processed at once):
 *   a_i = softmax over rows 0..i of scale * q_i . k_j          (query i sees rows 0..i)
 *   score[j] = sum_{i=j}^{n-1} a_i(j)
 * q, K are [n, d]; score_out[n] (float).  The same numbers n ordinary decode
 * steps without compression would accumulate.
 */
void ssd_oracle_prefill_scores(const float *q, const float *K, int d, int n,
                               double scale, float *score_out)
{
    int i, j, t;
    double *acc = (double *)calloc((size_t)(n > 0 ? n : 1), sizeof(double));
    double *z = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    for (i = 0; i < n; ++i) {
        double mx, sum = 0.0;
        for (j = 0; j <= i; ++j) {
            double dot = 0.0;
            for (t = 0; t < d; ++t) dot += (double)q[(size_t)i * d + t] * (double)K[(size_t)j * d + t];
            z[j] = scale * dot;
        }
        mx = z[0];
        for (j = 1; j <= i; ++j) if (z[j] > mx) mx = z[j];
        for (j = 0; j <= i; ++j) { z[j] = exp(z[j] - mx); sum += z[j]; }
        for (j = 0; j <= i; ++j) acc[j] += z[j] / sum;
    }
    for (j = 0; j < n; ++j) score_out[j] = (float)acc[j];
    free(acc);
    free(z);
}

/* ------------------------------------------------------------------ O6 -- */

/*
 * Classifier-free guidance, Eq. (1): for prompt i the conditional row is
 * sequence 2i, the unconditional row sequence 2i+1 (Sec. 3.1 names the two
 * passes; the adjacent pairing is this build's batch layout), and
 *   out[i, v] = p_c[v] + gamma * (p_c[v] - p_u[v]).
 * p is [2 * n_prompts, V]; out is [n_prompts, V].
 */
void ssd_oracle_cfg_mix(const float *p, int n_prompts, int V, double gamma, float *out)
{
    int i, v;
    for (i = 0; i < n_prompts; ++i) {
        const float *c = p + (size_t)(2 * i) * V, *u = p + (size_t)(2 * i + 1) * V;
        for (v = 0; v < V; ++v) out[(size_t)i * V + v] = (float)((double)c[v] + gamma * ((double)c[v] - (double)u[v]));
    }
}

/* ------------------------------------------------------------------ O7 -- */

/*
 * Rotary position embedding of one row x[d] at a position whose angles are
 * given by cosv[i], sinv[i], i = 0..d/2-1: every pair (a, b) of elements is
 * rotated in its plane,
 *     a' = a cos_i - b sin_i,   b' = b cos_i + a sin_i.
 * layout 1: pair i is (x[i], x[i + d/2]); layout 2: pair i is (x[2i], x[2i+1]).
 * Computed in double, returned as float.
 */
void ssd_oracle_rope(const float *x, int d, const float *cosv, const float *sinv, int layout, float *out)
{
    int i;
    for (i = 0; i < d / 2; ++i) {
        const int ia = layout == 1 ? i : 2 * i;
        const int ib = layout == 1 ? i + d / 2 : 2 * i + 1;
        const double a = x[ia], b = x[ib], c = cosv[i], s = sinv[i];
        out[ia] = (float)(a * c - b * s);
        out[ib] = (float)(b * c + a * s);
    }
}

/* ------------------------------------------------------------------ O3 -- */

typedef struct { float score; int32_t pos; int32_t idx; } cand_t;

/* the order of the selection: higher score first, then lower position */
static int cand_before(const void *a, const void *b)
{
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    if (x->pos < y->pos) return -1;
    if (x->pos > y->pos) return 1;
    return 0;
}

static int idx_by_pos(const void *a, const void *b)
{
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    return (x->pos > y->pos) - (x->pos < y->pos);
}

/*
 * Of n candidates (score[i], pos[i]) keep the M that come first under
 * "higher score, then lower position"; all of them if n <= M.  Writes the
 * kept candidates' indices into keep_out, ordered by ascending position, and
 * returns how many.  *gap_out (may be NULL) receives (s_M - s_{M+1}) / s_M,
 * the relative score margin at the cut, or -1 when nothing was cut.
 */
int ssd_oracle_top_m(const float *score, const int32_t *pos, int n, int M,
                     int32_t *keep_out, double *gap_out)
{
    int i, kept;
    cand_t *c;
    if (gap_out) *gap_out = -1.0;
    if (n <= 0 || M <= 0) return 0;
    c = (cand_t *)malloc(sizeof(cand_t) * (size_t)n);
    for (i = 0; i < n; ++i) { c[i].score = score[i]; c[i].pos = pos[i]; c[i].idx = i; }
    qsort(c, (size_t)n, sizeof(cand_t), cand_before);
    kept = n < M ? n : M;
    if (gap_out && n > M) {
        double a = (double)c[M - 1].score, b = (double)c[M].score;
        *gap_out = (a > 0.0) ? (a - b) / a : 0.0;
    }
    qsort(c, (size_t)kept, sizeof(cand_t), idx_by_pos);
    for (i = 0; i < kept; ++i) keep_out[i] = c[i].idx;
    free(c);
    return kept;
}

/* ------------------------------------------------------------------ O4 -- */

typedef struct ssd_oracle_unit {
    int is_semantic;
    int W, S, M, R, C;
    int buffered;        /* spatial head under Algorithm 2: window frozen at the last compression + row buffer */
    int n_c;             /* buffered spatial head: token count at the last compression                        */
    int n_buf;           /* buffered spatial head: tokens in the row buffer (same counting as a semantic head) */
    int n;               /* tokens appended so far; positions 0..n-1 */
    /* semantic heads only: retained positions with their running scores */
    int n_heavy;  int32_t *heavy_pos;  float *heavy_score;   /* cap M        */
    int n_staged; int32_t *staged_pos; float *staged_score;  /* grows freely */
    int staged_cap;
} ssd_oracle_unit;

ssd_oracle_unit *ssd_oracle_unit_new(int is_semantic, int W, int S, int M,
                                     int R, int C)
{
    ssd_oracle_unit *u = (ssd_oracle_unit *)calloc(1, sizeof(*u));
    u->is_semantic = is_semantic;
    u->W = W; u->S = S; u->M = M; u->R = R; u->C = C;
    if (is_semantic) {
        u->heavy_pos = (int32_t *)calloc((size_t)(M > 0 ? M : 1), sizeof(int32_t));
        u->heavy_score = (float *)calloc((size_t)(M > 0 ? M : 1), sizeof(float));
        u->staged_cap = C > 0 ? C : 1;
        u->staged_pos = (int32_t *)calloc((size_t)u->staged_cap, sizeof(int32_t));
        u->staged_score = (float *)calloc((size_t)u->staged_cap, sizeof(float));
    }
    return u;
}

void ssd_oracle_unit_free(ssd_oracle_unit *u)
{
    if (!u) return;
    free(u->heavy_pos); free(u->heavy_score);
    free(u->staged_pos); free(u->staged_score);
    free(u);
}

static void staged_reserve(ssd_oracle_unit *u, int need)
{
    if (need <= u->staged_cap) return;
    u->staged_cap = need;
    u->staged_pos = (int32_t *)realloc(u->staged_pos, sizeof(int32_t) * (size_t)need);
    u->staged_score = (float *)realloc(u->staged_score, sizeof(float) * (size_t)need);
}

/*
 * Append the next token (position p = n).  Spatial: the window slides by
 * itself (the retained set is a function of n).  Semantic: the token enters
 * the row buffer with score 0; returns -1 ("row buffer overflow",
 * Algorithm 2) and changes nothing if the buffer already holds C tokens.
 */
int ssd_oracle_unit_append(ssd_oracle_unit *u)
{
    if (!u->is_semantic && u->buffered) {
        if (u->n_buf >= u->C) return -1;
        u->n_buf += 1;
    }
    if (u->is_semantic) {
        if (u->n_staged >= u->C) return -1;
        u->staged_pos[u->n_staged] = u->n;
        u->staged_score[u->n_staged] = 0.0f;
        u->n_staged += 1;
    }
    u->n += 1;
    return 0;
}

int ssd_oracle_unit_n(const ssd_oracle_unit *u) { return u->n; }

/*
 * Algorithm 2 for spatial heads (off by default): the head attends to its cached entries -- the sink tokens
 * and the W most recent tokens as of the last compression -- concatenated with the row buffer, i.e. every
 * token appended since; a compression re-cuts the window ("Compress spatial cache (sink + recent)").
 */
void ssd_oracle_unit_set_buffered(ssd_oracle_unit *u, int on) { u->buffered = on; }

/*
 * Retained positions in ascending order; returns the count.
 * Spatial: {0..min(S,n)-1} U {max(S, n-W)..n-1}; under Algorithm 2 the window starts at max(S, n_c-W)
 * with n_c the token count at the last compression.
 * Semantic: Heavy U Staged (every heavy position is older than every staged
 * one, and both lists are kept ascending).
 */
int ssd_oracle_unit_retained(const ssd_oracle_unit *u, int32_t *pos_out)
{
    int c = 0, p;
    if (!u->is_semantic) {
        int s_end = u->S < u->n ? u->S : u->n;
        int w_begin = (u->buffered ? u->n_c : u->n) - u->W;
        if (w_begin < u->S) w_begin = u->S;
        for (p = 0; p < s_end; ++p) pos_out[c++] = p;
        for (p = w_begin; p < u->n; ++p) pos_out[c++] = p;
        return c;
    }
    for (p = 0; p < u->n_heavy; ++p) pos_out[c++] = u->heavy_pos[p];
    for (p = 0; p < u->n_staged; ++p) pos_out[c++] = u->staged_pos[p];
    return c;
}

int ssd_oracle_unit_max_retained(const ssd_oracle_unit *u)
{
    return u->is_semantic ? u->M + u->staged_cap : u->S + u->W + (u->buffered ? u->C : 0);
}

/*
 * Attention of q[d] over the retained rows of the dense K, V ([>= n, d]),
 * ascending position.  o_out[d]; p_out (may be NULL) gets the probabilities
 * aligned with ssd_oracle_unit_retained.  For a semantic head with
 * accumulate != 0: score[j] = (float)(score[j] + (float)p_j) for every
 * retained j (running sum of post-softmax probabilities, Algorithm 1).
 * Returns the number of rows attended.
 */
int ssd_oracle_unit_attend(ssd_oracle_unit *u, const float *q, const float *K,
                           const float *V, int d, double scale, int accumulate,
                           float *o_out, float *p_out)
{
    int cap = ssd_oracle_unit_max_retained(u) + 1;
    int32_t *rows = (int32_t *)malloc(sizeof(int32_t) * (size_t)cap);
    float *p = (float *)malloc(sizeof(float) * (size_t)cap);
    int n_rows = ssd_oracle_unit_retained(u, rows);
    int j;
    ssd_oracle_attend(q, K, V, d, rows, n_rows, scale, o_out, p, NULL);
    if (u->is_semantic && accumulate) {
        for (j = 0; j < u->n_heavy; ++j)
            u->heavy_score[j] = (float)(u->heavy_score[j] + p[j]);
        for (j = 0; j < u->n_staged; ++j)
            u->staged_score[j] = (float)(u->staged_score[j] + p[u->n_heavy + j]);
    }
    if (p_out) memcpy(p_out, p, sizeof(float) * (size_t)n_rows);
    free(rows);
    free(p);
    return n_rows;
}

/*
 * Compression of a semantic head: candidates = Heavy U (Staged minus its R
 * newest); Heavy := top-M of the candidates; Staged := its R newest (scores
 * kept).  Spatial heads: nothing to do.  *gap_out as in ssd_oracle_top_m.
 * Returns the new heavy count.
 */
int ssd_oracle_unit_compress(ssd_oracle_unit *u, double *gap_out)
{
    int n_old, n_cand, i, kept, keep_recent;
    float *cs; int32_t *cp, *keep;
    if (gap_out) *gap_out = -1.0;
    if (!u->is_semantic) {
        if (u->buffered) {          /* re-cut the window, empty the row buffer down to the R newest */
            u->n_c = u->n;
            if (u->n_buf > u->R) u->n_buf = u->R;
        }
        return 0;
    }
    keep_recent = u->R < u->n_staged ? u->R : u->n_staged;
    n_old = u->n_staged - keep_recent;          /* staged tokens that become candidates */
    if (n_old <= 0) return u->n_heavy;
    n_cand = u->n_heavy + n_old;
    cs = (float *)malloc(sizeof(float) * (size_t)n_cand);
    cp = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_cand);
    keep = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_cand);
    for (i = 0; i < u->n_heavy; ++i) { cs[i] = u->heavy_score[i]; cp[i] = u->heavy_pos[i]; }
    for (i = 0; i < n_old; ++i) { cs[u->n_heavy + i] = u->staged_score[i]; cp[u->n_heavy + i] = u->staged_pos[i]; }
    kept = ssd_oracle_top_m(cs, cp, n_cand, u->M, keep, gap_out);
    for (i = 0; i < kept; ++i) { u->heavy_pos[i] = cp[keep[i]]; u->heavy_score[i] = cs[keep[i]]; }
    u->n_heavy = kept;
    for (i = 0; i < keep_recent; ++i) {
        u->staged_pos[i] = u->staged_pos[n_old + i];
        u->staged_score[i] = u->staged_score[n_old + i];
    }
    u->n_staged = keep_recent;
    free(cs); free(cp); free(keep);
    return kept;
}

/*
 * Build the compressed state from a dense segment of n_src tokens with
 * accumulated scores score_src[n_src] (NULL = zeros): Heavy = {}, Staged =
 * {0..n_src-1}, then one compression (the prefill branch of Algorithm 2).
 */
int ssd_oracle_unit_load_dense(ssd_oracle_unit *u, int n_src,
                               const float *score_src, double *gap_out)
{
    int i;
    u->n = n_src;
    if (!u->is_semantic) {
        u->n_c = n_src;
        u->n_buf = u->R < n_src ? u->R : n_src;
        return 0;
    }
    staged_reserve(u, n_src > 0 ? n_src : 1);
    u->n_heavy = 0;
    u->n_staged = n_src;
    for (i = 0; i < n_src; ++i) {
        u->staged_pos[i] = i;
        u->staged_score[i] = score_src ? score_src[i] : 0.0f;
    }
    return ssd_oracle_unit_compress(u, gap_out);
}

/* Copy out the semantic state (positions ascending in each list). */
void ssd_oracle_unit_state(const ssd_oracle_unit *u, int32_t *heavy_pos,
                           float *heavy_score, int32_t *n_heavy,
                           int32_t *staged_pos, float *staged_score,
                           int32_t *n_staged)
{
    int i;
    *n_heavy = u->n_heavy;
    *n_staged = u->n_staged;
    for (i = 0; i < u->n_heavy; ++i) { heavy_pos[i] = u->heavy_pos[i]; heavy_score[i] = u->heavy_score[i]; }
    for (i = 0; i < u->n_staged; ++i) { staged_pos[i] = u->staged_pos[i]; staged_score[i] = u->staged_score[i]; }
}

/*
 * Decode positions [p_begin, p_end) of one (layer, sequence, head): for each
 * position p, append, attend with query row p of q over the retained rows of
 * K, V (all [>= p_end, d]), and compress when compress_after[p] != 0.
 *   o_out      [p_end - p_begin, d]
 *   heavy_log  [p_end - p_begin, M] retained heavy positions after step p
 *              (ascending, -1 padded), may be NULL
 *   gap_log    [p_end - p_begin] relative score margin of that step's cut
 *              (-1 if no cut happened), may be NULL
 * Returns 0, or -(p+1) if the row buffer overflowed at position p.
 */
int ssd_oracle_unit_run(ssd_oracle_unit *u, int d, int p_begin, int p_end,
                        const float *q, const float *K, const float *V,
                        double scale, const uint8_t *compress_after,
                        int accumulate, float *o_out, int32_t *heavy_log,
                        double *gap_log)
{
    int p, i;
    if (u->n != p_begin) return -(p_begin + 1);
    for (p = p_begin; p < p_end; ++p) {
        double gap = -1.0;
        size_t r = (size_t)(p - p_begin);
        if (ssd_oracle_unit_append(u) != 0) return -(p + 1);
        ssd_oracle_unit_attend(u, q + (size_t)p * (size_t)d, K, V, d, scale,
                               accumulate, o_out + r * (size_t)d, NULL);
        if (compress_after[p]) ssd_oracle_unit_compress(u, &gap);
        if (gap_log) gap_log[r] = gap;
        if (heavy_log && u->is_semantic) {
            for (i = 0; i < u->M; ++i)
                heavy_log[r * (size_t)u->M + i] = i < u->n_heavy ? u->heavy_pos[i] : -1;
        }
    }
    return 0;
}
