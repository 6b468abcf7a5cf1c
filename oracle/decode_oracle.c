/*
 * CPU oracle for one continuous-batching decode step of a decoder-only
 * transformer over a block-table KV pool.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU path is checked against.  It shares no code with the GPU path and must
 * never be linked into, imported by, or called from it.
 *
 * What it follows.  The paper's continuous-batching scheduler (Algorithm 1)
 * advances every active request by one token per iteration, each against its
 * own KV cache; its text prefix cache (Algorithm 2) hands a request a cached KV
 * state plus a start position.  The paper leaves the token-generation function
 * to the model library, so the arithmetic below is the public definition of the
 * Qwen3 / Llama-3 decoder families whose shapes the workloads take: RMSNorm,
 * grouped-query attention with half-split rotary embedding (optionally per-head
 * RMSNorm of q and k before the rotation), SwiGLU MLP or a softmax top-k
 * mixture of SwiGLU experts, final norm, lm_head, greedy argmax.
 *
 * Style.  Every stage is the textbook formula written as loops: all scores are
 * materialised, the maximum is subtracted, exponentials are divided by their
 * sum.  No blocking, no online softmax, no fusion.  Arithmetic is in `real`
 * (double unless built with -DORC_REAL_FLOAT); weights and cached K/V are read
 * as bf16 bit patterns, converted exactly.  Appended K/V are rounded to bf16
 * from their float32 value (round to nearest even), the precision in which the
 * GPU path takes the same decision.  The sequences of a batch are processed
 * one after another; there is no batch dimension in the arithmetic.  OpenMP
 * only spreads independent output rows / heads over threads.
 *
 * Parity pins: tests/test_oracle_*.py check every function here against closed
 * forms, invariants, brute force and library routines (numpy / torch CPU fp64).
 * Unpinned: agreement of the conventions (rotary pairing, q/k norm order) with
 * a trained checkpoint - none is available, so "parity unpinned" for that.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef ORC_REAL_FLOAT
typedef float real;
#define R_SQRT sqrtf
#define R_EXP expf
#else
typedef double real;
#define R_SQRT sqrt
#define R_EXP exp
#endif

typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    int32_t qk_norm, n_experts, top_k, expert_ffn;
    double rms_eps, rope_theta;
} orc_config;

/* bf16 bit patterns; matrices are W[out][in] row-major, y = W x. */
typedef struct {
    const uint16_t *g_attn;                 /* [H]                            */
    const uint16_t *wq, *wk, *wv;           /* [nq*d,H] [nkv*d,H] [nkv*d,H]   */
    const uint16_t *g_q, *g_k;              /* [d] each, or NULL              */
    const uint16_t *wo;                     /* [H, nq*d]                      */
    const uint16_t *g_mlp;                  /* [H]                            */
    const uint16_t *w_gate, *w_up, *w_down; /* dense [F,H] [F,H] [H,F];
                                               MoE [E,Fe,H] [E,Fe,H] [E,H,Fe] */
    const uint16_t *w_router;               /* [E,H] or NULL                  */
} orc_layer;

int orc_real_bytes(void) { return (int)sizeof(real); }

/* ---------------------------------------------------------------- bf16 -- */

static inline float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* float32 -> bf16, round to nearest, ties to even.  NaN stays NaN. */
static inline uint16_t f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lower = u & 0xffffu;
    uint32_t upper = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u)))
        upper += 1;
    return (uint16_t)upper;
}

void orc_bf16_to_f32(const uint16_t *in, int64_t n, float *out)
{
    for (int64_t i = 0; i < n; i++) out[i] = bf16_to_f32(in[i]);
}

void orc_f32_to_bf16(const float *in, int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; i++) out[i] = f32_to_bf16(in[i]);
}

/* ------------------------------------------------------------- RMSNorm -- */
/* out_i = x_i / sqrt(mean(x^2) + eps) * gain_i */
static void rmsnorm(const real *x, int n, const uint16_t *gain, real eps, real *out)
{
    real ss = 0;
    for (int i = 0; i < n; i++) ss += x[i] * x[i];
    real inv = (real)1 / R_SQRT(ss / (real)n + eps);
    for (int i = 0; i < n; i++) out[i] = x[i] * inv * (real)bf16_to_f32(gain[i]);
}

/* ------------------------------------------------------ matrix * vector -- */
/* y_r = sum_k W[r][k] x_k */
static void matvec(const uint16_t *W, int64_t rows, int64_t cols, const real *x, real *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; r++) {
        const uint16_t *w = W + r * cols;
        real acc = 0;
        for (int64_t k = 0; k < cols; k++) acc += (real)bf16_to_f32(w[k]) * x[k];
        y[r] = acc;
    }
}

/* ------------------------------------- 4-bit weights (group-wise affine) -- */
/*
 * The precision the paper benchmarks (4-bit MLX checkpoints): every row is cut
 * into groups of 64 consecutive columns; a group has 64 codes q in 0..15 and a
 * bf16 scale and bias, and stands for the weights  scale * q + bias.  The
 * matrix-vector product is the plain definition with those weights:
 *   y_r = sum_k (scale[r][k/64] * q[r][k] + bias[r][k/64]) * x_k
 * Canonical form: q uint8 [rows][cols], scale / bias bf16 bits [rows][cols/64].
 */
typedef struct {
    const uint8_t *q;
    const uint16_t *scale, *bias;
} orc_q4;

static void matvec_q4(const orc_q4 *m, int64_t rows, int64_t cols, const real *x, real *y)
{
    const int64_t groups = cols / 64;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; r++) {
        real acc = 0;
        for (int64_t k = 0; k < cols; k++) {
            const real w = (real)bf16_to_f32(m->scale[r * groups + k / 64]) * (real)m->q[r * cols + k] +
                           (real)bf16_to_f32(m->bias[r * groups + k / 64]);
            acc += w * x[k];
        }
        y[r] = acc;
    }
}

/* One projection of a layer: the 4-bit matrix if the model has them, else the bf16 one. */
static void project(const uint16_t *w_bf16, const orc_q4 *w_q4, int64_t rows, int64_t cols, const real *x, real *y)
{
    if (w_q4) matvec_q4(w_q4, rows, cols, x, y);
    else matvec(w_bf16, rows, cols, x, y);
}

/* --------------------------------------------------------------- RoPE --- */
/* Half-split rotary embedding of one head at position pos: element i is
 * paired with element i + d/2 and the pair is rotated by pos * theta^(-2i/d). */
static void rope(real *v, int d, int pos, double theta)
{
    int half = d / 2;
    for (int i = 0; i < half; i++) {
        double inv_freq = pow(theta, -2.0 * (double)i / (double)d);
        double ang = (double)pos * inv_freq;
        real c = (real)cos(ang), s = (real)sin(ang);
        real a = v[i], b = v[i + half];
        v[i] = a * c - b * s;
        v[i + half] = b * c + a * s;
    }
}

/* --------------------------------------------------------- pool layout -- */
/* pool[layer][block][kv][kv_head][slot][dim], kv: 0 = K, 1 = V. */
int64_t orc_pool_offset(const orc_config *c, int32_t num_blocks, int32_t block_size,
                        int32_t layer, int32_t block, int32_t kv, int32_t head,
                        int32_t slot, int32_t dim)
{
    int64_t o = layer;
    o = o * num_blocks + block;
    o = o * 2 + kv;
    o = o * c->n_kv_heads + head;
    o = o * block_size + slot;
    o = o * c->head_dim + dim;
    return o;
}

/* Store one token's K and V (all kv heads) of one layer at logical position
 * pos of the sequence whose block table row is `table`. */
static void append_kv(const orc_config *c, uint16_t *pool, int32_t num_blocks,
                      int32_t block_size, int32_t layer, const int32_t *table,
                      int32_t pos, const real *k, const real *v)
{
    int32_t block = table[pos / block_size];
    int32_t slot = pos % block_size;
    for (int j = 0; j < c->n_kv_heads; j++)
        for (int i = 0; i < c->head_dim; i++) {
            pool[orc_pool_offset(c, num_blocks, block_size, layer, block, 0, j, slot, i)] =
                f32_to_bf16((float)k[j * c->head_dim + i]);
            pool[orc_pool_offset(c, num_blocks, block_size, layer, block, 1, j, slot, i)] =
                f32_to_bf16((float)v[j * c->head_dim + i]);
        }
}

/* ------------------------------------------------------------- softmax -- */
static void softmax(const real *s, int n, real *p)
{
    real m = s[0];
    for (int i = 1; i < n; i++) if (s[i] > m) m = s[i];
    real sum = 0;
    for (int i = 0; i < n; i++) { p[i] = R_EXP(s[i] - m); sum += p[i]; }
    for (int i = 0; i < n; i++) p[i] = p[i] / sum;
}

/* ----------------------------------------------------------- attention -- */
/* Grouped-query attention of one new token over logical positions
 * 0..n_tokens-1 of its sequence, read through the block table.  q is
 * [nq][d]; query head h uses kv head h / (nq/nkv).  probs_out (optional) is
 * [nq][n_tokens]. */
static void attention(const orc_config *c, const uint16_t *pool, int32_t num_blocks,
                      int32_t block_size, int32_t layer, const int32_t *table,
                      int32_t n_tokens, const real *q, real *out, real *probs_out)
{
    int d = c->head_dim, G = c->n_q_heads / c->n_kv_heads;
    real scale = (real)1 / R_SQRT((real)d);
#pragma omp parallel for schedule(static)
    for (int h = 0; h < c->n_q_heads; h++) {
        int j = h / G;
        real *s = (real *)malloc(sizeof(real) * (size_t)n_tokens);
        real *p = (real *)malloc(sizeof(real) * (size_t)n_tokens);
        for (int t = 0; t < n_tokens; t++) {
            const uint16_t *kr = pool + orc_pool_offset(c, num_blocks, block_size, layer,
                                                        table[t / block_size], 0, j,
                                                        t % block_size, 0);
            real acc = 0;
            for (int i = 0; i < d; i++) acc += q[h * d + i] * (real)bf16_to_f32(kr[i]);
            s[t] = acc * scale;
        }
        softmax(s, n_tokens, p);
        for (int i = 0; i < d; i++) out[h * d + i] = 0;
        for (int t = 0; t < n_tokens; t++) {
            const uint16_t *vr = pool + orc_pool_offset(c, num_blocks, block_size, layer,
                                                        table[t / block_size], 1, j,
                                                        t % block_size, 0);
            for (int i = 0; i < d; i++) out[h * d + i] += p[t] * (real)bf16_to_f32(vr[i]);
        }
        if (probs_out) memcpy(probs_out + (size_t)h * n_tokens, p, sizeof(real) * (size_t)n_tokens);
        free(s);
        free(p);
    }
}

/* ---------------------------------------------------------------- MLPs -- */
static inline real silu(real z) { return z / ((real)1 + R_EXP(-z)); }

/* out = Wd (silu(Wg h) * (Wu h)) with Wg, Wu [F,H], Wd [H,F] */
static void swiglu_any(const uint16_t *wg, const uint16_t *wu, const uint16_t *wd,
                       const orc_q4 *qg, const orc_q4 *qu, const orc_q4 *qd,
                       int H, int F, const real *h, real *out)
{
    real *g = (real *)malloc(sizeof(real) * (size_t)F);
    real *u = (real *)malloc(sizeof(real) * (size_t)F);
    project(wg, qg, F, H, h, g);
    project(wu, qu, F, H, h, u);
    for (int i = 0; i < F; i++) g[i] = silu(g[i]) * u[i];
    project(wd, qd, H, F, g, out);
    free(g);
    free(u);
}

static void swiglu(const uint16_t *wg, const uint16_t *wu, const uint16_t *wd,
                   int H, int F, const real *h, real *out)
{
    swiglu_any(wg, wu, wd, NULL, NULL, NULL, H, F, h, out);
}

/* Near-ties of the router.  The top-k choice is an integer decided by floating
 * point: where the k-th and the (k+1)-th probability are closer than the arithmetic
 * of the path under test resolves, another choice is as correct as this file's own,
 * and everything after it (expert outputs, the cached k/v of later layers, the
 * logits) follows that choice.  A test may therefore PROPOSE an expert set for a
 * (layer, sequence).  route() adopts a proposal only if it is itself a valid top-k
 * set up to the relative tolerance `tol`: k distinct experts, each with a
 * probability of at least (1 - tol) times the largest probability left out.
 * Anything else is ignored and this file's own choice stands.  With no proposal
 * (every caller but that test) nothing changes. */
typedef struct {
    const int32_t *proposal;   /* [n_layers][B][top_k] or NULL */
    double tol;
    int32_t *adopted;          /* [n_layers][B] out: 1 where a differing proposal was adopted */
    double *margin;            /* [n_layers][B] out: (largest left out - smallest proposed) / largest
                                  left out, where the proposal differed from the own choice; else 0 */
} orc_tie;

/* Router: softmax over all experts, the top_k largest probabilities (ties to
 * the lower expert index), renormalised to sum to one.  proposal / tol /
 * adopted / margin: see orc_tie (proposal NULL: the plain definition). */
static void route(const orc_config *c, const uint16_t *w_router, const real *h,
                  int32_t *idx, real *wts, const int32_t *proposal, double tol,
                  int32_t *adopted, double *margin)
{
    int E = c->n_experts, K = c->top_k;
    real *logit = (real *)malloc(sizeof(real) * (size_t)E);
    real *prob = (real *)malloc(sizeof(real) * (size_t)E);
    char *taken = (char *)calloc((size_t)E, 1);
    matvec(w_router, E, c->hidden, h, logit);
    softmax(logit, E, prob);
    for (int k = 0; k < K; k++) {
        int best = -1;
        for (int e = 0; e < E; e++)
            if (!taken[e] && (best < 0 || prob[e] > prob[best])) best = e;
        taken[best] = 1;
        idx[k] = best;
    }
    if (adopted) *adopted = 0;
    if (margin) *margin = 0;
    if (proposal) {
        /* is the proposal a set of K distinct experts other than the own choice? */
        char *in = (char *)calloc((size_t)E, 1);
        int ok = 1, same = 1;
        for (int k = 0; k < K; k++) {
            int e = proposal[k];
            if (e < 0 || e >= E || in[e]) { ok = 0; break; }
            in[e] = 1;
            if (!taken[e]) same = 0;
        }
        if (ok && !same) {
            real pmin = 0, pout = 0;
            int first = 1, any_out = 0;
            for (int e = 0; e < E; e++) {
                if (in[e]) { if (first || prob[e] < pmin) pmin = prob[e]; first = 0; }
                else if (!any_out || prob[e] > pout) { pout = prob[e]; any_out = 1; }
            }
            double m = any_out && pout > 0 ? (double)(pout - pmin) / (double)pout : 0.0;
            if (margin) *margin = m;
            if (m <= tol) {
                /* adopt: the proposed experts, largest probability first (ties to the lower index) */
                memset(taken, 0, (size_t)E);
                for (int k = 0; k < K; k++) {
                    int best = -1;
                    for (int e = 0; e < E; e++)
                        if (in[e] && !taken[e] && (best < 0 || prob[e] > prob[best])) best = e;
                    taken[best] = 1;
                    idx[k] = best;
                }
                if (adopted) *adopted = 1;
            }
        }
        free(in);
    }
    real sum = 0;
    for (int k = 0; k < K; k++) { wts[k] = prob[idx[k]]; sum += wts[k]; }
    for (int k = 0; k < K; k++) wts[k] = wts[k] / sum;
    free(logit);
    free(prob);
    free(taken);
}

/* qg / qu / qd: NULL, or the 4-bit gate / up / down matrices of ALL experts stacked by rows
 * (expert e owns rows e*Fe.. of gate and up, rows e*H.. of down); the router stays bf16. */
static void moe_any(const orc_config *c, const orc_layer *L, const orc_q4 *qg, const orc_q4 *qu, const orc_q4 *qd,
                    const real *h, real *out, int32_t *idx_out, real *wts_out,
                    const int32_t *proposal, double tol, int32_t *adopted, double *margin)
{
    int H = c->hidden, Fe = c->expert_ffn, K = c->top_k;
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
    real *wts = (real *)malloc(sizeof(real) * (size_t)K);
    real *y = (real *)malloc(sizeof(real) * (size_t)H);
    route(c, L->w_router, h, idx, wts, proposal, tol, adopted, margin);
    for (int i = 0; i < H; i++) out[i] = 0;
    for (int k = 0; k < K; k++) {
        int64_t e = idx[k];
        if (qg) {
            /* expert e's rows of the stacked matrices */
            const orc_q4 g = {qg->q + e * Fe * H, qg->scale + e * Fe * (H / 64), qg->bias + e * Fe * (H / 64)};
            const orc_q4 u = {qu->q + e * Fe * H, qu->scale + e * Fe * (H / 64), qu->bias + e * Fe * (H / 64)};
            const orc_q4 d = {qd->q + e * H * Fe, qd->scale + e * H * (Fe / 64), qd->bias + e * H * (Fe / 64)};
            swiglu_any(NULL, NULL, NULL, &g, &u, &d, H, Fe, h, y);
        } else {
            swiglu(L->w_gate + e * Fe * H, L->w_up + e * Fe * H, L->w_down + e * H * Fe, H, Fe, h, y);
        }
        for (int i = 0; i < H; i++) out[i] += wts[k] * y[i];
    }
    if (idx_out) memcpy(idx_out, idx, sizeof(int32_t) * (size_t)K);
    if (wts_out) memcpy(wts_out, wts, sizeof(real) * (size_t)K);
    free(idx);
    free(wts);
    free(y);
}

static void moe(const orc_config *c, const orc_layer *L, const real *h, real *out,
                int32_t *idx_out, real *wts_out)
{
    moe_any(c, L, NULL, NULL, NULL, h, out, idx_out, wts_out, NULL, 0.0, NULL, NULL);
}

/* -------------------------------------------------------------- argmax -- */
/* Index of the largest value; the lowest index among equal maxima. */
int32_t orc_argmax_f32(const float *v, int32_t n)
{
    int32_t best = 0;
    for (int32_t i = 1; i < n; i++) if (v[i] > v[best]) best = i;
    return best;
}

/* ------------------------------------------------------------ sampling -- */
/*
 * The paper does not describe its sampler.  The definition used here:
 *   s_i = logit_i / T,  p_i = exp(s_i - max s);
 *   top-k (0 < k < n): candidates = every i with p_i >= the k-th largest p;
 *   top-p (p < 1): sort the candidates' p in descending order, take values until
 *     their running sum reaches p * (sum over the candidates); the kept set is
 *     every candidate with p_i >= the last value taken;
 *   draw: r = u * (sum over the kept set), the first kept index, in ascending
 *     index order, whose running sum exceeds r.
 * Plain double arithmetic, a full sort.
 */
static int cmp_desc(const void *a, const void *b)
{
    const double x = *(const double *)a, y = *(const double *)b;
    return (x < y) - (x > y);
}

int32_t orc_sample(const float *logits, int32_t n, double temperature, int32_t top_k, double top_p, double u)
{
    double *p = (double *)malloc(sizeof(double) * (size_t)n);
    double *sorted = (double *)malloc(sizeof(double) * (size_t)n);
    double mx = -INFINITY;
    for (int32_t i = 0; i < n; i++) { const double s = (double)logits[i] / temperature; if (s > mx) mx = s; }
    for (int32_t i = 0; i < n; i++) { p[i] = exp((double)logits[i] / temperature - mx); sorted[i] = p[i]; }
    qsort(sorted, (size_t)n, sizeof(double), cmp_desc);
    double tau = 0.0;
    int32_t ncand = n;
    if (top_k > 0 && top_k < n) {
        tau = sorted[top_k - 1];
        while (ncand > 0 && sorted[ncand - 1] < tau) ncand--;      /* candidates: the sorted prefix >= tau */
    }
    if (top_p < 1.0) {
        double z = 0.0, run = 0.0;
        for (int32_t i = 0; i < ncand; i++) z += sorted[i];
        for (int32_t i = 0; i < ncand; i++) {
            run += sorted[i];
            if (run >= top_p * z) { tau = sorted[i]; break; }
        }
    }
    double total = 0.0;
    int32_t last = 0;
    for (int32_t i = 0; i < n; i++) if (p[i] >= tau) { total += p[i]; last = i; }
    const double r = u * total;
    double run = 0.0;
    int32_t pick = last;
    for (int32_t i = 0; i < n; i++)
        if (p[i] >= tau) { run += p[i]; if (run > r) { pick = i; break; } }
    free(p); free(sorted);
    return pick;
}

/* Philox4x32-10 (Salmon et al., "Parallel random numbers: as easy as 1, 2, 3"). */
void orc_philox4x32_10(const uint32_t counter[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = counter[0], c1 = counter[1], c2 = counter[2], c3 = counter[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; r++) {
        const uint64_t a = (uint64_t)0xD2511F53u * c0, b = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(b >> 32) ^ c1 ^ k0, n1 = (uint32_t)b;
        const uint32_t n2 = (uint32_t)(a >> 32) ^ c3 ^ k1, n3 = (uint32_t)a;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The uniform number of (seed, step, row): 24 bits of the first Philox word. */
double orc_sample_uniform(uint64_t seed, uint64_t step, uint32_t row)
{
    const uint32_t ctr[4] = {(uint32_t)step, (uint32_t)(step >> 32), row, 0u};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return (double)(out[0] >> 8) / 16777216.0;
}

/* ---------------------------------------------------- one decode step --- */
/*
 * For each sequence b (independently): embed tokens[b]; for every layer
 * normalise, project to q,k,v, (q/k head norm,) rotate q and k at position
 * seq_lens[b], store k,v (bf16) at that position through the block table,
 * attend over positions 0..seq_lens[b], project, add; normalise, MLP / MoE,
 * add; final norm, lm_head, argmax.  seq_lens and block tables are not
 * modified.  The pool is modified (one token per layer per sequence).
 *
 * logits: float32 [B][vocab] or NULL.  next_tokens: int32 [B].
 * trace_x (optional): float32 [n_layers+1][B][hidden], residual stream after
 * the embedding and after each layer.
 * trace_experts (optional, MoE): int32 [n_layers][B][top_k] chosen experts.
 * Returns 0, or a negative value for an invalid argument.
 */
/* q4: NULL (bf16 weights), or the model's 4-bit matrices, seven per layer in
 * the order wq wk wv wo w_gate w_up w_down, then lm_head; the bf16 pointers of
 * those matrices are then not read (norm gains and the embedding stay bf16). */
enum { Q4_WQ, Q4_WK, Q4_WV, Q4_WO, Q4_GATE, Q4_UP, Q4_DOWN, Q4_PER_LAYER };

static int decode_step_body(const orc_config *c, const orc_layer *layers, const orc_q4 *q4,
                            const uint16_t *embed, const uint16_t *g_final, const uint16_t *lm_head,
                            uint16_t *pool, int32_t num_blocks, int32_t block_size,
                            const int32_t *block_tables, int32_t max_blocks_per_seq,
                            const int32_t *seq_lens, const int32_t *tokens, int32_t B,
                            float *logits, int32_t *next_tokens, float *trace_x,
                            int32_t *trace_experts, const orc_tie *tie)
{
    int H = c->hidden, d = c->head_dim, nq = c->n_q_heads, nkv = c->n_kv_heads;
    int V = c->vocab;
    if (nq % nkv || d % 2 || B < 0) return -1;
    for (int b = 0; b < B; b++) {
        if (tokens[b] < 0 || tokens[b] >= V) return -2;
        if (seq_lens[b] < 0 || seq_lens[b] / block_size >= max_blocks_per_seq) return -3;
        for (int t = 0; t <= seq_lens[b]; t += block_size) {
            int32_t id = block_tables[(int64_t)b * max_blocks_per_seq + t / block_size];
            if (id < 0 || id >= num_blocks) return -4;
        }
    }
    real *x = (real *)malloc(sizeof(real) * (size_t)H);
    real *h = (real *)malloc(sizeof(real) * (size_t)H);
    real *q = (real *)malloc(sizeof(real) * (size_t)(nq * d));
    real *k = (real *)malloc(sizeof(real) * (size_t)(nkv * d));
    real *v = (real *)malloc(sizeof(real) * (size_t)(nkv * d));
    real *o = (real *)malloc(sizeof(real) * (size_t)(nq * d));
    real *y = (real *)malloc(sizeof(real) * (size_t)H);
    real *lg = (real *)malloc(sizeof(real) * (size_t)V);
    float *lgf = (float *)malloc(sizeof(float) * (size_t)V);
    real *tmp = (real *)malloc(sizeof(real) * (size_t)d);

    for (int b = 0; b < B; b++) {
        const int32_t *table = block_tables + (int64_t)b * max_blocks_per_seq;
        int pos = seq_lens[b];
        for (int i = 0; i < H; i++) x[i] = (real)bf16_to_f32(embed[(int64_t)tokens[b] * H + i]);
        if (trace_x)
            for (int i = 0; i < H; i++) trace_x[((int64_t)0 * B + b) * H + i] = (float)x[i];

        for (int l = 0; l < c->n_layers; l++) {
            const orc_layer *L = &layers[l];
            const orc_q4 *Q = q4 ? q4 + (int64_t)l * Q4_PER_LAYER : NULL;
            rmsnorm(x, H, L->g_attn, (real)c->rms_eps, h);
            project(L->wq, Q ? Q + Q4_WQ : NULL, (int64_t)nq * d, H, h, q);
            project(L->wk, Q ? Q + Q4_WK : NULL, (int64_t)nkv * d, H, h, k);
            project(L->wv, Q ? Q + Q4_WV : NULL, (int64_t)nkv * d, H, h, v);
            if (c->qk_norm) {
                for (int hh = 0; hh < nq; hh++) {
                    rmsnorm(q + hh * d, d, L->g_q, (real)c->rms_eps, tmp);
                    memcpy(q + hh * d, tmp, sizeof(real) * (size_t)d);
                }
                for (int j = 0; j < nkv; j++) {
                    rmsnorm(k + j * d, d, L->g_k, (real)c->rms_eps, tmp);
                    memcpy(k + j * d, tmp, sizeof(real) * (size_t)d);
                }
            }
            for (int hh = 0; hh < nq; hh++) rope(q + hh * d, d, pos, c->rope_theta);
            for (int j = 0; j < nkv; j++) rope(k + j * d, d, pos, c->rope_theta);
            append_kv(c, pool, num_blocks, block_size, l, table, pos, k, v);
            attention(c, pool, num_blocks, block_size, l, table, pos + 1, q, o, NULL);
            project(L->wo, Q ? Q + Q4_WO : NULL, H, (int64_t)nq * d, o, y);
            for (int i = 0; i < H; i++) x[i] += y[i];

            rmsnorm(x, H, L->g_mlp, (real)c->rms_eps, h);
            if (c->n_experts > 0)
                moe_any(c, L, Q ? Q + Q4_GATE : NULL, Q ? Q + Q4_UP : NULL, Q ? Q + Q4_DOWN : NULL, h, y,
                        trace_experts ? trace_experts + ((int64_t)l * B + b) * c->top_k : NULL, NULL,
                        tie && tie->proposal ? tie->proposal + ((int64_t)l * B + b) * c->top_k : NULL,
                        tie ? tie->tol : 0.0, tie && tie->adopted ? tie->adopted + (int64_t)l * B + b : NULL,
                        tie && tie->margin ? tie->margin + (int64_t)l * B + b : NULL);
            else
                swiglu_any(L->w_gate, L->w_up, L->w_down, Q ? Q + Q4_GATE : NULL, Q ? Q + Q4_UP : NULL,
                           Q ? Q + Q4_DOWN : NULL, H, c->ffn, h, y);
            for (int i = 0; i < H; i++) x[i] += y[i];
            if (trace_x)
                for (int i = 0; i < H; i++)
                    trace_x[((int64_t)(l + 1) * B + b) * H + i] = (float)x[i];
        }
        rmsnorm(x, H, g_final, (real)c->rms_eps, h);
        project(lm_head, q4 ? q4 + (int64_t)c->n_layers * Q4_PER_LAYER : NULL, V, H, h, lg);
        for (int i = 0; i < V; i++) lgf[i] = (float)lg[i];
        if (logits) memcpy(logits + (int64_t)b * V, lgf, sizeof(float) * (size_t)V);
        next_tokens[b] = orc_argmax_f32(lgf, V);
    }
    free(x); free(h); free(q); free(k); free(v); free(o); free(y); free(lg); free(lgf); free(tmp);
    return 0;
}

int orc_decode_step(const orc_config *c, const orc_layer *layers,
                    const uint16_t *embed, const uint16_t *g_final, const uint16_t *lm_head,
                    uint16_t *pool, int32_t num_blocks, int32_t block_size,
                    const int32_t *block_tables, int32_t max_blocks_per_seq,
                    const int32_t *seq_lens, const int32_t *tokens, int32_t B,
                    float *logits, int32_t *next_tokens, float *trace_x,
                    int32_t *trace_experts)
{
    return decode_step_body(c, layers, NULL, embed, g_final, lm_head, pool, num_blocks, block_size,
                            block_tables, max_blocks_per_seq, seq_lens, tokens, B, logits,
                            next_tokens, trace_x, trace_experts, NULL);
}

/* orc_decode_step of a mixture-of-experts model with proposed expert sets for the
 * router's near-ties (see orc_tie): proposal int32 [n_layers][B][top_k]; a proposal
 * is adopted only where it is a valid top-k set up to tie_tol; adopted int32
 * [n_layers][B] and margin double [n_layers][B] report what happened. */
int orc_decode_step_tie(const orc_config *c, const orc_layer *layers,
                        const uint16_t *embed, const uint16_t *g_final, const uint16_t *lm_head,
                        uint16_t *pool, int32_t num_blocks, int32_t block_size,
                        const int32_t *block_tables, int32_t max_blocks_per_seq,
                        const int32_t *seq_lens, const int32_t *tokens, int32_t B,
                        float *logits, int32_t *next_tokens, int32_t *trace_experts,
                        const int32_t *proposal, double tie_tol, int32_t *adopted, double *margin)
{
    const orc_tie tie = {proposal, tie_tol, adopted, margin};
    return decode_step_body(c, layers, NULL, embed, g_final, lm_head, pool, num_blocks, block_size,
                            block_tables, max_blocks_per_seq, seq_lens, tokens, B, logits,
                            next_tokens, NULL, trace_experts, &tie);
}

/* The same step for a model with 4-bit projections.  q_ptrs / scale_ptrs /
 * bias_ptrs: n_layers * 7 + 1 pointers each (order as above; canonical form).
 * hidden, n_q_heads * head_dim and ffn (expert_ffn) must be multiples of 64.
 * Mixture-of-experts layers: gate / up / down hold all experts stacked by rows;
 * layers supplies the norm gains and the (bf16) router. */
int orc_decode_step_q4(const orc_config *c, const orc_layer *layers,
                       const uint8_t *const *q_ptrs, const uint16_t *const *scale_ptrs,
                       const uint16_t *const *bias_ptrs,
                       const uint16_t *embed, const uint16_t *g_final,
                       uint16_t *pool, int32_t num_blocks, int32_t block_size,
                       const int32_t *block_tables, int32_t max_blocks_per_seq,
                       const int32_t *seq_lens, const int32_t *tokens, int32_t B,
                       float *logits, int32_t *next_tokens, float *trace_x, int32_t *trace_experts)
{
    const int width = c->n_experts > 0 ? c->expert_ffn : c->ffn;
    if (c->hidden % 64 || (c->n_q_heads * c->head_dim) % 64 || width % 64) return -6;
    const int n = c->n_layers * Q4_PER_LAYER + 1;
    orc_q4 *m = (orc_q4 *)malloc(sizeof(orc_q4) * (size_t)n);
    for (int i = 0; i < n; i++) {
        m[i].q = q_ptrs[i];
        m[i].scale = scale_ptrs[i];
        m[i].bias = bias_ptrs[i];
    }
    int rc = decode_step_body(c, layers, m, embed, g_final, NULL, pool, num_blocks, block_size,
                              block_tables, max_blocks_per_seq, seq_lens, tokens, B, logits,
                              next_tokens, trace_x, trace_experts, NULL);
    free(m);
    return rc;
}

/* ------------------------------------- stage entry points for the tests -- */
/* route() alone, with an optional proposal: idx int32 [top_k], wts double [top_k]. */
void orc_route(const orc_config *c, const uint16_t *w_router, const double *h, int32_t *idx, double *wts,
               const int32_t *proposal, double tol, int32_t *adopted, double *margin);

/* Thin wrappers taking float64 arrays so that each stage can be pinned alone. */

static real *to_real(const double *a, int64_t n)
{
    real *r = (real *)malloc(sizeof(real) * (size_t)(n > 0 ? n : 1));
    for (int64_t i = 0; i < n; i++) r[i] = (real)a[i];
    return r;
}
static void from_real(const real *r, int64_t n, double *a)
{
    for (int64_t i = 0; i < n; i++) a[i] = (double)r[i];
}

void orc_rmsnorm(const double *x, int32_t n, const uint16_t *gain, double eps, double *out)
{
    real *xr = to_real(x, n), *o = (real *)malloc(sizeof(real) * (size_t)n);
    rmsnorm(xr, n, gain, (real)eps, o);
    from_real(o, n, out);
    free(xr); free(o);
}

void orc_matvec(const uint16_t *W, int64_t rows, int64_t cols, const double *x, double *y)
{
    real *xr = to_real(x, cols), *yr = (real *)malloc(sizeof(real) * (size_t)rows);
    matvec(W, rows, cols, xr, yr);
    from_real(yr, rows, y);
    free(xr); free(yr);
}

void orc_matvec_q4(const uint8_t *q, const uint16_t *scale, const uint16_t *bias, int64_t rows,
                   int64_t cols, const double *x, double *y)
{
    const orc_q4 m = {q, scale, bias};
    real *xr = to_real(x, cols), *yr = (real *)malloc(sizeof(real) * (size_t)rows);
    matvec_q4(&m, rows, cols, xr, yr);
    from_real(yr, rows, y);
    free(xr); free(yr);
}

void orc_rope(double *v, int32_t d, int32_t pos, double theta)
{
    real *vr = to_real(v, d);
    rope(vr, d, pos, theta);
    from_real(vr, d, v);
    free(vr);
}

void orc_softmax(const double *s, int32_t n, double *p)
{
    real *sr = to_real(s, n), *pr = (real *)malloc(sizeof(real) * (size_t)n);
    softmax(sr, n, pr);
    from_real(pr, n, p);
    free(sr); free(pr);
}

void orc_append_kv(const orc_config *c, uint16_t *pool, int32_t num_blocks, int32_t block_size,
                   int32_t layer, const int32_t *table, int32_t pos,
                   const double *k, const double *v)
{
    int n = c->n_kv_heads * c->head_dim;
    real *kr = to_real(k, n), *vr = to_real(v, n);
    append_kv(c, pool, num_blocks, block_size, layer, table, pos, kr, vr);
    free(kr); free(vr);
}

void orc_attention(const orc_config *c, const uint16_t *pool, int32_t num_blocks,
                   int32_t block_size, int32_t layer, const int32_t *table, int32_t n_tokens,
                   const double *q, double *out, double *probs_out)
{
    int n = c->n_q_heads * c->head_dim;
    real *qr = to_real(q, n), *o = (real *)malloc(sizeof(real) * (size_t)n);
    real *p = probs_out ? (real *)malloc(sizeof(real) * (size_t)c->n_q_heads * (size_t)n_tokens) : NULL;
    attention(c, pool, num_blocks, block_size, layer, table, n_tokens, qr, o, p);
    from_real(o, n, out);
    if (p) { from_real(p, (int64_t)c->n_q_heads * n_tokens, probs_out); free(p); }
    free(qr); free(o);
}

void orc_swiglu(const uint16_t *wg, const uint16_t *wu, const uint16_t *wd, int32_t H, int32_t F,
                const double *h, double *out)
{
    real *hr = to_real(h, H), *o = (real *)malloc(sizeof(real) * (size_t)H);
    swiglu(wg, wu, wd, H, F, hr, o);
    from_real(o, H, out);
    free(hr); free(o);
}

void orc_moe(const orc_config *c, const orc_layer *L, const double *h, double *out,
             int32_t *idx_out, double *wts_out)
{
    int H = c->hidden;
    real *hr = to_real(h, H), *o = (real *)malloc(sizeof(real) * (size_t)H);
    real *w = (real *)malloc(sizeof(real) * (size_t)c->top_k);
    moe(c, L, hr, o, idx_out, w);
    from_real(o, H, out);
    if (wts_out) from_real(w, c->top_k, wts_out);
    free(hr); free(o); free(w);
}

double orc_silu(double z) { return (double)silu((real)z); }

void orc_route(const orc_config *c, const uint16_t *w_router, const double *h, int32_t *idx, double *wts,
               const int32_t *proposal, double tol, int32_t *adopted, double *margin)
{
    real *hr = (real *)malloc(sizeof(real) * (size_t)c->hidden);
    real *w = (real *)malloc(sizeof(real) * (size_t)c->top_k);
    for (int i = 0; i < c->hidden; i++) hr[i] = (real)h[i];
    route(c, w_router, hr, idx, w, proposal, tol, adopted, margin);
    for (int k = 0; k < c->top_k; k++) wts[k] = (double)w[k];
    free(hr);
    free(w);
}
