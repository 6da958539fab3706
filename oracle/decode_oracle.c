/*
 * decode_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow CPU statement of what one rollout decode step computes: one autoregressive
 * step of a Qwen2-style decoder (RMSNorm, q/k/v projection with bias, rotate-half RoPE,
 * grouped-query attention over a paged KV cache, SwiGLU MLP, LM head, greedy argmax) for a
 * batch of independent sequences.  The paper only characterises this stage (rollout
 * generation is HBM-I/O-bound inference, Section 1 and Section 3 Observation 1; the policy
 * models are distilled Qwen-2.5 at 1.5B/7B/14B, Section 5.2); the arithmetic below is the
 * textbook definition of that decoder, written out naively.
 *
 * Numeric contract ("bf16 in, fp32 accumulate"): weights, the KV cache and every matrix
 * input are bf16 values; all arithmetic is fp32, sums run in ascending index order; an
 * activation is rounded to bf16 (round-to-nearest-even) at exactly these points: the input of
 * each of the five matrix products, the rotated query, and K / V on entering the cache.  With
 * round_act = 0 those roundings are skipped (used only to compare with fp32 library code).
 * With kv_fp8 = 1, K and V enter the cache rounded to the 8-bit format E4M3 instead (a later variant
 * that halves the dominant byte term; everything else is unchanged).
 *
 * Nothing here is blocked, fused, tiled or reordered.  It shares no code, table or header
 * with the GPU library.  Only tests, the smoke check and the benchmark's CPU-baseline leg call
 * it.  Built with -DORC_SUM_DESCENDING every sum of the step (matrix products, the norm's mean of squares, the
 * score dot products, the softmax denominator, the probability-weighted sum of V) adds its terms in descending
 * instead of ascending index order: an equally valid fp32 evaluation of the same definition, used only to measure
 * how far two correct implementations drift apart.
 * Parity status: every function is pinned by tests/test_oracle_*.py against closed
 * forms, invariants, numpy / torch library routines and brute-force recomputation; the paper
 * prints no worked numbers for this stage, so there is no golden value from it.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, intermediate, vocab, block_size;
    int32_t qkv_bias;  /* 1: add the q/k/v bias                                   */
    int32_t round_act; /* 1: bf16 rounding points on (the contract); 0: pure fp32 */
    int32_t kv_fp8;    /* 1: K and V enter the cache as 8-bit floats (E4M3), see orc_e4m3_round */
    float rms_eps, rope_theta;
} orc_config;

/* bf16 tensors of one layer, logical row-major [in, out] */
typedef struct {
    const uint16_t *g1, *wqkv, *bqkv, *wo, *g2, *wg, *wu, *wd;
} orc_layer;

typedef struct {
    const uint16_t *embed; /* [vocab, hidden] */
    const uint16_t *gf;    /* [hidden]        */
    const uint16_t *wlm;   /* [hidden, vocab] */
    const orc_layer *layers;
} orc_weights;

/* ---- bf16 <-> fp32 --------------------------------------------------------------------- */

float orc_bf16_to_f32(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round-to-nearest, ties to even, on the upper 16 bits of the fp32 pattern */
uint16_t orc_f32_to_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u); /* NaN stays NaN */
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

static float round_act(const orc_config *c, float f) {
    return c->round_act ? orc_bf16_to_f32(orc_f32_to_bf16(f)) : f;
}

/* ---- 8-bit cache variant ------------------------------------------------------------------ */

/* Nearest value of the 8-bit floating-point format E4M3 of the OCP 8-bit floating point specification (1 sign,
   4 exponent bits with bias 7, 3 mantissa bits; no infinities; largest finite value 448 = 1.75 * 2^8; subnormals
   are multiples of 2^-9 below 2^-6), ties to the even mantissa, magnitudes above 448 saturate to 448.  Every such
   value is exactly a bf16 value, so the cache keeps holding bf16 patterns; the variant only changes the rounding
   K and V undergo on entering the cache -- directly from fp32, not through bf16 first. */
float orc_e4m3_round(float f) {
    if (f != f) return f;
    float a = fabsf(f);
    if (a > 448.0f) a = 448.0f;
    float q;
    if (a < 0.015625f) {                       /* below 2^-6: subnormal, spacing 2^-9 */
        q = nearbyintf(a * 512.0f) / 512.0f;   /* exact scalings; nearbyint rounds half to even */
    } else {
        int e;
        frexpf(a, &e);                         /* a = m * 2^e, m in [0.5, 1): spacing 2^(e - 4) */
        float ulp = ldexpf(1.0f, e - 4);
        q = nearbyintf(a / ulp) * ulp;         /* may carry into the next binade: still a format value */
    }
    return copysignf(q, f);
}

/* what K or V becomes on entering the cache, as a bf16 pattern */
static uint16_t kv_round(const orc_config *c, float f) {
    return c->kv_fp8 ? orc_f32_to_bf16(orc_e4m3_round(f)) : orc_f32_to_bf16(f);
}

/* ---- the elementary operations ---------------------------------------------------------- */

/* order in which a sum over i = 0..n-1 adds its terms: ascending (the contract), or descending in the
   sensitivity variant */
#ifdef ORC_SUM_DESCENDING
#define ORC_FOR_SUM(i, n) for (int i = (n) - 1; i >= 0; --i)
#else
#define ORC_FOR_SUM(i, n) for (int i = 0; i < (n); ++i)
#endif

/* y_i = x_i * rsqrt(mean_j x_j^2 + eps) * g_i */
void orc_rmsnorm(const float *x, const uint16_t *g, int n, float eps, float *y) {
    float ss = 0.0f;
    ORC_FOR_SUM(i, n) ss += x[i] * x[i];
    float r = 1.0f / sqrtf(ss / (float)n + eps);
    for (int i = 0; i < n; ++i) y[i] = x[i] * r * orc_bf16_to_f32(g[i]);
}

/* y[n] = sum_k x[k] * W[k][n] (+ bias[n]);  W is [K, N] row-major bf16, k ascending */
void orc_linear(const float *x, const uint16_t *W, const uint16_t *bias, int K, int N, float *y) {
    for (int n = 0; n < N; ++n) y[n] = 0.0f;
    ORC_FOR_SUM(k, K) {
        const float xk = x[k];
        const uint16_t *w = W + (size_t)k * N;
        for (int n = 0; n < N; ++n) y[n] += xk * orc_bf16_to_f32(w[n]);
    }
    if (bias)
        for (int n = 0; n < N; ++n) y[n] += orc_bf16_to_f32(bias[n]);
}

/* rotate-half RoPE on one head vector: pairs (i, i + d/2), angle pos * theta^(-2i/d);
   the angle and its cos/sin are evaluated in double, then used as fp32 */
void orc_rope(float *v, int d, int pos, float theta) {
    int half = d / 2;
    for (int i = 0; i < half; ++i) {
        double ang = (double)pos * pow((double)theta, -2.0 * (double)i / (double)d);
        float c = (float)cos(ang), s = (float)sin(ang);
        float a = v[i], b = v[i + half];
        v[i] = a * c - b * s;
        v[i + half] = b * c + a * s;
    }
}

/* p = softmax(s), max subtracted first */
void orc_softmax(const float *s, int n, float *p) {
    float m = s[0];
    for (int i = 1; i < n; ++i)
        if (s[i] > m) m = s[i];
    float sum = 0.0f;
    ORC_FOR_SUM(i, n) {
        p[i] = expf(s[i] - m);
        sum += p[i];
    }
    for (int i = 0; i < n; ++i) p[i] = p[i] / sum;
}

float orc_silu(float x) { return x / (1.0f + expf(-x)); }

/* smallest index attaining the maximum */
int32_t orc_argmax(const float *x, int n) {
    int32_t best = 0;
    for (int i = 1; i < n; ++i)
        if (x[i] > x[best]) best = i;
    return best;
}

/* ---- paged KV cache: pool[block][slot][kv_head][head_dim] bf16, one pool per layer ------- */

static size_t kv_index(const orc_config *c, int32_t block, int slot, int kvh) {
    return (((size_t)block * c->block_size + slot) * c->n_kv_heads + kvh) * c->head_dim;
}

/* copy the K/V rows of `batch` sequences (concatenated, [tokens, n_kv_heads, head_dim]) of ONE
   layer into the pool at the places the block table names */
void orc_kv_fill(const orc_config *c, uint16_t *kpool, uint16_t *vpool, const uint16_t *k,
                 const uint16_t *v, const int32_t *seq_start, const int32_t *block_table,
                 int max_blocks, int batch) {
    size_t row = (size_t)c->n_kv_heads * c->head_dim;
    for (int b = 0; b < batch; ++b)
        for (int t = seq_start[b]; t < seq_start[b + 1]; ++t) {
            int p = t - seq_start[b];
            int32_t blk = block_table[(size_t)b * max_blocks + p / c->block_size];
            size_t at = kv_index(c, blk, p % c->block_size, 0);
            for (size_t j = 0; j < row; ++j) {   /* bf16 values pass unchanged unless the cache is 8-bit */
                kpool[at + j] = kv_round(c, orc_bf16_to_f32(k[(size_t)t * row + j]));
                vpool[at + j] = kv_round(c, orc_bf16_to_f32(v[(size_t)t * row + j]));
            }
        }
}

/* attention of one sequence: q [n_q_heads, head_dim] against keys 0..T-1 found through `table`;
   o [n_q_heads, head_dim].  Query head h reads KV head h / (n_q_heads / n_kv_heads). */
void orc_attention(const orc_config *c, const float *q, const uint16_t *kpool, const uint16_t *vpool,
                   const int32_t *table, int T, float *o) {
    int d = c->head_dim, G = c->n_q_heads / c->n_kv_heads;
    float scale = 1.0f / sqrtf((float)d);
    float *s = (float *)malloc(sizeof(float) * (size_t)T);
    float *p = (float *)malloc(sizeof(float) * (size_t)T);
    for (int h = 0; h < c->n_q_heads; ++h) {
        int kvh = h / G;
        for (int t = 0; t < T; ++t) {
            const uint16_t *kr = kpool + kv_index(c, table[t / c->block_size], t % c->block_size, kvh);
            float dot = 0.0f;
            ORC_FOR_SUM(j, d) dot += q[h * d + j] * orc_bf16_to_f32(kr[j]);
            s[t] = dot * scale;
        }
        orc_softmax(s, T, p);
        for (int j = 0; j < d; ++j) o[h * d + j] = 0.0f;
        ORC_FOR_SUM(t, T) {
            const uint16_t *vr = vpool + kv_index(c, table[t / c->block_size], t % c->block_size, kvh);
            for (int j = 0; j < d; ++j) o[h * d + j] += p[t] * orc_bf16_to_f32(vr[j]);
        }
    }
    free(s);
    free(p);
}

/* ---- one decoder layer for one sequence -------------------------------------------------- */

/* x [hidden] is the fp32 residual stream (updated in place).  The new token's K and V are
   written at position `pos` through `table`, then positions 0..pos are attended.
   attn_out (may be NULL) receives o before its rounding. */
/* Intermediate results of one layer step, for stage-by-stage comparisons (every pointer may be NULL):
   u1 [hidden] rounded input of the q/k/v projection; qkv [qkv_dim] projection + bias before the rotation;
   q [n_q_heads*head_dim] rotated, rounded query; k_new, v_new [n_kv_heads*head_dim] what entered the cache (as fp32);
   o [n_q_heads*head_dim] attention output before rounding; y_o [hidden] output projection; x_mid [hidden] residual
   stream after the attention block; u2 [hidden]; m [intermediate] rounded SwiGLU output; y_d [hidden] down projection. */
typedef struct {
    float *u1, *qkv, *q, *k_new, *v_new, *o, *y_o, *x_mid, *u2, *m, *y_d;
} orc_trace;

static void trace_copy(float *dst, const float *src, int n) {
    if (dst) memcpy(dst, src, sizeof(float) * (size_t)n);
}

void orc_layer_step_trace(const orc_config *c, const orc_layer *w, float *x, int pos, uint16_t *kpool,
                          uint16_t *vpool, const int32_t *table, float *attn_out, const orc_trace *tr) {
    static const orc_trace none = {0};
    if (!tr) tr = &none;
    int H = c->hidden, d = c->head_dim, nq = c->n_q_heads, nkv = c->n_kv_heads, I = c->intermediate;
    int QD = nq * d, KD = nkv * d, N = QD + 2 * KD;
    float *u = (float *)malloc(sizeof(float) * (size_t)H);
    float *qkv = (float *)malloc(sizeof(float) * (size_t)N);
    float *o = (float *)malloc(sizeof(float) * (size_t)QD);
    float *y = (float *)malloc(sizeof(float) * (size_t)H);
    float *gt = (float *)malloc(sizeof(float) * (size_t)I);
    float *up = (float *)malloc(sizeof(float) * (size_t)I);

    /* attention block */
    orc_rmsnorm(x, w->g1, H, c->rms_eps, u);
    for (int i = 0; i < H; ++i) u[i] = round_act(c, u[i]);
    trace_copy(tr->u1, u, H);
    orc_linear(u, w->wqkv, c->qkv_bias ? w->bqkv : NULL, H, N, qkv);
    trace_copy(tr->qkv, qkv, N);
    float *q = qkv, *k = qkv + QD, *v = qkv + QD + KD;
    for (int h = 0; h < nq; ++h) orc_rope(q + h * d, d, pos, c->rope_theta);
    for (int h = 0; h < nkv; ++h) orc_rope(k + h * d, d, pos, c->rope_theta);
    for (int i = 0; i < QD; ++i) q[i] = round_act(c, q[i]);
    trace_copy(tr->q, q, QD);
    {
        int32_t blk = table[pos / c->block_size];
        int slot = pos % c->block_size;
        for (int h = 0; h < nkv; ++h) {
            size_t at = kv_index(c, blk, slot, h);
            for (int j = 0; j < d; ++j) {
                kpool[at + j] = kv_round(c, k[h * d + j]);
                vpool[at + j] = kv_round(c, v[h * d + j]);
                if (tr->k_new) tr->k_new[h * d + j] = orc_bf16_to_f32(kpool[at + j]);
                if (tr->v_new) tr->v_new[h * d + j] = orc_bf16_to_f32(vpool[at + j]);
            }
        }
    }
    orc_attention(c, q, kpool, vpool, table, pos + 1, o);
    if (attn_out) memcpy(attn_out, o, sizeof(float) * (size_t)QD);
    trace_copy(tr->o, o, QD);
    for (int i = 0; i < QD; ++i) o[i] = round_act(c, o[i]);
    orc_linear(o, w->wo, NULL, QD, H, y);
    for (int i = 0; i < H; ++i) x[i] += y[i];
    trace_copy(tr->y_o, y, H);
    trace_copy(tr->x_mid, x, H);

    /* SwiGLU block */
    orc_rmsnorm(x, w->g2, H, c->rms_eps, u);
    for (int i = 0; i < H; ++i) u[i] = round_act(c, u[i]);
    trace_copy(tr->u2, u, H);
    orc_linear(u, w->wg, NULL, H, I, gt);
    orc_linear(u, w->wu, NULL, H, I, up);
    for (int i = 0; i < I; ++i) gt[i] = round_act(c, orc_silu(gt[i]) * up[i]);
    orc_linear(gt, w->wd, NULL, I, H, y);
    trace_copy(tr->m, gt, I);
    trace_copy(tr->y_d, y, H);
    for (int i = 0; i < H; ++i) x[i] += y[i];

    free(u); free(qkv); free(o); free(y); free(gt); free(up);
}

void orc_layer_step(const orc_config *c, const orc_layer *w, float *x, int pos, uint16_t *kpool,
                    uint16_t *vpool, const int32_t *table, float *attn_out) {
    orc_layer_step_trace(c, w, x, pos, kpool, vpool, table, attn_out, NULL);
}

/* x = embedding row of the token, as fp32 */
void orc_embed(const orc_config *c, const orc_weights *w, int32_t token, float *x) {
    for (int i = 0; i < c->hidden; ++i) x[i] = orc_bf16_to_f32(w->embed[(size_t)token * c->hidden + i]);
}

/* final norm, LM head, greedy token */
int32_t orc_head(const orc_config *c, const orc_weights *w, const float *x, float *logits) {
    int H = c->hidden;
    float *u = (float *)malloc(sizeof(float) * (size_t)H);
    orc_rmsnorm(x, w->gf, H, c->rms_eps, u);
    for (int i = 0; i < H; ++i) u[i] = round_act(c, u[i]);
    orc_linear(u, w->wlm, NULL, H, c->vocab, logits);
    free(u);
    return orc_argmax(logits, c->vocab);
}

/* ---- one decode step over a batch --------------------------------------------------------- */

/* tokens/positions/seq_lens [batch]; block_table [batch, max_blocks]; kpools/vpools: one pool
   pointer per layer; logits [batch, vocab]; next_tokens [batch]; attn_out (may be NULL)
   [n_layers, batch, n_q_heads*head_dim].  seq_lens[b] must equal positions[b] + 1.
   Rows are independent, so they run in parallel; each row's arithmetic is sequential. */
int orc_decode_step(const orc_config *c, const orc_weights *w, int batch, const int32_t *tokens,
                    const int32_t *positions, const int32_t *seq_lens, const int32_t *block_table,
                    int max_blocks, uint16_t *const *kpools, uint16_t *const *vpools, float *logits,
                    int32_t *next_tokens, float *attn_out) {
    for (int b = 0; b < batch; ++b)
        if (seq_lens[b] != positions[b] + 1) return -1;
    size_t QD = (size_t)c->n_q_heads * c->head_dim;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < batch; ++b) {
        float *x = (float *)malloc(sizeof(float) * (size_t)c->hidden);
        orc_embed(c, w, tokens[b], x);
        for (int l = 0; l < c->n_layers; ++l)
            orc_layer_step(c, &w->layers[l], x, positions[b], kpools[l], vpools[l],
                           block_table + (size_t)b * max_blocks,
                           attn_out ? attn_out + ((size_t)l * batch + b) * QD : NULL);
        next_tokens[b] = orc_head(c, w, x, logits + (size_t)b * c->vocab);
        free(x);
    }
    return 0;
}

/* ---- brute force: all n positions of one sequence at once, no cache, no paging ------------ */

/* Dense causal recomputation: every layer processes all n positions, scores are an n x n
   lower-triangular matrix.  logits [n, vocab].  attn_out (may be NULL) [n_layers, n, nq*d]. */
void orc_full_causal(const orc_config *c, const orc_weights *w, const int32_t *tokens, int n,
                     float *logits, float *attn_out) {
    int H = c->hidden, d = c->head_dim, nq = c->n_q_heads, nkv = c->n_kv_heads, I = c->intermediate;
    int QD = nq * d, KD = nkv * d, N = QD + 2 * KD, G = nq / nkv;
    float scale = 1.0f / sqrtf((float)d);
    float *X = (float *)malloc(sizeof(float) * (size_t)n * H);
    float *Q = (float *)malloc(sizeof(float) * (size_t)n * QD);
    float *Km = (float *)malloc(sizeof(float) * (size_t)n * KD);
    float *Vm = (float *)malloc(sizeof(float) * (size_t)n * KD);
    float *u = (float *)malloc(sizeof(float) * (size_t)H);
    float *qkv = (float *)malloc(sizeof(float) * (size_t)N);
    float *o = (float *)malloc(sizeof(float) * (size_t)QD);
    float *y = (float *)malloc(sizeof(float) * (size_t)H);
    float *gt = (float *)malloc(sizeof(float) * (size_t)I);
    float *up = (float *)malloc(sizeof(float) * (size_t)I);
    float *s = (float *)malloc(sizeof(float) * (size_t)n);
    float *p = (float *)malloc(sizeof(float) * (size_t)n);

    for (int t = 0; t < n; ++t) orc_embed(c, w, tokens[t], X + (size_t)t * H);
    for (int l = 0; l < c->n_layers; ++l) {
        const orc_layer *lw = &w->layers[l];
        for (int t = 0; t < n; ++t) {
            orc_rmsnorm(X + (size_t)t * H, lw->g1, H, c->rms_eps, u);
            for (int i = 0; i < H; ++i) u[i] = round_act(c, u[i]);
            orc_linear(u, lw->wqkv, c->qkv_bias ? lw->bqkv : NULL, H, N, qkv);
            for (int h = 0; h < nq; ++h) orc_rope(qkv + h * d, d, t, c->rope_theta);
            for (int h = 0; h < nkv; ++h) orc_rope(qkv + QD + h * d, d, t, c->rope_theta);
            for (int i = 0; i < QD; ++i) Q[(size_t)t * QD + i] = round_act(c, qkv[i]);
            for (int i = 0; i < KD; ++i) {
                Km[(size_t)t * KD + i] = c->kv_fp8 ? orc_e4m3_round(qkv[QD + i]) : round_act(c, qkv[QD + i]);
                Vm[(size_t)t * KD + i] = c->kv_fp8 ? orc_e4m3_round(qkv[QD + KD + i]) : round_act(c, qkv[QD + KD + i]);
            }
        }
        for (int t = 0; t < n; ++t) {
            for (int h = 0; h < nq; ++h) {
                int kvh = h / G;
                for (int r = 0; r <= t; ++r) { /* causal mask: keys 0..t only */
                    float dot = 0.0f;
                    ORC_FOR_SUM(j, d)
                        dot += Q[(size_t)t * QD + h * d + j] * Km[(size_t)r * KD + kvh * d + j];
                    s[r] = dot * scale;
                }
                orc_softmax(s, t + 1, p);
                for (int j = 0; j < d; ++j) o[h * d + j] = 0.0f;
                ORC_FOR_SUM(r, t + 1)
                    for (int j = 0; j < d; ++j) o[h * d + j] += p[r] * Vm[(size_t)r * KD + kvh * d + j];
            }
            if (attn_out) memcpy(attn_out + ((size_t)l * n + t) * QD, o, sizeof(float) * (size_t)QD);
            for (int i = 0; i < QD; ++i) o[i] = round_act(c, o[i]);
            orc_linear(o, lw->wo, NULL, QD, H, y);
            float *x = X + (size_t)t * H;
            for (int i = 0; i < H; ++i) x[i] += y[i];
            orc_rmsnorm(x, lw->g2, H, c->rms_eps, u);
            for (int i = 0; i < H; ++i) u[i] = round_act(c, u[i]);
            orc_linear(u, lw->wg, NULL, H, I, gt);
            orc_linear(u, lw->wu, NULL, H, I, up);
            for (int i = 0; i < I; ++i) gt[i] = round_act(c, orc_silu(gt[i]) * up[i]);
            orc_linear(gt, lw->wd, NULL, I, H, y);
            for (int i = 0; i < H; ++i) x[i] += y[i];
        }
    }
    for (int t = 0; t < n; ++t) orc_head(c, w, X + (size_t)t * H, logits + (size_t)t * c->vocab);
    free(X); free(Q); free(Km); free(Vm); free(u); free(qkv); free(o); free(y); free(gt); free(up);
    free(s); free(p);
}

/* ---- sampling and log-probabilities ------------------------------------------------------------
 * Rollout generation draws several responses per prompt (paper Section 1, stage (i)) and the policy
 * update needs the behaviour policy's log-probability of every drawn token (GRPO workloads, Section 5),
 * so the step can end in a temperature sample instead of the arg-max.
 *
 * Random numbers come from Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
 * as 1, 2, 3", SC'11), written here from its published definition: 10 rounds of
 *     (c0, c1, c2, c3) <- (hi(M1*c2) ^ c1 ^ k0,  lo(M1*c2),  hi(M0*c0) ^ c3 ^ k1,  lo(M0*c0))
 * with M0 = 0xD2511F53, M1 = 0xCD9E8D57, the key advanced by (0x9E3779B9, 0xBB67AE85) after every round.
 * Vocabulary entry i of the row with id `row` at position `pos` uses word i % 4 of the block with
 * counter (i / 4, row, pos, 0x53414D50) and key (seed low word, seed high word).
 *
 * Definition of the draw (Gumbel-max; all of it fp32 -- a floating-point value decides an integer here,
 * so this is the precision of the decision -- except the log-sum-exp, which is plain fp64):
 *     z_i = logit_i * (1 / T)            u_i = ((word_i >> 9) + 0.5) * 2^-23   in (0, 1), exact in fp32
 *     y_i = z_i - log(-log(u_i))         token = lowest index attaining max_i y_i
 *     logprob = z_token - log(sum_i exp(z_i))
 * P(token = i) = softmax(z)_i exactly (the Gumbel-max identity).  `gap` returns max y minus the runner-up:
 * implementations whose log differs in the last bits may disagree only when it is tiny. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

float orc_uniform_open(uint32_t word) { return ((float)(word >> 9) + 0.5f) * (1.0f / 8388608.0f); }

void orc_sample(const float *logits, int V, float temperature, uint64_t seed, uint32_t row, uint32_t pos,
                int32_t *token, float *logprob, float *gap) {
    const float inv_t = 1.0f / temperature;
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    float best = -INFINITY, second = -INFINITY, zmax = -INFINITY;
    int32_t best_i = 0;
    for (int i = 0; i < V; ++i) {
        const uint32_t ctr[4] = {(uint32_t)(i / 4), row, pos, 0x53414D50u};
        uint32_t r[4];
        orc_philox4x32_10(ctr, key, r);
        const float z = logits[i] * inv_t;
        const float u = orc_uniform_open(r[i % 4]);
        const float y = z - logf(-logf(u));
        if (y > best) { second = best; best = y; best_i = i; }
        else if (y > second) second = y;
        if (z > zmax) zmax = z;
    }
    double sum = 0.0;
    for (int i = 0; i < V; ++i) sum += exp((double)(logits[i] * inv_t) - (double)zmax);
    *token = best_i;
    *logprob = (float)((double)(logits[best_i] * inv_t) - ((double)zmax + log(sum)));
    *gap = best - second;
}

/* Nucleus (top-p) sampling, Holtzman et al., "The Curious Case of Neural Text Degeneration" (ICLR 2020), on the
   temperature-scaled distribution p = softmax(z), z = logits / T as in orc_sample: order the vocabulary by
   decreasing z, keep the shortest prefix whose probability mass reaches top_p, renormalise over it, draw from it.
   Entries equal to the last kept z are all kept (their mutual order is arbitrary, so the kept set stays a
   threshold set {z_i >= tau}).  The draw is the Gumbel-max of orc_sample restricted to the kept set, with the same
   noise per vocabulary entry; logprob is that of the renormalised distribution, log(p_token / mass of the set).
   Probabilities and the running mass are double.  margin = distance of top_p from the nearer of the two running
   masses that decide the prefix length (the last one below top_p and the first one reaching it): a comparison in
   another precision can decide differently only where margin is of the order of that precision.  gap = best minus
   runner-up of the perturbed scores among the kept entries. */
typedef struct { float z; int32_t i; } orc_zi;
static int orc_zi_desc(const void *a, const void *b) {
    const orc_zi *x = (const orc_zi *)a, *y = (const orc_zi *)b;
    if (x->z > y->z) return -1;
    if (x->z < y->z) return 1;
    return (x->i > y->i) - (x->i < y->i);
}

void orc_sample_top_p(const float *logits, int V, float temperature, float top_p, uint64_t seed, uint32_t row,
                      uint32_t pos, int32_t *token, float *logprob, int32_t *nucleus_size, double *margin, float *gap) {
    const float inv_t = 1.0f / temperature;
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    orc_zi *ord = (orc_zi *)malloc((size_t)V * sizeof(orc_zi));
    unsigned char *kept = (unsigned char *)calloc((size_t)V, 1);
    float zmax = -INFINITY;
    for (int i = 0; i < V; ++i) {
        ord[i].z = logits[i] * inv_t;
        ord[i].i = i;
        if (ord[i].z > zmax) zmax = ord[i].z;
    }
    double sum = 0.0;
    for (int i = 0; i < V; ++i) sum += exp((double)ord[i].z - (double)zmax);
    qsort(ord, (size_t)V, sizeof(orc_zi), orc_zi_desc);

    double cum = 0.0, below = 0.0;
    int n = 0;
    while (n < V) {
        below = cum;
        cum += exp((double)ord[n].z - (double)zmax) / sum;
        ++n;
        if (cum >= (double)top_p) break;
    }
    *margin = fmin(fabs(cum - (double)top_p), fabs((double)top_p - below));
    while (n < V && ord[n].z == ord[n - 1].z) ++n;
    double mass = 0.0;
    for (int k = 0; k < n; ++k) {
        kept[ord[k].i] = 1;
        mass += exp((double)ord[k].z - (double)zmax);
    }

    float best = -INFINITY, second = -INFINITY;
    int32_t best_i = ord[0].i;
    for (int i = 0; i < V; ++i) {
        if (!kept[i]) continue;
        const uint32_t ctr[4] = {(uint32_t)(i / 4), row, pos, 0x53414D50u};
        uint32_t r[4];
        orc_philox4x32_10(ctr, key, r);
        const float z = logits[i] * inv_t;
        const float y = z - logf(-logf(orc_uniform_open(r[i % 4])));
        if (y > best) { second = best; best = y; best_i = i; }
        else if (y > second) second = y;
    }
    *token = best_i;
    *logprob = (float)((double)(logits[best_i] * inv_t) - ((double)zmax + log(mass)));
    *nucleus_size = n;
    *gap = best - second;                         /* +inf when one entry is kept */
    free(ord);
    free(kept);
}

int orc_num_threads(void) {
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
