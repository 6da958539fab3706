/*
 * Sanitizer driver of the CPU oracle -- TEST INFRASTRUCTURE.  Compiled together with oracle/decode_oracle.c under
 * -fsanitize=address,undefined and run as an ordinary program by tests/test_sanitizers.py: a small decoder (2 layers,
 * hidden 64, 4 query / 2 KV heads of 16, vocabulary 96) with pseudo-random bf16 weights goes through every entry point
 * of the oracle -- cache fill through a shuffled block table with ragged lengths, several decode steps that append
 * to the cache, the dense causal recomputation, both samplers, the 8-bit cache variant -- so that an out-of-bounds
 * index, a misaligned access, an integer overflow or a use of uninitialised heap shows as a sanitizer report.
 * The values are checked only for finiteness and for stepwise == dense (the oracle's own invariant).
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, intermediate, vocab, block_size;
    int32_t qkv_bias, round_act, kv_fp8;
    float rms_eps, rope_theta;
} orc_config;
typedef struct { const uint16_t *g1, *wqkv, *bqkv, *wo, *g2, *wg, *wu, *wd; } orc_layer;
typedef struct { const uint16_t *embed, *gf, *wlm; const orc_layer *layers; } orc_weights;

uint16_t orc_f32_to_bf16(float f);
float orc_e4m3_round(float f);
void orc_kv_fill(const orc_config *c, uint16_t *kpool, uint16_t *vpool, const uint16_t *k, const uint16_t *v,
                 const int32_t *seq_start, const int32_t *block_table, int max_blocks, int batch);
int orc_decode_step(const orc_config *c, const orc_weights *w, int batch, const int32_t *tokens, const int32_t *positions,
                    const int32_t *seq_lens, const int32_t *block_table, int max_blocks, uint16_t *const *kpools,
                    uint16_t *const *vpools, float *logits, int32_t *next_tokens, float *attn_out);
void orc_full_causal(const orc_config *c, const orc_weights *w, const int32_t *tokens, int n, float *logits, float *attn_out);
void orc_sample(const float *logits, int V, float temperature, uint64_t seed, uint32_t row, uint32_t pos, int32_t *token,
                float *logprob, float *gap);
void orc_sample_top_p(const float *logits, int V, float temperature, float top_p, uint64_t seed, uint32_t row, uint32_t pos,
                      int32_t *token, float *logprob, int32_t *nucleus_size, double *margin, float *gap);

static uint64_t rng_state = 0x2511007960ull;
static float uniform01(void) {                      /* splitmix64 */
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return (float)((z >> 40) + 1) / 16777218.0f;
}
static float normal(void) { return sqrtf(-2.0f * logf(uniform01())) * cosf(6.2831853f * uniform01()); }
static uint16_t *tensor(size_t n, float mean, float std) {
    uint16_t *t = (uint16_t *)malloc(n * sizeof(uint16_t));
    for (size_t i = 0; i < n; ++i) t[i] = orc_f32_to_bf16(mean + std * normal());
    return t;
}

static int run(int kv_fp8) {
    orc_config c = {2, 64, 4, 2, 16, 80, 96, 16, 1, 1, kv_fp8, 1e-6f, 1e6f};
    const int H = c.hidden, QD = c.n_q_heads * c.head_dim, KD = c.n_kv_heads * c.head_dim, N = QD + 2 * KD, I = c.intermediate;
    orc_layer layers[2];
    for (int l = 0; l < 2; ++l) {
        layers[l].g1 = tensor(H, 1.f, 0.02f); layers[l].wqkv = tensor((size_t)H * N, 0.f, 0.05f);
        layers[l].bqkv = tensor(N, 0.f, 0.05f); layers[l].wo = tensor((size_t)QD * H, 0.f, 0.05f);
        layers[l].g2 = tensor(H, 1.f, 0.02f); layers[l].wg = tensor((size_t)H * I, 0.f, 0.05f);
        layers[l].wu = tensor((size_t)H * I, 0.f, 0.05f); layers[l].wd = tensor((size_t)I * H, 0.f, 0.05f);
    }
    orc_weights w = {tensor((size_t)c.vocab * H, 0.f, 0.5f), tensor(H, 1.f, 0.02f), tensor((size_t)H * c.vocab, 0.f, 0.05f), layers};

    /* ---- stepwise decode of one sequence == dense causal recomputation (bit for bit) ---- */
    enum { NTOK = 37 };
    int32_t toks[NTOK];
    for (int i = 0; i < NTOK; ++i) toks[i] = (int32_t)(uniform01() * c.vocab) % c.vocab;
    const int nblk = (NTOK + 15) / 16;
    int32_t table1[3] = {2, 0, 1};                     /* shuffled physical blocks */
    size_t pool_elems = (size_t)nblk * 16 * KD;
    uint16_t *kp[2], *vp[2];
    for (int l = 0; l < 2; ++l) { kp[l] = (uint16_t *)calloc(pool_elems, 2); vp[l] = (uint16_t *)calloc(pool_elems, 2); }
    float *step_logits = (float *)malloc(sizeof(float) * NTOK * c.vocab);
    float *attn = (float *)malloc(sizeof(float) * 2 * QD);
    for (int p = 0; p < NTOK; ++p) {
        int32_t pos = p, len = p + 1, nxt;
        if (orc_decode_step(&c, &w, 1, &toks[p], &pos, &len, table1, nblk, kp, vp, step_logits + (size_t)p * c.vocab, &nxt, attn)) return 1;
    }
    float *dense = (float *)malloc(sizeof(float) * NTOK * c.vocab);
    float *dense_attn = (float *)malloc(sizeof(float) * 2 * NTOK * QD);
    orc_full_causal(&c, &w, toks, NTOK, dense, dense_attn);
    if (memcmp(dense, step_logits, sizeof(float) * NTOK * c.vocab) != 0) { printf("stepwise != dense (kv_fp8 %d)\n", kv_fp8); return 2; }
    for (int i = 0; i < NTOK * c.vocab; ++i) if (!isfinite(dense[i])) return 3;

    /* ---- a ragged batch over a filled cache, wrong seq_lens rejected ---- */
    enum { B = 3 };
    int32_t ctx[B] = {1, 16, 33}, start[B + 1] = {0, 1, 17, 50};
    int32_t table[B][4] = {{5, -1, -1, -1}, {1, 0, -1, -1}, {4, 2, 3, -1}};
    uint16_t *kf = tensor((size_t)50 * KD, 0.f, 1.f), *vf = tensor((size_t)50 * KD, 0.f, 1.f);
    uint16_t *kq[2], *vq[2];
    for (int l = 0; l < 2; ++l) {
        kq[l] = (uint16_t *)calloc((size_t)6 * 16 * KD, 2); vq[l] = (uint16_t *)calloc((size_t)6 * 16 * KD, 2);
        orc_kv_fill(&c, kq[l], vq[l], kf, vf, start, &table[0][0], 4, B);
    }
    int32_t bt[B] = {3, 95, 0}, pos[B], len[B], nxt[B];
    for (int b = 0; b < B; ++b) { pos[b] = ctx[b]; len[b] = ctx[b] + 1; }
    float *bl = (float *)malloc(sizeof(float) * B * c.vocab), *ba = (float *)malloc(sizeof(float) * 2 * B * QD);
    if (orc_decode_step(&c, &w, B, bt, pos, len, &table[0][0], 4, kq, vq, bl, nxt, ba)) return 4;
    len[1] += 1;
    if (orc_decode_step(&c, &w, B, bt, pos, len, &table[0][0], 4, kq, vq, bl, nxt, ba) == 0) return 5;

    /* ---- samplers on those logits ---- */
    for (int b = 0; b < B; ++b) {
        int32_t tok, size; float lp, gap; double margin;
        orc_sample(bl + (size_t)b * c.vocab, c.vocab, 0.7f, 0x123456789abcdefull, (uint32_t)b, (uint32_t)pos[b], &tok, &lp, &gap);
        if (tok < 0 || tok >= c.vocab || !(lp <= 0.f)) return 6;
        orc_sample_top_p(bl + (size_t)b * c.vocab, c.vocab, 1.3f, 0.4f, 77u, (uint32_t)b, (uint32_t)pos[b], &tok, &lp, &size, &margin, &gap);
        if (tok < 0 || tok >= c.vocab || size < 1 || size > c.vocab || !(lp <= 0.f)) return 7;
        orc_sample_top_p(bl + (size_t)b * c.vocab, c.vocab, 1.0f, 1.0f, 77u, (uint32_t)b, (uint32_t)pos[b], &tok, &lp, &size, &margin, &gap);
        if (size != c.vocab) return 8;
    }
    if (orc_e4m3_round(1000.f) != 448.f || orc_e4m3_round(-0.0f) != 0.f) return 9;

    for (int l = 0; l < 2; ++l) {
        free(kp[l]); free(vp[l]); free(kq[l]); free(vq[l]);
        free((void *)layers[l].g1); free((void *)layers[l].wqkv); free((void *)layers[l].bqkv); free((void *)layers[l].wo);
        free((void *)layers[l].g2); free((void *)layers[l].wg); free((void *)layers[l].wu); free((void *)layers[l].wd);
    }
    free((void *)w.embed); free((void *)w.gf); free((void *)w.wlm);
    free(step_logits); free(attn); free(dense); free(dense_attn); free(kf); free(vf); free(bl); free(ba);
    return 0;
}

int main(void) {
    int rc = run(0);
    if (rc == 0) rc = run(1) ? 100 + run(1) : 0;
    printf(rc == 0 ? "oracle sanitizer driver: OK\n" : "oracle sanitizer driver: FAILED (%d)\n", rc);
    return rc;
}
