// Sanitizer driver of the library's HOST-side logic -- TEST INFRASTRUCTURE.  Linked with the host halves of
// paper_2511_00796_amd/csrc/*.hip (no device code) under -fsanitize=address,undefined and run as an ordinary program
// by tests/test_sanitizers.py, without a GPU: size queries, configuration checks, the buffer maps of engines of all
// five model shapes (created over fake device addresses, which creation only records), argument validation of
// every step entry point before anything is enqueued, the launch planner, handle release.  No kernel is launched.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <initializer_list>

#include "../../include/hexdecode.h"

static int fails = 0;
#define EXPECT(cond) do { if (!(cond)) { printf("host driver: %s failed at line %d (%s)\n", #cond, __LINE__, hx_last_error()); ++fails; } } while (0)

static hx_model_config shape(int layers, int hidden, int nq, int nkv, int d, int inter, int vocab, int batch, int seq) {
    hx_model_config c;
    memset(&c, 0, sizeof(c));
    c.struct_size = sizeof(c);
    c.n_layers = layers; c.hidden = hidden; c.n_q_heads = nq; c.n_kv_heads = nkv; c.head_dim = d; c.intermediate = inter;
    c.vocab = vocab; c.block_size = 16; c.qkv_bias = 1; c.rms_eps = 1e-6f; c.rope_theta = 1e6f; c.max_batch = batch;
    c.max_seq_len = seq; c.kv_dtype = HX_KV_BF16;
    return c;
}

int main() {
    const hx_model_config shapes[] = {
        shape(2, 256, 4, 2, 64, 688, 1024, 4, 256),            shape(28, 1536, 12, 2, 128, 8960, 151936, 64, 8200),
        shape(28, 1536, 12, 2, 128, 8960, 151936, 256, 16400), shape(28, 3584, 28, 4, 128, 18944, 152064, 128, 16400),
        shape(48, 5120, 40, 8, 128, 13824, 152064, 64, 16400)};
    void *fake = (void *)(uintptr_t)0x10000000;              // never dereferenced
    for (const hx_model_config &c0 : shapes) {
        for (int kvd = 0; kvd < 2; ++kvd) {
            hx_model_config c = c0;
            c.kv_dtype = kvd;
            size_t wb = 0, sb = 0, kb = 0;
            EXPECT(hx_weights_bytes(&c, &wb) == HX_OK && wb > 0);
            EXPECT(hx_workspace_bytes(&c, &sb) == HX_OK && sb > 0);
            EXPECT(hx_kv_bytes(&c, 1000, &kb) == HX_OK && kb == (size_t)c.n_layers * 1000 * c.n_kv_heads * 2 * 16 * c.head_dim * (kvd ? 1 : 2));
            hx_engine *e = nullptr;
            EXPECT(hx_engine_create(&c, fake, wb - 1, fake, sb, &e) == HX_E_TOO_SMALL && e == nullptr);
            EXPECT(hx_engine_create(&c, (char *)fake + 64, wb, fake, sb, &e) == HX_E_ALIGN);
            EXPECT(hx_engine_create(&c, fake, wb, nullptr, sb, &e) == HX_E_NULL);
            EXPECT(hx_engine_create(&c, fake, wb, fake, sb, &e) == HX_OK && e != nullptr);
            if (!e) continue;
            EXPECT(hx_attention_waves(e) >= 64);
            hx_kv *kv = nullptr;
            EXPECT(kv_alloc(e, fake, kb - 1, 1000, &kv) == HX_E_TOO_SMALL);
            EXPECT(kv_alloc(e, fake, kb, 1000, &kv) == HX_OK && kv != nullptr);
            const int32_t *ip = (const int32_t *)fake;
            int32_t *op = (int32_t *)fake;
            float *fp = (float *)fake;
            EXPECT(decode_step(e, kv, 0, ip, ip, ip, ip, 4, nullptr, op, nullptr) == HX_E_RANGE);
            EXPECT(decode_step(e, kv, c.max_batch + 1, ip, ip, ip, ip, 4, nullptr, op, nullptr) == HX_E_RANGE);
            EXPECT(decode_step(e, kv, 1, ip, ip, ip, ip, 0, nullptr, op, nullptr) == HX_E_RANGE);
            EXPECT(decode_step(e, kv, 1, nullptr, ip, ip, ip, 4, nullptr, op, nullptr) == HX_E_NULL);
            EXPECT(decode_step(e, nullptr, 1, ip, ip, ip, ip, 4, nullptr, op, nullptr) == HX_E_NULL);
            EXPECT(decode_step_sample(e, kv, 1, ip, ip, ip, ip, 4, 0.0f, 1, nullptr, nullptr, op, fp, nullptr) == HX_E_RANGE);
            EXPECT(decode_step_sample(e, kv, 1, ip, ip, ip, ip, 4, 1.0f, 1, nullptr, nullptr, op, nullptr, nullptr) == HX_E_NULL);
            EXPECT(decode_step_top_p(e, kv, 1, ip, ip, ip, ip, 4, 1.0f, 1.5f, 1, nullptr, fp, op, fp, nullptr, nullptr) == HX_E_RANGE);
            EXPECT(decode_step_top_p(e, kv, 1, ip, ip, ip, ip, 4, 1.0f, 0.5f, 1, nullptr, nullptr, op, fp, nullptr, nullptr) == HX_E_NULL);
            EXPECT(prefill_chunk(e, kv, c.max_batch + 1, ip, ip, ip, ip, 4, nullptr) == HX_E_RANGE);
            // prompt rows: refused before anything is launched (row count, engine size, workspace)
            EXPECT(prefill_rows(e, kv, 300, ip, ip, ip, ip, 4, fake, (size_t)1 << 40, nullptr) == HX_E_RANGE);
            EXPECT(prefill_rows(e, kv, 256, ip, ip, ip, ip, 4, nullptr, 0, nullptr) == HX_E_NULL);
            EXPECT(prefill_rows(e, nullptr, 256, ip, ip, ip, ip, 4, fake, (size_t)1 << 40, nullptr) == HX_E_NULL);
            if (c.max_batch == 256) {
                EXPECT(prefill_rows(e, kv, 256, ip, ip, ip, ip, 4, fake, 1024, nullptr) == HX_E_RANGE);
                EXPECT(hx_stage_linear_rows(e, HX_T_WLM, 0, 256, fp, fp, fake, (size_t)1 << 40, nullptr) == HX_E_SHAPE);
                EXPECT(hx_stage_linear_rows(e, HX_T_WO, 0, 256, fp, fp, fake, 1024, nullptr) == HX_E_RANGE);
            } else {
                EXPECT(prefill_rows(e, kv, 256, ip, ip, ip, ip, 4, fake, (size_t)1 << 40, nullptr) == HX_E_RANGE);
                EXPECT(hx_stage_linear_rows(e, HX_T_WO, 0, 256, fp, fp, fake, (size_t)1 << 40, nullptr) == HX_E_RANGE);
            }
            EXPECT(prefill_fill(kv, c.n_layers, fake, fake, ip, ip, 4, 1, 16, nullptr) == HX_E_SHAPE);
            EXPECT(prefill_fill(kv, 0, fake, fake, ip, ip, 4, 0, 16, nullptr) == HX_E_RANGE);
            EXPECT(hx_kv_gather(kv, 0, fake, nullptr, ip, ip, 4, 1, 16, nullptr) == HX_E_NULL);
            EXPECT(hx_weights_pack(e, HX_T_WO, 0, fake, 3, 3, nullptr) == HX_E_SHAPE);
            EXPECT(hx_weights_pack(e, HX_T_WD, c.n_layers, fake, c.intermediate, c.hidden, nullptr) == HX_E_SHAPE);
            EXPECT(hx_weights_pack(e, 99, 0, fake, 1, 1, nullptr) == HX_E_SHAPE);
            EXPECT(hx_stage_linear(e, HX_T_WO, 0, c.max_batch + 1, fp, fp, nullptr, nullptr) == HX_E_RANGE);
            EXPECT(hx_stage_linear(e, HX_T_WO, 0, 1, fp, fp, op, nullptr) == HX_E_SHAPE);
            EXPECT(hx_stage_rmsnorm(e, HX_T_WO, 0, 1, fp, fp, nullptr) == HX_E_SHAPE);
            EXPECT(hx_profile_enable(e, 1u << 20) == HX_E_RANGE);
            EXPECT(hx_profile_sample_every(e, 0) == HX_E_RANGE);
            double ms = 0;
            int64_t n = 0;
            EXPECT(hx_profile_read(e, 0, &ms, &n) == HX_OK && n == 0);
            EXPECT(hx_set_attn_capture(e, nullptr) == HX_OK);
            EXPECT(kv_free(kv) == HX_OK);
            EXPECT(hx_engine_destroy(e) == HX_OK);
            // the planner, for every product of the shape and every m-group count
            const int qkv = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
            const int prod[5][3] = {{c.hidden, qkv, 1}, {c.n_q_heads * c.head_dim, c.hidden, 1}, {c.hidden, 2 * c.intermediate, 0},
                                    {c.intermediate, c.hidden, 1}, {c.hidden, c.vocab, 0}};
            for (const auto &p : prod)
                for (int batch : {1, 33, 64, 128, 256}) {
                    int32_t wn = 0, wk = 0, sp = 0;
                    EXPECT(hx_plan_product((p[1] + 31) / 32, p[0] / 16, batch, p[2], &wn, &wk, &sp) == HX_OK);
                    EXPECT(((wn >= 4 && wn <= 6) || (wn == 10 && !p[2] && batch <= 128)) && wk >= 1 && sp >= 1 && sp <= 9 && (p[2] || sp == 1));
                }
        }
    }
    {   // prompt-row workspace sizing: only for engines of 256 rows, multiples of 256 up to the limit
        hx_model_config c256 = shapes[0];
        c256.max_batch = 256;
        size_t one = 0, four = 0;
        EXPECT(hx_prefill_workspace_bytes(&c256, 256, &one) == HX_OK && one > 0);
        EXPECT(hx_prefill_workspace_bytes(&c256, 1024, &four) == HX_OK && four == 4 * one);
        EXPECT(hx_prefill_workspace_bytes(&c256, 300, &one) == HX_E_RANGE);
        EXPECT(hx_prefill_workspace_bytes(&c256, HX_PREFILL_MAX_ROWS + 256, &one) == HX_E_RANGE);
        EXPECT(hx_prefill_workspace_bytes(&c256, 256, nullptr) == HX_E_NULL);
        hx_model_config c64 = shapes[0];
        c64.max_batch = 64;
        EXPECT(hx_prefill_workspace_bytes(&c64, 256, &one) == HX_E_RANGE);
    }
    hx_model_config bad = shapes[0];
    bad.head_dim = 96;
    size_t out = 0;
    EXPECT(hx_weights_bytes(&bad, &out) == HX_E_CONFIG);
    EXPECT(hx_weights_bytes(nullptr, &out) == HX_E_NULL);
    EXPECT(hx_engine_destroy(nullptr) == HX_E_NULL && kv_free(nullptr) == HX_E_NULL);
    printf(fails ? "host ABI sanitizer driver: %d FAILED\n" : "host ABI sanitizer driver: OK\n", fails);
    return fails ? 1 : 0;
}
