// The C ABI: argument validation, buffer maps, and the launch sequence of one decode step.
// All device work is enqueued on the caller's stream; nothing here allocates device memory.
#include "hx_internal.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

// ---- errors ------------------------------------------------------------------------------------------------------
static thread_local char g_err[512] = "";

int hx_fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

extern "C" const char *hx_last_error(void) { return g_err; }

// ---- configuration and maps --------------------------------------------------------------------------------------
static size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

static int env_int(const char *name, int dflt) {
    const char *s = getenv(name);
    if (!s || !*s) return dflt;
    return atoi(s);
}

static int check_config(const hx_model_config *c) {
    if (!c) return hx_fail(HX_E_NULL, "config is NULL");
    if (c->struct_size != sizeof(hx_model_config))
        return hx_fail(HX_E_CONFIG, "struct_size %u, expected %zu", c->struct_size, sizeof(hx_model_config));
    if (c->n_layers < 1 || c->vocab < 1) return hx_fail(HX_E_CONFIG, "n_layers and vocab must be positive");
    if (c->head_dim != 64 && c->head_dim != 128) return hx_fail(HX_E_CONFIG, "head_dim %d: only 64 and 128", c->head_dim);
    if (c->n_kv_heads < 1 || c->n_q_heads < 1 || c->n_q_heads % c->n_kv_heads != 0)
        return hx_fail(HX_E_CONFIG, "n_q_heads %d must be a positive multiple of n_kv_heads %d", c->n_q_heads, c->n_kv_heads);
    if (c->n_q_heads / c->n_kv_heads > 16) return hx_fail(HX_E_CONFIG, "more than 16 query heads per KV head");
    if (c->hidden < 32 || c->hidden % 32 != 0 || c->hidden > HX_MAX_HIDDEN)
        return hx_fail(HX_E_CONFIG, "hidden %d must be a multiple of 32 in [32, %d]", c->hidden, HX_MAX_HIDDEN);
    if (c->intermediate < 16 || c->intermediate % 16 != 0)
        return hx_fail(HX_E_CONFIG, "intermediate %d must be a positive multiple of 16", c->intermediate);
    if (c->vocab % 4 != 0) return hx_fail(HX_E_CONFIG, "vocab %d must be a multiple of 4", c->vocab);
    if (c->block_size != HX_BLOCK_TOKENS) return hx_fail(HX_E_CONFIG, "block_size %d: only 16", c->block_size);
    if (c->max_batch < 1 || c->max_batch > 256) return hx_fail(HX_E_CONFIG, "max_batch %d not in [1, 256]", c->max_batch);
    if (c->max_seq_len < 1 || c->max_seq_len > (1 << 20)) return hx_fail(HX_E_CONFIG, "max_seq_len %d not in [1, 2^20]", c->max_seq_len);
    if (!(c->rms_eps > 0.f) || !(c->rope_theta > 1.f)) return hx_fail(HX_E_CONFIG, "rms_eps must be > 0 and rope_theta > 1");
    if (c->kv_dtype != HX_KV_BF16 && c->kv_dtype != HX_KV_FP8_E4M3)
        return hx_fail(HX_E_CONFIG, "kv_dtype %d: HX_KV_BF16 or HX_KV_FP8_E4M3", c->kv_dtype);
    return HX_OK;
}

// Compute units of the current device, asked once; 256 (an MI355X) where no device can be asked, so that the size
// queries and the launch planner also answer on a host without a GPU.
int hx_device_cus() {
    static std::once_flag once;
    static int cus = 256;
    std::call_once(once, [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
        (void)hipGetLastError();
    });
    return cus;
}

static int attention_waves() {      // 8 wavefronts per compute unit (all resident at once); HX_ATTN_WAVES overrides (tuning)
    int w = env_int("HX_ATTN_WAVES", 8 * hx_device_cus());
    if (w < 64) w = 64;
    if (w > 16384) w = 16384;
    return w;
}

static void init_matrix(hx_matrix *m, size_t *at, int K, int N, bool gate_up) {
    m->K = K;
    m->N = gate_up ? 2 * N : N;
    m->k_steps = K / 16;
    m->n_tiles = gate_up ? N / 16 : (N + 31) / 32;
    m->offset = *at;
    *at = align_up(*at + (size_t)m->n_tiles * m->k_steps * 1024);
}

struct derived {
    int G, D, q_dim, kv_dim, qkv_dim;
};
static derived derive(const hx_model_config *c) {
    derived d;
    d.D = c->head_dim;
    d.G = c->n_q_heads / c->n_kv_heads;
    d.q_dim = c->n_q_heads * c->head_dim;
    d.kv_dim = c->n_kv_heads * c->head_dim;
    d.qkv_dim = d.q_dim + 2 * d.kv_dim;
    return d;
}

// fills e->layers (if not NULL), e->embed/gf/wlm and returns the total weight bytes
static size_t map_weights(hx_engine *e) {
    const hx_model_config *c = &e->cfg;
    size_t at = 0;
    for (int l = 0; l < c->n_layers; ++l) {
        hx_layer_map tmp;
        hx_layer_map *lm = e->layers ? &e->layers[l] : &tmp;
        init_matrix(&lm->wqkv, &at, c->hidden, e->qkv_dim, false);
        init_matrix(&lm->wo, &at, e->q_dim, c->hidden, false);
        init_matrix(&lm->wgu, &at, c->hidden, c->intermediate, true);
        init_matrix(&lm->wd, &at, c->intermediate, c->hidden, false);
        lm->g1 = at; at = align_up(at + (size_t)c->hidden * 2);
        lm->g2 = at; at = align_up(at + (size_t)c->hidden * 2);
        lm->bqkv = at; at = align_up(at + (size_t)e->qkv_dim * 2);
    }
    e->embed = at; at = align_up(at + (size_t)c->vocab * c->hidden * 2);
    e->gf = at; at = align_up(at + (size_t)c->hidden * 2);
    init_matrix(&e->wlm, &at, c->hidden, c->vocab, false);
    return at;
}

static size_t map_workspace(hx_engine *e) {
    const hx_model_config *c = &e->cfg;
    hx_ws_map *m = &e->map;
    const size_t B = c->max_batch, MG = hx_m_groups(c->max_batch);
    size_t at = 0;
    auto take = [&](size_t bytes) { size_t o = at; at = align_up(at + bytes); return o; };
    m->x = take(B * c->hidden * 4);
    m->xp = take((size_t)(c->hidden / 16) * MG * 1024);
    m->ap = take((size_t)(e->q_dim / 16) * MG * 1024);
    m->mp = take((size_t)(c->intermediate / 16) * MG * 1024);
    size_t wide = (size_t)(e->qkv_dim > c->hidden ? e->qkv_dim : c->hidden);
    m->ypart = take((size_t)HX_MAX_SPLITS * B * wide * 4);
    m->qp = take(B * c->n_kv_heads * (size_t)(e->D / 32) * 1024 + 16 * (size_t)e->D * 2);   // + one K tile of slack: the attention
                                                                                          // kernel may read a whole K|V tile starting at any query
    m->cs = take(2 * B * (e->D / 2) * 4);
    m->pre = take(HX_PREFIX_LEN * 4);
    m->lens = take(256 * 4);
    m->sched = take(256);
    m->blk_new = take(256 * 4);
    const size_t slots = (size_t)e->attn_waves + B * c->n_kv_heads;
    m->part_ml = take(slots * 32 * 4);
    m->part_o = take(slots * e->G * e->D * 4);
    m->chunk_cont = take(256 * 4);
    m->chunk_ginfo = take(256 * 4);
    m->chunk_rgrp = take(256 * 4);
    m->chunk_part_ml = take(slots * 4 * 32 * 4);
    m->chunk_part_o = take(slots * 4 * 16 * e->D * 4);
    m->amax_val = take(B * e->wlm.n_tiles * 4);
    m->amax_idx = take(B * e->wlm.n_tiles * 4);
    m->samp_z = take(B * e->wlm.n_tiles * 4);
    m->samp_m = take(B * e->wlm.n_tiles * 4);
    m->samp_s = take(B * e->wlm.n_tiles * 4);
    size_t widest = wide;
    if ((size_t)c->intermediate > widest) widest = c->intermediate;
    if ((size_t)e->q_dim > widest) widest = e->q_dim;
    m->scratch_f32 = take(B * widest * 4);
    m->total = at;
    return at;
}

static int init_engine_shape(hx_engine *e, const hx_model_config *cfg) {
    int rc = check_config(cfg);
    if (rc) return rc;
    memset(e, 0, sizeof(*e));
    e->cfg = *cfg;
    derived d = derive(cfg);
    e->G = d.G; e->D = d.D; e->q_dim = d.q_dim; e->kv_dim = d.kv_dim; e->qkv_dim = d.qkv_dim;
    e->m_groups_max = hx_m_groups(cfg->max_batch);
    e->attn_waves = attention_waves();
    // HX_CHUNK_ATTENTION=0: prompt rows go through the decode step's attention, one K/V stream per row (comparison)
    const char *ca = getenv("HX_CHUNK_ATTENTION");
    e->chunk_attention = !(ca && atoi(ca) == 0);
    e->chunk_rows = 64 / e->G < HX_CHUNK_ROWS ? 64 / e->G : HX_CHUNK_ROWS;     // G <= 16: at least 4 rows
    return HX_OK;
}

extern "C" int hx_weights_bytes(const hx_model_config *cfg, size_t *out) {
    if (!out) return hx_fail(HX_E_NULL, "out is NULL");
    hx_engine e;
    int rc = init_engine_shape(&e, cfg);
    if (rc) return rc;
    *out = map_weights(&e);
    return HX_OK;
}

extern "C" int hx_workspace_bytes(const hx_model_config *cfg, size_t *out) {
    if (!out) return hx_fail(HX_E_NULL, "out is NULL");
    hx_engine e;
    int rc = init_engine_shape(&e, cfg);
    if (rc) return rc;
    map_weights(&e);
    *out = map_workspace(&e);
    return HX_OK;
}

extern "C" int hx_kv_bytes(const hx_model_config *cfg, int64_t num_blocks, size_t *out) {
    if (!out) return hx_fail(HX_E_NULL, "out is NULL");
    int rc = check_config(cfg);
    if (rc) return rc;
    if (num_blocks < 1 || num_blocks > (int64_t)0x7fffffff) return hx_fail(HX_E_RANGE, "num_blocks %lld out of range", (long long)num_blocks);
    const size_t elem = cfg->kv_dtype == HX_KV_FP8_E4M3 ? 1 : 2;
    *out = (size_t)cfg->n_layers * (size_t)num_blocks * cfg->n_kv_heads * 2 * (16 * (size_t)cfg->head_dim * elem);
    return HX_OK;
}

static int check_dev_buffer(const void *p, size_t have, size_t need, const char *what) {
    if (!p) return hx_fail(HX_E_NULL, "%s is NULL", what);
    if (((uintptr_t)p & 255) != 0) return hx_fail(HX_E_ALIGN, "%s is not 256-byte aligned", what);
    if (have < need) return hx_fail(HX_E_TOO_SMALL, "%s has %zu bytes, needs %zu", what, have, need);
    return HX_OK;
}

extern "C" int hx_engine_create(const hx_model_config *cfg, void *weights_dev, size_t weights_bytes, void *workspace_dev,
                                size_t workspace_bytes, hx_engine **out) {
    if (!out) return hx_fail(HX_E_NULL, "out is NULL");
    *out = nullptr;
    hx_engine shape;
    int rc = init_engine_shape(&shape, cfg);
    if (rc) return rc;
    hx_engine *e = new (std::nothrow) hx_engine(shape);
    if (!e) return hx_fail(HX_E_HIP, "out of host memory");
    e->layers = new (std::nothrow) hx_layer_map[cfg->n_layers];
    if (!e->layers) { delete e; return hx_fail(HX_E_HIP, "out of host memory"); }
    size_t wneed = map_weights(e);
    size_t sneed = map_workspace(e);
    if ((rc = check_dev_buffer(weights_dev, weights_bytes, wneed, "weights buffer")) ||
        (rc = check_dev_buffer(workspace_dev, workspace_bytes, sneed, "workspace"))) {
        delete[] e->layers;
        delete e;
        return rc;
    }
    e->weights = (char *)weights_dev;
    e->ws = (char *)workspace_dev;
    e->weights_bytes = weights_bytes;
    e->ws_bytes = workspace_bytes;
    e->profile_mask = 0;
    e->profile_stride = 1;
    e->profile_events = new (std::nothrow) std::vector<std::pair<hipEvent_t, hipEvent_t>>[HX_K_COUNT];
    *out = e;
    return HX_OK;
}

extern "C" int hx_engine_destroy(hx_engine *e) {
    if (!e) return hx_fail(HX_E_NULL, "engine is NULL");
    if (e->profile_events) {
        for (int k = 0; k < HX_K_COUNT; ++k)
            for (auto &p : e->profile_events[k]) { (void)hipEventDestroy(p.first); (void)hipEventDestroy(p.second); }
        delete[] e->profile_events;
    }
    delete[] e->layers;
    delete e;
    return HX_OK;
}

extern "C" int hx_attention_waves(const hx_engine *e) { return e ? e->attn_waves : hx_fail(HX_E_NULL, "engine is NULL"); }

extern "C" int hx_set_attn_capture(hx_engine *e, float *attn_dev) {
    if (!e) return hx_fail(HX_E_NULL, "engine is NULL");
    e->attn_capture = attn_dev;
    return HX_OK;
}

// ---- weight packing ----------------------------------------------------------------------------------------------
extern "C" int hx_weights_pack(hx_engine *e, int kind, int layer, const void *src, int64_t rows, int64_t cols, void *stream) {
    if (!e) return hx_fail(HX_E_NULL, "engine is NULL");
    if (!src) return hx_fail(HX_E_NULL, "src is NULL");
    hipStream_t st = (hipStream_t)stream;
    const hx_model_config *c = &e->cfg;
    const bool per_layer = !(kind == HX_T_EMBED || kind == HX_T_GF || kind == HX_T_WLM);
    if (per_layer && (layer < 0 || layer >= c->n_layers)) return hx_fail(HX_E_SHAPE, "layer %d out of range", layer);
    const hx_layer_map *lm = per_layer ? &e->layers[layer] : nullptr;
    auto want = [&](int64_t r, int64_t cc) -> int {
        if (rows != r || cols != cc)
            return hx_fail(HX_E_SHAPE, "tensor kind %d: got [%lld, %lld], expected [%lld, %lld]", kind, (long long)rows,
                           (long long)cols, (long long)r, (long long)cc);
        return HX_OK;
    };
    auto copy_vec = [&](size_t off, size_t n) -> int {
        HX_CHECK_HIP(hipMemcpyAsync(e->weights + off, src, n * 2, hipMemcpyDeviceToDevice, st));
        return HX_OK;
    };
    int rc;
    switch (kind) {
        case HX_T_EMBED: if ((rc = want(c->vocab, c->hidden))) return rc; return copy_vec(e->embed, (size_t)c->vocab * c->hidden);
        case HX_T_GF:    if ((rc = want(c->hidden, 1)) && (rc = want(1, c->hidden))) return rc; return copy_vec(e->gf, c->hidden);
        case HX_T_G1:    if ((rc = want(c->hidden, 1)) && (rc = want(1, c->hidden))) return rc; return copy_vec(lm->g1, c->hidden);
        case HX_T_G2:    if ((rc = want(c->hidden, 1)) && (rc = want(1, c->hidden))) return rc; return copy_vec(lm->g2, c->hidden);
        case HX_T_BQKV:  if ((rc = want(e->qkv_dim, 1)) && (rc = want(1, e->qkv_dim))) return rc; return copy_vec(lm->bqkv, e->qkv_dim);
        case HX_T_WQKV:  if ((rc = want(c->hidden, e->qkv_dim))) return rc; return hx_launch_pack_matrix(e, &lm->wqkv, src, rows, cols, 0, st);
        case HX_T_WO:    if ((rc = want(e->q_dim, c->hidden))) return rc; return hx_launch_pack_matrix(e, &lm->wo, src, rows, cols, 0, st);
        case HX_T_WG:    if ((rc = want(c->hidden, c->intermediate))) return rc; return hx_launch_pack_matrix(e, &lm->wgu, src, rows, cols, 1, st);
        case HX_T_WU:    if ((rc = want(c->hidden, c->intermediate))) return rc; return hx_launch_pack_matrix(e, &lm->wgu, src, rows, cols, 2, st);
        case HX_T_WD:    if ((rc = want(c->intermediate, c->hidden))) return rc; return hx_launch_pack_matrix(e, &lm->wd, src, rows, cols, 0, st);
        case HX_T_WLM:   if ((rc = want(c->hidden, c->vocab))) return rc; return hx_launch_pack_matrix(e, &e->wlm, src, rows, cols, 0, st);
        default: return hx_fail(HX_E_SHAPE, "unknown tensor kind %d", kind);
    }
}

// ---- KV cache ------------------------------------------------------------------------------------------------------
extern "C" int kv_alloc(hx_engine *e, void *kv_dev, size_t kv_bytes, int64_t num_blocks, hx_kv **out) {
    if (!out) return hx_fail(HX_E_NULL, "out is NULL");
    *out = nullptr;
    if (!e) return hx_fail(HX_E_NULL, "engine is NULL");
    size_t need;
    int rc = hx_kv_bytes(&e->cfg, num_blocks, &need);
    if (rc) return rc;
    if ((rc = check_dev_buffer(kv_dev, kv_bytes, need, "kv pool"))) return rc;
    hx_kv *kv = new (std::nothrow) hx_kv;
    if (!kv) return hx_fail(HX_E_HIP, "out of host memory");
    kv->engine = e;
    kv->pool = (char *)kv_dev;
    kv->num_blocks = num_blocks;
    kv->fp8 = e->cfg.kv_dtype == HX_KV_FP8_E4M3;
    kv->tile_bytes = 16 * (size_t)e->D * (kv->fp8 ? 1 : 2);
    kv->block_bytes = (size_t)e->cfg.n_kv_heads * 2 * kv->tile_bytes;
    kv->layer_bytes = (size_t)num_blocks * kv->block_bytes;
    *out = kv;
    return HX_OK;
}

extern "C" int kv_free(hx_kv *kv) {
    if (!kv) return hx_fail(HX_E_NULL, "kv is NULL");
    delete kv;
    return HX_OK;
}

static int check_table_args(const hx_kv *kv, int layer, const void *a, const void *b, const void *c, const void *d,
                            int32_t max_blocks, int32_t batch) {
    if (!kv) return hx_fail(HX_E_NULL, "kv is NULL");
    if (!a || !b || !c || !d) return hx_fail(HX_E_NULL, "a device pointer argument is NULL");
    if (layer < 0 || layer >= kv->engine->cfg.n_layers) return hx_fail(HX_E_SHAPE, "layer %d out of range", layer);
    if (batch < 1) return hx_fail(HX_E_RANGE, "batch %d must be positive", batch);
    if (max_blocks < 1) return hx_fail(HX_E_RANGE, "max_blocks_per_seq %d must be positive", max_blocks);
    return HX_OK;
}

extern "C" int prefill_fill(hx_kv *kv, int layer, const void *k_dev, const void *v_dev, const int32_t *seq_start_dev,
                            const int32_t *block_table_dev, int32_t max_blocks, int32_t batch, int64_t total_tokens,
                            void *stream) {
    int rc = check_table_args(kv, layer, k_dev, v_dev, seq_start_dev, block_table_dev, max_blocks, batch);
    if (rc) return rc;
    if (total_tokens < 0) return hx_fail(HX_E_RANGE, "total_tokens negative");
    return hx_launch_kv_scatter(kv, layer, k_dev, v_dev, seq_start_dev, block_table_dev, max_blocks, batch, total_tokens,
                                false, (hipStream_t)stream);
}

extern "C" int hx_kv_gather(hx_kv *kv, int layer, void *k_out_dev, void *v_out_dev, const int32_t *seq_start_dev,
                            const int32_t *block_table_dev, int32_t max_blocks, int32_t batch, int64_t total_tokens,
                            void *stream) {
    int rc = check_table_args(kv, layer, k_out_dev, v_out_dev, seq_start_dev, block_table_dev, max_blocks, batch);
    if (rc) return rc;
    if (total_tokens < 0) return hx_fail(HX_E_RANGE, "total_tokens negative");
    return hx_launch_kv_scatter(kv, layer, k_out_dev, v_out_dev, seq_start_dev, block_table_dev, max_blocks, batch,
                                total_tokens, true, (hipStream_t)stream);
}

// ---- per-kernel timing ---------------------------------------------------------------------------------------------
struct timed_launch {   // brackets one launch with two events when its class is selected
    hx_engine *e; int k; hipStream_t st; hipEvent_t a = nullptr, b = nullptr;
    timed_launch(hx_engine *e_, int k_, hipStream_t st_) : e(e_), k(k_), st(st_) {
        if (e->profile_events && (e->profile_mask >> k) & 1u && e->profile_seen[k]++ % e->profile_stride == 0) {
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { a = b = nullptr; return; }
            (void)hipEventRecord(a, st);
        }
    }
    ~timed_launch() {
        if (a) { (void)hipEventRecord(b, st); e->profile_events[k].push_back({a, b}); }
    }
};
#define HX_TIMED(klass, call) do { timed_launch t_(e, klass, st); if ((rc = (call))) return rc; } while (0)

extern "C" int hx_profile_enable(hx_engine *e, uint32_t class_mask) {
    if (!e) return hx_fail(HX_E_NULL, "engine is NULL");
    if (class_mask >> HX_K_COUNT) return hx_fail(HX_E_RANGE, "class_mask has bits beyond HX_K_COUNT");
    e->profile_mask = class_mask;
    for (int k = 0; k < HX_K_COUNT; ++k) e->profile_seen[k] = 0;
    return HX_OK;
}

extern "C" int hx_profile_sample_every(hx_engine *e, int32_t n) {
    if (!e) return hx_fail(HX_E_NULL, "engine is NULL");
    if (n < 1) return hx_fail(HX_E_RANGE, "sampling stride %d must be at least 1", n);
    e->profile_stride = n;
    return HX_OK;
}

extern "C" int hx_profile_read(hx_engine *e, int kernel_class, double *total_ms_out, int64_t *launches_out) {
    if (!e || !total_ms_out || !launches_out) return hx_fail(HX_E_NULL, "a pointer argument is NULL");
    if (kernel_class < 0 || kernel_class >= HX_K_COUNT) return hx_fail(HX_E_RANGE, "kernel class %d out of range", kernel_class);
    double total = 0.0;
    int64_t n = 0;
    if (e->profile_events) {
        auto &v = e->profile_events[kernel_class];
        for (auto &p : v) {
            HX_CHECK_HIP(hipEventSynchronize(p.second));
            float ms = 0.f;
            HX_CHECK_HIP(hipEventElapsedTime(&ms, p.first, p.second));
            total += ms;
            ++n;
            (void)hipEventDestroy(p.first);
            (void)hipEventDestroy(p.second);
        }
        v.clear();
    }
    *total_ms_out = total;
    *launches_out = n;
    return HX_OK;
}

// ---- the decode step -------------------------------------------------------------------------------------------------
static int check_step_args(const hx_engine *e, const hx_kv *kv, int32_t batch, int32_t max_blocks) {
    if (!e) return hx_fail(HX_E_NULL, "engine is NULL");
    if (kv && kv->engine != e) return hx_fail(HX_E_SHAPE, "kv belongs to another engine");
    if (batch < 1 || batch > e->cfg.max_batch) return hx_fail(HX_E_RANGE, "batch %d not in [1, max_batch %d]", batch, e->cfg.max_batch);
    if (max_blocks < 1) return hx_fail(HX_E_RANGE, "max_blocks_per_seq %d must be positive", max_blocks);
    return HX_OK;
}

static int run_step(hx_engine *e, hx_kv *kv, int32_t batch, const int32_t *tokens, const int32_t *positions,
                    const int32_t *seq_lens, const int32_t *block_table, int32_t max_blocks, float *logits_out,
                    int32_t *next_tokens_out, float *logprobs_out, const hx_sample_params *sample, bool with_head,
                    void *stream) {
    int rc = check_step_args(e, kv, batch, max_blocks);
    if (rc) return rc;
    if (!kv) return hx_fail(HX_E_NULL, "kv is NULL");
    if (!tokens || !positions || !seq_lens || !block_table || (with_head && !next_tokens_out))
        return hx_fail(HX_E_NULL, "a device pointer argument is NULL");
    hipStream_t st = (hipStream_t)stream;
    const hx_model_config *c = &e->cfg;
    char *ws = e->ws;
    float *ypart = (float *)(ws + e->map.ypart);
    const size_t attn_stride = (size_t)batch * e->q_dim;

    HX_TIMED(HX_K_SETUP, hx_launch_step_setup(e, batch, positions, seq_lens, block_table, max_blocks, st));
    // prompt rows: consecutive rows of a sequence share one K/V stream (their schedule replaces the decode step's)
    const bool chunked = !with_head && e->chunk_attention;
    if (chunked) HX_TIMED(HX_K_SETUP, hx_launch_chunk_setup(e, batch, seq_lens, block_table, max_blocks, st));
    HX_TIMED(HX_K_NORM, hx_launch_embed_norm(e, batch, tokens, e->layers[0].g1, st));
    for (int l = 0; l < c->n_layers; ++l) {
        const hx_layer_map *lm = &e->layers[l];
        HX_TIMED(HX_K_GEMM_QKV, hx_launch_gemm(e, &lm->wqkv, batch, ws + e->map.xp, HX_EPI_PARTIAL, ypart, nullptr, st));
        HX_TIMED(HX_K_ROPE, hx_launch_rope_append(e, kv, l, batch, ypart, hx_gemm_splits(&lm->wqkv, batch), (size_t)batch * e->qkv_dim,
                                                 positions, st));
        if (!with_head && l + 1 == c->n_layers) break;   // prompt rows: of the last layer only its K and V are needed
        float *capture = e->attn_capture ? e->attn_capture + l * attn_stride : nullptr;
        if (chunked) {
            HX_TIMED(HX_K_ATTENTION, hx_launch_chunk_attention(e, kv, l, block_table, max_blocks, st));
            HX_TIMED(HX_K_COMBINE, hx_launch_chunk_combine(e, batch, capture, st));
        } else {
            if (kv->fp8) HX_TIMED(HX_K_ATTENTION, hx_launch_attention_fp8(e, kv, l, block_table, max_blocks, st));
            else HX_TIMED(HX_K_ATTENTION, hx_launch_attention(e, kv, l, batch, seq_lens, block_table, max_blocks, st));
            HX_TIMED(HX_K_COMBINE, hx_launch_combine(e, batch, capture, st));
        }
        HX_TIMED(HX_K_GEMM_O, hx_launch_gemm(e, &lm->wo, batch, ws + e->map.ap, HX_EPI_PARTIAL, ypart, nullptr, st));
        HX_TIMED(HX_K_NORM, hx_launch_reduce_norm(e, batch, ypart, hx_gemm_splits(&lm->wo, batch), (size_t)batch * c->hidden, lm->g2, st));
        HX_TIMED(HX_K_GEMM_GATE_UP, hx_launch_gemm(e, &lm->wgu, batch, ws + e->map.xp, HX_EPI_SWIGLU, nullptr, ws + e->map.mp, st));
        HX_TIMED(HX_K_GEMM_DOWN, hx_launch_gemm(e, &lm->wd, batch, ws + e->map.mp, HX_EPI_PARTIAL, ypart, nullptr, st));
        const size_t next_gain = (l + 1 < c->n_layers) ? e->layers[l + 1].g1 : e->gf;
        HX_TIMED(HX_K_NORM, hx_launch_reduce_norm(e, batch, ypart, hx_gemm_splits(&lm->wd, batch), (size_t)batch * c->hidden, next_gain, st));
    }
    if (!with_head) return HX_OK;
    if (sample && sample->top_p < 1.0f) {
        // the kept set needs every logit of the row again: the head writes them (with its per-tile maxima), then
        // one workgroup per row selects and draws
        HX_TIMED(HX_K_GEMM_LM, hx_launch_gemm(e, &e->wlm, batch, ws + e->map.xp, HX_EPI_LOGITS, logits_out, nullptr, st));
        HX_TIMED(HX_K_SETUP, hx_launch_nucleus(e, batch, logits_out, sample, next_tokens_out, logprobs_out, st));
    } else if (sample) {
        HX_TIMED(HX_K_GEMM_LM, hx_launch_gemm(e, &e->wlm, batch, ws + e->map.xp, HX_EPI_SAMPLE, logits_out, nullptr, st, sample));
        HX_TIMED(HX_K_SETUP, hx_launch_sample_final(e, batch, next_tokens_out, logprobs_out, st));
    } else {
        HX_TIMED(HX_K_GEMM_LM, hx_launch_gemm(e, &e->wlm, batch, ws + e->map.xp, HX_EPI_LOGITS, logits_out, nullptr, st));
        HX_TIMED(HX_K_SETUP, hx_launch_argmax_final(e, batch, next_tokens_out, st));
    }
    return HX_OK;
}

extern "C" int decode_step(hx_engine *e, hx_kv *kv, int32_t batch, const int32_t *tokens, const int32_t *positions,
                           const int32_t *seq_lens, const int32_t *block_table, int32_t max_blocks, float *logits_out,
                           int32_t *next_tokens_out, void *stream) {
    return run_step(e, kv, batch, tokens, positions, seq_lens, block_table, max_blocks, logits_out, next_tokens_out,
                    nullptr, nullptr, true, stream);
}

extern "C" int prefill_chunk(hx_engine *e, hx_kv *kv, int32_t n_rows, const int32_t *tokens, const int32_t *positions,
                             const int32_t *seq_lens, const int32_t *block_table, int32_t max_blocks, void *stream) {
    return run_step(e, kv, n_rows, tokens, positions, seq_lens, block_table, max_blocks, nullptr, nullptr, nullptr, nullptr,
                    false, stream);
}

// ---- prompt rows in blocks of 256, the products over all blocks at once ------------------------------------------
// Each block of 256 rows has a workspace of its own, laid out like the engine's; a shallow copy of the engine that
// points at it lets every row kernel and the attention run per block exactly as in prefill_chunk, while each matrix
// product is ONE launch over all blocks (gemm_wide.hip), so a weight is read once per call.
static size_t wide_block_stride(const hx_engine *e) { return align_up(e->map.total, 4096); }

extern "C" int hx_prefill_workspace_bytes(const hx_model_config *cfg, int32_t max_rows, size_t *out) {
    if (!out) return hx_fail(HX_E_NULL, "out is NULL");
    hx_engine e;
    int rc = init_engine_shape(&e, cfg);
    if (rc) return rc;
    if (cfg->max_batch != 256) return hx_fail(HX_E_RANGE, "prefill_rows needs an engine with max_batch 256, not %d", cfg->max_batch);
    if (max_rows < 256 || max_rows > HX_PREFILL_MAX_ROWS || max_rows % 256)
        return hx_fail(HX_E_RANGE, "max_rows %d is not a multiple of 256 in [256, %d]", max_rows, HX_PREFILL_MAX_ROWS);
    map_weights(&e);
    map_workspace(&e);
    *out = (size_t)(max_rows / 256) * wide_block_stride(&e);
    return HX_OK;
}

extern "C" int prefill_rows(hx_engine *e, hx_kv *kv, int32_t n_rows, const int32_t *tokens, const int32_t *positions,
                            const int32_t *seq_lens, const int32_t *block_table, int32_t max_blocks, void *workspace_dev,
                            size_t workspace_bytes, void *stream) {
    if (!e || !kv) return hx_fail(HX_E_NULL, "engine or kv is NULL");
    if (kv->engine != e) return hx_fail(HX_E_SHAPE, "kv belongs to another engine");
    if (!tokens || !positions || !seq_lens || !block_table || !workspace_dev) return hx_fail(HX_E_NULL, "a device pointer argument is NULL");
    const hx_model_config *c = &e->cfg;
    if (c->max_batch != 256) return hx_fail(HX_E_RANGE, "prefill_rows needs an engine with max_batch 256, not %d", c->max_batch);
    if (n_rows < 256 || n_rows > HX_PREFILL_MAX_ROWS || n_rows % 256)
        return hx_fail(HX_E_RANGE, "n_rows %d is not a multiple of 256 in [256, %d] (prefill_chunk takes the remainder)", n_rows,
                       HX_PREFILL_MAX_ROWS);
    if (max_blocks < 1) return hx_fail(HX_E_RANGE, "max_blocks_per_seq %d must be positive", max_blocks);
    if (c->hidden % 32 || c->intermediate % 32 || e->q_dim % 32)
        return hx_fail(HX_E_SHAPE, "prefill_rows needs hidden, intermediate and n_q_heads * head_dim to be multiples of 32");
    const int R = n_rows / 256;
    const size_t stride = wide_block_stride(e);
    if ((uintptr_t)workspace_dev % 256) return hx_fail(HX_E_RANGE, "workspace is not 256-byte aligned");
    if (workspace_bytes < (size_t)R * stride)
        return hx_fail(HX_E_RANGE, "workspace holds %zu bytes, %d rows need %zu (hx_prefill_workspace_bytes)", workspace_bytes, n_rows,
                       (size_t)R * stride);
    hipStream_t st = (hipStream_t)stream;
    char *ws0 = (char *)workspace_dev;
    std::vector<hx_engine> view(R, *e);                  // shallow copies: same weights, schedule sizes and hooks
    for (int b = 0; b < R; ++b) { view[b].ws = ws0 + (size_t)b * stride; view[b].ws_bytes = stride; }
    const hx_ws_map &m = e->map;
    const size_t attn_stride = (size_t)n_rows * e->q_dim;
    int rc;
    auto rows = [&](const int32_t *p, int b) { return p + (size_t)b * 256; };
    auto table = [&](int b) { return block_table + (size_t)b * 256 * max_blocks; };
    const bool chunked = e->chunk_attention;

    // The schedules are per block (one small launch each); the row kernels and the grouped attention take all blocks in
    // one launch (their block dimension strides through the workspaces), as do the products.
    const hx_engine *v0 = &view[0];
    const float *ypart0 = (const float *)(ws0 + m.ypart);
    for (int b = 0; b < R; ++b) {
        const hx_engine *vb = &view[b];
        HX_TIMED(HX_K_SETUP, hx_launch_step_setup(vb, 256, rows(positions, b), rows(seq_lens, b), table(b), max_blocks, st));
        if (chunked) HX_TIMED(HX_K_SETUP, hx_launch_chunk_setup(vb, 256, rows(seq_lens, b), table(b), max_blocks, st));
    }
    HX_TIMED(HX_K_NORM, hx_launch_embed_norm(v0, 256, tokens, e->layers[0].g1, st, R, stride));
    for (int l = 0; l < c->n_layers; ++l) {
        const hx_layer_map *lm = &e->layers[l];
        const hx_wide_plan p_qkv = hx_plan_wide(&lm->wqkv, R, true), p_o = hx_plan_wide(&lm->wo, R, true),
                           p_gu = hx_plan_wide(&lm->wgu, R, false), p_d = hx_plan_wide(&lm->wd, R, true);
        const int s_qkv = p_qkv.splits, s_o = p_o.splits, s_d = p_d.splits;
        HX_TIMED(HX_K_GEMM_QKV, hx_launch_gemm_wide(e, &lm->wqkv, R, ws0, stride, m.xp, HX_EPI_PARTIAL, m.ypart, 0, p_qkv, st));
        // K and V of every row of the call enter the cache before any row attends
        HX_TIMED(HX_K_ROPE, hx_launch_rope_append(v0, kv, l, 256, ypart0, s_qkv, (size_t)256 * e->qkv_dim, positions, st, R, stride));
        if (l + 1 == c->n_layers) break;     // of the last layer only its K and V are needed
        float *capture = e->attn_capture ? e->attn_capture + l * attn_stride : nullptr;
        if (chunked) {
            // one launch over all blocks: each block has its own schedule; the wavefronts beyond a block's runs exit
            HX_TIMED(HX_K_ATTENTION, hx_launch_chunk_attention(v0, kv, l, block_table, max_blocks, st, R, stride, 256));
        } else {
            for (int b = 0; b < R; ++b) {
                const hx_engine *vb = &view[b];
                if (kv->fp8) HX_TIMED(HX_K_ATTENTION, hx_launch_attention_fp8(vb, kv, l, table(b), max_blocks, st));
                else HX_TIMED(HX_K_ATTENTION, hx_launch_attention(vb, kv, l, 256, rows(seq_lens, b), table(b), max_blocks, st));
                HX_TIMED(HX_K_COMBINE, hx_launch_combine(vb, 256, capture ? capture + (size_t)b * 256 * e->q_dim : nullptr, st));
            }
        }
        if (chunked) HX_TIMED(HX_K_COMBINE, hx_launch_chunk_combine(v0, 256, capture, st, R, stride));
        HX_TIMED(HX_K_GEMM_O, hx_launch_gemm_wide(e, &lm->wo, R, ws0, stride, m.ap, HX_EPI_PARTIAL, m.ypart, 0, p_o, st));
        HX_TIMED(HX_K_NORM, hx_launch_reduce_norm(v0, 256, ypart0, s_o, (size_t)256 * c->hidden, lm->g2, st, R, stride));
        HX_TIMED(HX_K_GEMM_GATE_UP, hx_launch_gemm_wide(e, &lm->wgu, R, ws0, stride, m.xp, HX_EPI_SWIGLU, 0, m.mp, p_gu, st));
        HX_TIMED(HX_K_GEMM_DOWN, hx_launch_gemm_wide(e, &lm->wd, R, ws0, stride, m.mp, HX_EPI_PARTIAL, m.ypart, 0, p_d, st));
        const size_t next_gain = (l + 1 < c->n_layers) ? e->layers[l + 1].g1 : e->gf;
        HX_TIMED(HX_K_NORM, hx_launch_reduce_norm(v0, 256, ypart0, s_d, (size_t)256 * c->hidden, next_gain, st, R, stride));
    }
    return HX_OK;
}

extern "C" int decode_step_sample(hx_engine *e, hx_kv *kv, int32_t batch, const int32_t *tokens, const int32_t *positions,
                                  const int32_t *seq_lens, const int32_t *block_table, int32_t max_blocks,
                                  float temperature, uint64_t seed, const int32_t *row_ids, float *logits_out,
                                  int32_t *tokens_out, float *logprobs_out, void *stream) {
    if (!(temperature > 0.0f) || !(temperature < 1e30f))
        return hx_fail(HX_E_RANGE, "temperature %g must be positive and finite", (double)temperature);
    if (!logprobs_out) return hx_fail(HX_E_NULL, "logprobs_out is NULL");
    hx_sample_params sp;
    sp.positions = positions;
    sp.row_ids = row_ids;
    sp.inv_temperature = 1.0f / temperature;
    sp.key0 = (uint32_t)seed;
    sp.key1 = (uint32_t)(seed >> 32);
    sp.top_p = 1.0f;
    sp.nucleus_sizes = nullptr;
    return run_step(e, kv, batch, tokens, positions, seq_lens, block_table, max_blocks, logits_out, tokens_out,
                    logprobs_out, &sp, true, stream);
}

extern "C" int decode_step_top_p(hx_engine *e, hx_kv *kv, int32_t batch, const int32_t *tokens, const int32_t *positions,
                                 const int32_t *seq_lens, const int32_t *block_table, int32_t max_blocks,
                                 float temperature, float top_p, uint64_t seed, const int32_t *row_ids, float *logits_out,
                                 int32_t *tokens_out, float *logprobs_out, int32_t *nucleus_sizes_out, void *stream) {
    if (!(temperature > 0.0f) || !(temperature < 1e30f))
        return hx_fail(HX_E_RANGE, "temperature %g must be positive and finite", (double)temperature);
    if (!(top_p > 0.0f) || !(top_p <= 1.0f)) return hx_fail(HX_E_RANGE, "top_p %g must be in (0, 1]", (double)top_p);
    if (!logprobs_out) return hx_fail(HX_E_NULL, "logprobs_out is NULL");
    if (top_p < 1.0f && !logits_out) return hx_fail(HX_E_NULL, "logits_out is NULL (the kept set is selected from the stored logits)");
    if (top_p >= 1.0f && nucleus_sizes_out) return hx_fail(HX_E_RANGE, "nucleus_sizes_out is only written for top_p < 1");
    hx_sample_params sp;
    sp.positions = positions;
    sp.row_ids = row_ids;
    sp.inv_temperature = 1.0f / temperature;
    sp.key0 = (uint32_t)seed;
    sp.key1 = (uint32_t)(seed >> 32);
    sp.top_p = top_p;
    sp.nucleus_sizes = nucleus_sizes_out;
    return run_step(e, kv, batch, tokens, positions, seq_lens, block_table, max_blocks, logits_out, tokens_out,
                    logprobs_out, &sp, true, stream);
}

// ---- validation of device-side inputs ---------------------------------------------------------------------------
// One thread per row; the first offending row (smallest index) is reported as {code, row, value}.
enum { HX_BAD_NONE = 0, HX_BAD_TOKEN = 1, HX_BAD_POSITION = 2, HX_BAD_SEQ_LEN = 3, HX_BAD_BLOCK = 4 };

__global__ void validate_step_kernel(int batch, const int32_t *__restrict__ tokens, const int32_t *__restrict__ positions,
                                     const int32_t *__restrict__ seq_lens, const int32_t *__restrict__ table,
                                     int max_blocks, int vocab, int max_seq_len, long long num_blocks,
                                     int32_t *__restrict__ report) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    int code = HX_BAD_NONE, value = 0;
    const int tok = tokens[b], pos = positions[b], T = seq_lens[b];
    if (tok < 0 || tok >= vocab) { code = HX_BAD_TOKEN; value = tok; }
    else if (pos < 0 || pos >= max_seq_len || (long long)pos >= (long long)max_blocks * 16) { code = HX_BAD_POSITION; value = pos; }
    else if (T != pos + 1) { code = HX_BAD_SEQ_LEN; value = T; }
    else {
        const int nblk = (T + 15) >> 4;                       // <= max_blocks by the position check
        for (int i = 0; i < nblk; ++i) {
            const int blk = table[(size_t)b * max_blocks + i];
            if (blk < 0 || (long long)blk >= num_blocks) { code = HX_BAD_BLOCK; value = blk; break; }
        }
    }
    (void)value;
    if (code != HX_BAD_NONE) atomicMin(&report[0], b * 8 + code);   // smallest offending row wins, with its reason
}

extern "C" int hx_validate_step_inputs(hx_engine *e, hx_kv *kv, int32_t batch, const int32_t *tokens, const int32_t *positions,
                                       const int32_t *seq_lens, const int32_t *block_table, int32_t max_blocks, void *stream) {
    int rc = check_step_args(e, kv, batch, max_blocks);
    if (rc) return rc;
    if (!kv) return hx_fail(HX_E_NULL, "kv is NULL");
    if (!tokens || !positions || !seq_lens || !block_table) return hx_fail(HX_E_NULL, "a device pointer argument is NULL");
    hipStream_t st = (hipStream_t)stream;
    int32_t *report = (int32_t *)(e->ws + e->map.sched) + 8;             // 3 words of the per-step table area
    const int32_t init = 0x7fffffff;
    HX_CHECK_HIP(hipMemcpyAsync(report, &init, sizeof(init), hipMemcpyHostToDevice, st));
    hipLaunchKernelGGL(validate_step_kernel, dim3((batch + 63) / 64), dim3(64), 0, st, batch, tokens, positions, seq_lens,
                       block_table, max_blocks, e->cfg.vocab, e->cfg.max_seq_len, (long long)kv->num_blocks, report);
    HX_CHECK_LAUNCH("validate_step");
    int32_t out = 0;
    HX_CHECK_HIP(hipMemcpyAsync(&out, report, sizeof(out), hipMemcpyDeviceToHost, st));
    HX_CHECK_HIP(hipStreamSynchronize(st));
    if (out == 0x7fffffff) return HX_OK;
    const int row = out >> 3, code = out & 7;
    int32_t value = 0;
    const int32_t *src = code == HX_BAD_TOKEN ? tokens : code == HX_BAD_POSITION ? positions : seq_lens;
    HX_CHECK_HIP(hipMemcpy(&value, src + row, sizeof(value), hipMemcpyDeviceToHost));
    switch (code) {
        case HX_BAD_TOKEN: return hx_fail(HX_E_RANGE, "row %d: token id %d is outside [0, %d)", row, value, e->cfg.vocab);
        case HX_BAD_POSITION: return hx_fail(HX_E_RANGE, "row %d: position %d is outside the engine's max_seq_len %d or the %d table entries",
                                             row, value, e->cfg.max_seq_len, max_blocks);
        case HX_BAD_SEQ_LEN: return hx_fail(HX_E_RANGE, "row %d: seq_len %d is not position + 1", row, value);
        default: return hx_fail(HX_E_RANGE, "row %d: a block id among its first %d table entries is outside [0, %lld)", row,
                                (value + 15) / 16, (long long)kv->num_blocks);
    }
}

// ---- single stages ---------------------------------------------------------------------------------------------------
extern "C" int hx_stage_schedule(hx_engine *e, int32_t batch, const int32_t *seq_lens, int32_t *prefix_out,
                                 int32_t *sched_out, void *stream) {
    int rc = check_step_args(e, nullptr, batch, 1);
    if (rc) return rc;
    if (!seq_lens || !prefix_out || !sched_out) return hx_fail(HX_E_NULL, "a device pointer argument is NULL");
    hipStream_t st = (hipStream_t)stream;
    if ((rc = hx_launch_step_setup(e, batch, nullptr, seq_lens, nullptr, 0, st))) return rc;
    HX_CHECK_HIP(hipMemcpyAsync(prefix_out, e->ws + e->map.pre, ((size_t)batch + 1) * 4, hipMemcpyDeviceToDevice, st));
    HX_CHECK_HIP(hipMemcpyAsync(sched_out, e->ws + e->map.sched, 8, hipMemcpyDeviceToDevice, st));
    return HX_OK;
}

extern "C" int hx_stage_rope_append(hx_engine *e, hx_kv *kv, int layer, int32_t batch, const float *qkv_dev,
                                    const int32_t *positions, const int32_t *block_table, int32_t max_blocks,
                                    float *q_out_dev, void *stream) {
    int rc = check_step_args(e, kv, batch, max_blocks);
    if (rc) return rc;
    if (!kv || !qkv_dev || !positions || !block_table || !q_out_dev) return hx_fail(HX_E_NULL, "a pointer argument is NULL");
    if (layer < 0 || layer >= e->cfg.n_layers) return hx_fail(HX_E_SHAPE, "layer %d out of range", layer);
    hipStream_t st = (hipStream_t)stream;
    if ((rc = hx_launch_step_setup(e, batch, positions, nullptr, block_table, max_blocks, st))) return rc;
    if ((rc = hx_launch_rope_append(e, kv, layer, batch, qkv_dev, 1, 0, positions, st))) return rc;
    return hx_launch_unpack_q(e, batch, q_out_dev, st);
}

extern "C" int hx_stage_attention(hx_engine *e, hx_kv *kv, int layer, int32_t batch, const float *q_dev,
                                  const int32_t *seq_lens, const int32_t *block_table, int32_t max_blocks,
                                  float *out_dev, void *stream) {
    int rc = check_step_args(e, kv, batch, max_blocks);
    if (rc) return rc;
    if (!kv || !q_dev || !seq_lens || !block_table || !out_dev) return hx_fail(HX_E_NULL, "a pointer argument is NULL");
    if (layer < 0 || layer >= e->cfg.n_layers) return hx_fail(HX_E_SHAPE, "layer %d out of range", layer);
    hipStream_t st = (hipStream_t)stream;
    if ((rc = hx_launch_pack_q(e, batch, q_dev, st))) return rc;
    if ((rc = hx_launch_step_setup(e, batch, nullptr, seq_lens, nullptr, 0, st))) return rc;
    if (kv->fp8) rc = hx_launch_attention_fp8(e, kv, layer, block_table, max_blocks, st);
    else rc = hx_launch_attention(e, kv, layer, batch, seq_lens, block_table, max_blocks, st);
    if (rc) return rc;
    return hx_launch_combine(e, batch, out_dev, st);
}

// ---- the attention stage without a workspace ---------------------------------------------------------------------
// For callers that cannot provide or allocate scratch memory (code under graph capture, tight serving loops,
// harnesses that forbid allocation): the packed queries, the schedule and the split-K partial results of
// hx_stage_attention live in a file-scope device array of fixed size instead of the engine's workspace.  Each GPU
// holds its own copy of the array at its own address; the address is asked once per device (hipGetSymbolAddress)
// and only that pointer is ever handed to kernels.
static __device__ __align__(256) unsigned char hx_static_scratch[HX_STATIC_SCRATCH_BYTES];

#define HX_MAX_DEVICES 64
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[HX_MAX_DEVICES];      // per device; NULL until first used there

static int static_scratch_of_current_device(char **out) {
    int dev = -1;
    HX_CHECK_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= HX_MAX_DEVICES) return hx_fail(HX_E_RANGE, "device ordinal %d outside [0, %d)", dev, HX_MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HX_CHECK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(hx_static_scratch)));
        if (!p) return hx_fail(HX_E_HIP, "hipGetSymbolAddress returned no address for the static scratch array");
        g_scratch_ptr[dev] = p;
    }
    *out = (char *)g_scratch_ptr[dev];
    return HX_OK;
}

extern "C" int hx_stage_attention_static(hx_engine *e, hx_kv *kv, int layer, int32_t batch, const float *q_dev,
                                         const int32_t *seq_lens, const int32_t *block_table, int32_t max_blocks,
                                         float *out_dev, void *stream) {
    int rc = check_step_args(e, kv, batch, max_blocks);
    if (rc) return rc;
    if (!kv || !q_dev || !seq_lens || !block_table || !out_dev) return hx_fail(HX_E_NULL, "a pointer argument is NULL");
    if (layer < 0 || layer >= e->cfg.n_layers) return hx_fail(HX_E_SHAPE, "layer %d out of range", layer);
    // carve the array: packed queries (+ one K tile of slack, see map_workspace), schedule, partial results
    const size_t slots = (size_t)e->attn_waves + (size_t)batch * e->cfg.n_kv_heads;
    size_t at = 0;
    auto take = [&](size_t bytes) { size_t o = at; at = align_up(at + bytes); return o; };
    const size_t o_qp = take((size_t)batch * e->cfg.n_kv_heads * (size_t)(e->D / 32) * 1024 + 16 * (size_t)e->D * 2);
    const size_t o_pre = take(HX_PREFIX_LEN * 4), o_lens = take(256 * 4), o_sched = take(256);
    const size_t o_ml = take(slots * 32 * 4), o_o = take(slots * e->G * e->D * 4);
    if (at > (size_t)HX_STATIC_SCRATCH_BYTES)
        return hx_fail(HX_E_RANGE, "this call needs %zu bytes of scratch (batch %d, %d KV heads, %d query heads per KV head, head "
                       "size %d, %d wavefronts); the static array holds %d: use hx_stage_attention with a workspace",
                       at, batch, e->cfg.n_kv_heads, e->G, e->D, e->attn_waves, HX_STATIC_SCRATCH_BYTES);
    char *base = nullptr;
    if ((rc = static_scratch_of_current_device(&base))) return rc;
    const hx_attn_bufs bufs{(uint16_t *)(base + o_qp), (int32_t *)(base + o_pre), (int32_t *)(base + o_lens),
                            (int32_t *)(base + o_sched), (float *)(base + o_ml), (float *)(base + o_o), nullptr};
    hipStream_t st = (hipStream_t)stream;
    // Nothing has to start at zero: every word of the array that a kernel of this call reads was written by an earlier
    // kernel of the same call (queries of all batch rows incl. their zero padding, the whole schedule, every partial
    // slot the combine visits), except the slack behind the last query, which only feeds masked-out positions.
    if ((rc = hx_launch_pack_q(e, batch, q_dev, st, &bufs))) return rc;
    if ((rc = hx_launch_step_setup(e, batch, nullptr, seq_lens, nullptr, 0, st, &bufs))) return rc;
    if (kv->fp8) rc = hx_launch_attention_fp8(e, kv, layer, block_table, max_blocks, st, &bufs);
    else rc = hx_launch_attention(e, kv, layer, batch, seq_lens, block_table, max_blocks, st, &bufs);
    if (rc) return rc;
    return hx_launch_combine(e, batch, out_dev, st, &bufs);
}

extern "C" int hx_stage_rmsnorm(hx_engine *e, int gain_kind, int layer, int32_t batch, const float *x_dev, float *y_dev,
                                void *stream) {
    int rc = check_step_args(e, nullptr, batch, 1);
    if (rc) return rc;
    if (!x_dev || !y_dev) return hx_fail(HX_E_NULL, "a pointer argument is NULL");
    size_t off;
    if (gain_kind == HX_T_GF) off = e->gf;
    else {
        if (layer < 0 || layer >= e->cfg.n_layers) return hx_fail(HX_E_SHAPE, "layer %d out of range", layer);
        if (gain_kind == HX_T_G1) off = e->layers[layer].g1;
        else if (gain_kind == HX_T_G2) off = e->layers[layer].g2;
        else return hx_fail(HX_E_SHAPE, "tensor kind %d is not a gain", gain_kind);
    }
    return hx_launch_norm_only(e, batch, x_dev, off, y_dev, (hipStream_t)stream);
}

extern "C" int hx_stage_lm_head_top_p(hx_engine *e, int32_t batch, const float *x_dev, const int32_t *positions,
                                      const int32_t *row_ids, float temperature, float top_p, uint64_t seed,
                                      float *logits_out, int32_t *tokens_out, float *logprobs_out,
                                      int32_t *nucleus_sizes_out, void *stream) {
    int rc = check_step_args(e, nullptr, batch, 1);
    if (rc) return rc;
    if (!x_dev || !positions || !logits_out || !tokens_out || !logprobs_out) return hx_fail(HX_E_NULL, "a pointer argument is NULL");
    if (!(temperature > 0.0f) || !(temperature < 1e30f))
        return hx_fail(HX_E_RANGE, "temperature %g must be positive and finite", (double)temperature);
    if (!(top_p > 0.0f) || !(top_p < 1.0f)) return hx_fail(HX_E_RANGE, "top_p %g must be in (0, 1)", (double)top_p);
    hipStream_t st = (hipStream_t)stream;
    hx_sample_params sp;
    sp.positions = positions;
    sp.row_ids = row_ids;
    sp.inv_temperature = 1.0f / temperature;
    sp.key0 = (uint32_t)seed;
    sp.key1 = (uint32_t)(seed >> 32);
    sp.top_p = top_p;
    sp.nucleus_sizes = nucleus_sizes_out;
    if ((rc = hx_launch_pack_x(e, batch, x_dev, e->cfg.hidden, e->ws + e->map.xp, st))) return rc;
    if ((rc = hx_launch_gemm(e, &e->wlm, batch, e->ws + e->map.xp, HX_EPI_LOGITS, logits_out, nullptr, st))) return rc;
    return hx_launch_nucleus(e, batch, logits_out, &sp, tokens_out, logprobs_out, st);
}

// One product of prefill_rows alone, on caller-supplied rows: x [n_rows, K] fp32 (rounded to bf16 on entry) -> y
// [n_rows, N] fp32; for HX_T_WG y [n_rows, intermediate] = bf16(SiLU(gate) * up) as fp32.  Same kernels, plan and
// workspace layout as prefill_rows.
extern "C" int hx_stage_linear_rows(hx_engine *e, int kind, int layer, int32_t n_rows, const float *x_dev, float *y_dev,
                                    void *workspace_dev, size_t workspace_bytes, void *stream) {
    if (!e) return hx_fail(HX_E_NULL, "engine is NULL");
    if (!x_dev || !y_dev || !workspace_dev) return hx_fail(HX_E_NULL, "a pointer argument is NULL");
    const hx_model_config *c = &e->cfg;
    if (c->max_batch != 256) return hx_fail(HX_E_RANGE, "wide products need an engine with max_batch 256, not %d", c->max_batch);
    if (n_rows < 256 || n_rows > HX_PREFILL_MAX_ROWS || n_rows % 256)
        return hx_fail(HX_E_RANGE, "n_rows %d is not a multiple of 256 in [256, %d]", n_rows, HX_PREFILL_MAX_ROWS);
    if (layer < 0 || layer >= c->n_layers) return hx_fail(HX_E_SHAPE, "layer %d out of range", layer);
    const int R = n_rows / 256;
    const size_t stride = wide_block_stride(e);
    if ((uintptr_t)workspace_dev % 256) return hx_fail(HX_E_RANGE, "workspace is not 256-byte aligned");
    if (workspace_bytes < (size_t)R * stride)
        return hx_fail(HX_E_RANGE, "workspace holds %zu bytes, %d rows need %zu (hx_prefill_workspace_bytes)", workspace_bytes, n_rows,
                       (size_t)R * stride);
    hipStream_t st = (hipStream_t)stream;
    char *ws0 = (char *)workspace_dev;
    const hx_layer_map *lm = &e->layers[layer];
    const hx_ws_map &m = e->map;
    const hx_matrix *w;
    size_t in_off;
    int K, N;
    switch (kind) {
        case HX_T_WQKV: w = &lm->wqkv; in_off = m.xp; K = c->hidden; N = e->qkv_dim; break;
        case HX_T_WO: w = &lm->wo; in_off = m.ap; K = e->q_dim; N = c->hidden; break;
        case HX_T_WG: w = &lm->wgu; in_off = m.xp; K = c->hidden; N = c->intermediate; break;
        case HX_T_WD: w = &lm->wd; in_off = m.mp; K = c->intermediate; N = c->hidden; break;
        default: return hx_fail(HX_E_SHAPE, "tensor kind %d has no wide product", kind);
    }
    const bool swiglu = kind == HX_T_WG;
    const hx_wide_plan plan = hx_plan_wide(w, R, !swiglu);
    hx_engine view = *e;
    int rc;
    for (int b = 0; b < R; ++b) {
        view.ws = ws0 + (size_t)b * stride;
        if ((rc = hx_launch_pack_x(&view, 256, x_dev + (size_t)b * 256 * K, K, view.ws + in_off, st))) return rc;
    }
    if ((rc = hx_launch_gemm_wide(e, w, R, ws0, stride, in_off, swiglu ? HX_EPI_SWIGLU : HX_EPI_PARTIAL, m.ypart, m.mp, plan, st))) return rc;
    for (int b = 0; b < R; ++b) {
        view.ws = ws0 + (size_t)b * stride;
        float *y = y_dev + (size_t)b * 256 * N;
        if (swiglu) rc = hx_launch_unpack_x(&view, 256, view.ws + m.mp, N, y, st);
        else rc = hx_launch_sum_partials(&view, 256, (const float *)(view.ws + m.ypart), plan.splits, (size_t)256 * N, N, y, st);
        if (rc) return rc;
    }
    return HX_OK;
}

extern "C" int hx_stage_linear(hx_engine *e, int kind, int layer, int32_t batch, const float *x_dev, float *y_dev,
                               int32_t *argmax_out_dev, void *stream) {
    int rc = check_step_args(e, nullptr, batch, 1);
    if (rc) return rc;
    if (!x_dev || !y_dev) return hx_fail(HX_E_NULL, "a pointer argument is NULL");
    if (kind != HX_T_WLM && argmax_out_dev) return hx_fail(HX_E_SHAPE, "argmax_out_dev only with HX_T_WLM");
    if (kind != HX_T_WLM && (layer < 0 || layer >= e->cfg.n_layers)) return hx_fail(HX_E_SHAPE, "layer %d out of range", layer);
    hipStream_t st = (hipStream_t)stream;
    const hx_model_config *c = &e->cfg;
    char *ws = e->ws;
    float *ypart = (float *)(ws + e->map.ypart);
    const hx_layer_map *lm = (kind == HX_T_WLM) ? nullptr : &e->layers[layer];
    switch (kind) {
        case HX_T_WQKV:
            if ((rc = hx_launch_pack_x(e, batch, x_dev, c->hidden, ws + e->map.xp, st))) return rc;
            if ((rc = hx_launch_gemm(e, &lm->wqkv, batch, ws + e->map.xp, HX_EPI_PARTIAL, ypart, nullptr, st))) return rc;
            return hx_launch_sum_partials(e, batch, ypart, hx_gemm_splits(&lm->wqkv, batch), (size_t)batch * e->qkv_dim, e->qkv_dim, y_dev, st);
        case HX_T_WO:
            if ((rc = hx_launch_pack_x(e, batch, x_dev, e->q_dim, ws + e->map.ap, st))) return rc;
            if ((rc = hx_launch_gemm(e, &lm->wo, batch, ws + e->map.ap, HX_EPI_PARTIAL, ypart, nullptr, st))) return rc;
            return hx_launch_sum_partials(e, batch, ypart, hx_gemm_splits(&lm->wo, batch), (size_t)batch * c->hidden, c->hidden, y_dev, st);
        case HX_T_WG:
            if ((rc = hx_launch_pack_x(e, batch, x_dev, c->hidden, ws + e->map.xp, st))) return rc;
            if ((rc = hx_launch_gemm(e, &lm->wgu, batch, ws + e->map.xp, HX_EPI_SWIGLU, nullptr, ws + e->map.mp, st))) return rc;
            return hx_launch_unpack_x(e, batch, ws + e->map.mp, c->intermediate, y_dev, st);
        case HX_T_WD:
            if ((rc = hx_launch_pack_x(e, batch, x_dev, c->intermediate, ws + e->map.mp, st))) return rc;
            if ((rc = hx_launch_gemm(e, &lm->wd, batch, ws + e->map.mp, HX_EPI_PARTIAL, ypart, nullptr, st))) return rc;
            return hx_launch_sum_partials(e, batch, ypart, hx_gemm_splits(&lm->wd, batch), (size_t)batch * c->hidden, c->hidden, y_dev, st);
        case HX_T_WLM:
            if ((rc = hx_launch_pack_x(e, batch, x_dev, c->hidden, ws + e->map.xp, st))) return rc;
            if ((rc = hx_launch_gemm(e, &e->wlm, batch, ws + e->map.xp, HX_EPI_LOGITS, y_dev, nullptr, st))) return rc;
            if (argmax_out_dev) return hx_launch_argmax_final(e, batch, argmax_out_dev, st);
            return HX_OK;
        default:
            return hx_fail(HX_E_SHAPE, "tensor kind %d is not a matrix", kind);
    }
}
