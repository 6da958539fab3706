// Paged KV cache: scatter / gather between the logical layout [token, kv_head, head_dim] and the
// pool's operand-order tiles, and the per-layer "bias + RoPE + append" kernel that turns the q/k/v
// projection of the new token into the packed query and the cache entry at its position.
#include "hx_internal.h"

// ---- prefill_fill / hx_kv_gather ---------------------------------------------------------------------
// One 64-thread group per (token, kv_head): each thread moves 16 bytes of K and 16 bytes of V
// (head_dim 128: 8 bf16 x 16 threads ... all 64 threads busy over K and V halves).
template <int D, bool GATHER>
__global__ __launch_bounds__(256) void kv_scatter_kernel(char *pool_layer, size_t block_bytes, size_t tile_bytes,
                                                         uint16_t *k_log, uint16_t *v_log,
                                                         const int32_t *__restrict__ seq_start,
                                                         const int32_t *__restrict__ table, int max_blocks,
                                                         int batch, int64_t total_tokens, int n_kv) {
    // thread -> (token, kv_head, chunk of 8 d)
    constexpr int CH = D / 8;
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t per_token = (int64_t)n_kv * CH;
    int64_t tok = gid / per_token;
    if (tok >= total_tokens) return;
    int rem = (int)(gid - tok * per_token);
    int kvh = rem / CH, c = rem % CH;
    // sequence of this token: largest b with seq_start[b] <= tok
    int lo = 0, hi = batch;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if ((int64_t)seq_start[mid] <= tok) lo = mid; else hi = mid;
    }
    int p = (int)(tok - seq_start[lo]);
    int32_t blk = table[(size_t)lo * max_blocks + (p >> 4)];
    int slot = p & 15;
    uint16_t *ktile = (uint16_t *)(pool_layer + (size_t)blk * block_bytes + (size_t)kvh * 2 * tile_bytes);
    uint16_t *vtile = (uint16_t *)((char *)ktile + tile_bytes);
    size_t src = ((size_t)tok * n_kv + kvh) * D + c * 8;
    if (!GATHER) {
        uint4 kk = *(const uint4 *)(k_log + src);
        *(uint4 *)(ktile + hx_ktile_index(slot, c * 8)) = kk;      // 8 consecutive d stay together in a K tile
        uint4 vv = *(const uint4 *)(v_log + src);
        const uint16_t *ve = (const uint16_t *)&vv;
#pragma unroll
        for (int j = 0; j < 8; ++j) vtile[hx_vtile_index(slot, c * 8 + j)] = ve[j];
    } else {
        *(uint4 *)(k_log + src) = *(const uint4 *)(ktile + hx_ktile_index(slot, c * 8));
        uint4 vv;
        uint16_t *ve = (uint16_t *)&vv;
#pragma unroll
        for (int j = 0; j < 8; ++j) ve[j] = vtile[hx_vtile_index(slot, c * 8 + j)];
        *(uint4 *)(v_log + src) = vv;
    }
}

int hx_launch_kv_scatter(const hx_kv *kv, int layer, const void *k, const void *v, const int32_t *seq_start,
                         const int32_t *table, int max_blocks, int batch, int64_t total_tokens, bool gather,
                         hipStream_t st) {
    const hx_engine *e = kv->engine;
    if (total_tokens == 0) return HX_OK;
    int D = e->D, n_kv = e->cfg.n_kv_heads;
    int64_t threads = total_tokens * n_kv * (D / 8);
    int64_t blocks = (threads + 255) / 256;
    if (blocks > 0x7fffffffLL) return hx_fail(HX_E_RANGE, "total_tokens too large for one launch");
    char *pool_layer = kv->pool + (size_t)layer * kv->layer_bytes;
    dim3 grid((unsigned)blocks), block(256);
#define HX_KV_LAUNCH(DD, GG)                                                                                   \
    hipLaunchKernelGGL((kv_scatter_kernel<DD, GG>), grid, block, 0, st, pool_layer, kv->block_bytes,          \
                       kv->tile_bytes, (uint16_t *)k, (uint16_t *)v, seq_start, table, max_blocks, batch,     \
                       total_tokens, n_kv)
    if (D == 128) { if (gather) HX_KV_LAUNCH(128, true); else HX_KV_LAUNCH(128, false); }
    else          { if (gather) HX_KV_LAUNCH(64, true);  else HX_KV_LAUNCH(64, false); }
#undef HX_KV_LAUNCH
    HX_CHECK_LAUNCH("kv_scatter");
    return HX_OK;
}

// ---- bias + RoPE + append -------------------------------------------------------------------------------
// grid = batch, 256 threads.  The q/k/v projection arrives as `splits` fp32 partial results
// [split][batch][qkv_dim] (summed here in split order), the bias is added, q and k heads are rotated
// by the position's angles (pairs (i, i + D/2)), q is written as the packed bf16 B operand of the
// attention kernel, k and v are rounded to bf16 and stored at (block_table[b][pos/16], pos%16).
template <int D>
__global__ __launch_bounds__(256) void rope_append_kernel(const float *__restrict__ ypart, int splits,
                                                          size_t split_stride, const uint16_t *__restrict__ bias,
                                                          int has_bias, const float *__restrict__ cs,
                                                          const int32_t *__restrict__ positions,
                                                          const int32_t *__restrict__ table, int max_blocks,
                                                          char *pool_layer, size_t block_bytes, size_t tile_bytes,
                                                          uint16_t *__restrict__ qp, int n_q, int n_kv, int G,
                                                          int max_batch) {
    constexpr int HALF = D / 2;
    const int b = blockIdx.x;
    const int qkv_dim = (n_q + 2 * n_kv) * D;
    const float *cosv = cs + (size_t)b * HALF;
    const float *sinv = cs + (size_t)max_batch * HALF + (size_t)b * HALF;
    const int pos = positions[b];
    const int32_t blk = table[(size_t)b * max_blocks + (pos >> 4)];
    const int slot = pos & 15;

    auto value = [&](int col) -> float {
        float s = 0.f;
        for (int sp = 0; sp < splits; ++sp) s += ypart[sp * split_stride + (size_t)b * qkv_dim + col];
        if (has_bias) s += hx_bf16_to_f32(bias[col]);
        return s;
    };

    // rotated heads: q heads then k heads, one thread per pair (i, i + HALF)
    const int rot_pairs = (n_q + n_kv) * HALF;
    for (int idx = threadIdx.x; idx < rot_pairs; idx += blockDim.x) {
        int head = idx / HALF, i = idx % HALF;
        float a = value(head * D + i), c2 = value(head * D + i + HALF);
        float c = cosv[i], s = sinv[i];
        float r0 = a * c - c2 * s, r1 = c2 * c + a * s;
        if (head < n_q) {
            int kvh = head / G, g = head % G;
            uint16_t *dst = qp + ((size_t)b * n_kv + kvh) * (D / 32) * 512;
            int d0 = i, d1 = i + HALF;
            dst[(d0 >> 5) * 512 + ((((d0 >> 3) & 3) * 16 + g) << 3) + (d0 & 7)] = hx_f32_to_bf16(r0);
            dst[(d1 >> 5) * 512 + ((((d1 >> 3) & 3) * 16 + g) << 3) + (d1 & 7)] = hx_f32_to_bf16(r1);
        } else {
            int kvh = head - n_q;
            uint16_t *ktile = (uint16_t *)(pool_layer + (size_t)blk * block_bytes + (size_t)kvh * 2 * tile_bytes);
            ktile[hx_ktile_index(slot, i)] = hx_f32_to_bf16(r0);
            ktile[hx_ktile_index(slot, i + HALF)] = hx_f32_to_bf16(r1);
        }
    }
    // v heads: plain rounding
    for (int idx = threadIdx.x; idx < n_kv * D; idx += blockDim.x) {
        int kvh = idx / D, d = idx % D;
        uint16_t *vtile = (uint16_t *)(pool_layer + (size_t)blk * block_bytes + (size_t)kvh * 2 * tile_bytes + tile_bytes);
        vtile[hx_vtile_index(slot, d)] = hx_f32_to_bf16(value((n_q + n_kv) * D + idx));
    }
    // unused query rows g >= G of every packed operand are zero
    if (G < 16) {
        const int zero_per_kvh = (16 - G) * D;
        for (int idx = threadIdx.x; idx < n_kv * zero_per_kvh; idx += blockDim.x) {
            int kvh = idx / zero_per_kvh, r = idx % zero_per_kvh;
            int g = G + r / D, d = r % D;
            uint16_t *dst = qp + ((size_t)b * n_kv + kvh) * (D / 32) * 512;
            dst[(d >> 5) * 512 + ((((d >> 3) & 3) * 16 + g) << 3) + (d & 7)] = 0;
        }
    }
}

int hx_launch_rope_append(const hx_engine *e, const hx_kv *kv, int layer, int batch, const float *ypart,
                          int splits, size_t split_stride, const int32_t *positions, const int32_t *table,
                          int max_blocks, hipStream_t st) {
    const hx_layer_map &lm = e->layers[layer];
    char *pool_layer = kv->pool + (size_t)layer * kv->layer_bytes;
    const uint16_t *bias = (const uint16_t *)(e->weights + lm.bqkv);
    const float *cs = (const float *)(e->ws + e->map.cs);
    uint16_t *qp = (uint16_t *)(e->ws + e->map.qp);
    dim3 grid(batch), block(256);
    if (e->D == 128)
        hipLaunchKernelGGL((rope_append_kernel<128>), grid, block, 0, st, ypart, splits, split_stride, bias,
                           e->cfg.qkv_bias, cs, positions, table, max_blocks, pool_layer, kv->block_bytes,
                           kv->tile_bytes, qp, e->cfg.n_q_heads, e->cfg.n_kv_heads, e->G, e->cfg.max_batch);
    else
        hipLaunchKernelGGL((rope_append_kernel<64>), grid, block, 0, st, ypart, splits, split_stride, bias,
                           e->cfg.qkv_bias, cs, positions, table, max_blocks, pool_layer, kv->block_bytes,
                           kv->tile_bytes, qp, e->cfg.n_q_heads, e->cfg.n_kv_heads, e->G, e->cfg.max_batch);
    HX_CHECK_LAUNCH("rope_append");
    return HX_OK;
}
