// Paged KV cache: scatter / gather between the logical layout [token, kv_head, head_dim] and the
// pool's operand-order tiles, and the per-layer "bias + RoPE + append" kernel that turns the q/k/v
// projection of the new token into the packed query and the cache entry at its position.
#include "hx_internal.h"

// ---- prefill_fill / hx_kv_gather ---------------------------------------------------------------------
// One 64-thread group per (token, kv_head): each thread moves 16 bytes of K and 16 bytes of V
// (head_dim 128: 8 bf16 x 16 threads ... all 64 threads busy over K and V halves).
template <int D, bool GATHER, bool FP8>
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
    if (FP8) {
        // 8-bit cache: bf16 <-> E4M3 on the way (rounding on the way in, exact on the way out)
        uint8_t *k8 = (uint8_t *)ktile, *v8 = (uint8_t *)vtile;
        if (!GATHER) {
            const uint4 kk = *(const uint4 *)(k_log + src), vv = *(const uint4 *)(v_log + src);
            const uint16_t *ke = (const uint16_t *)&kk, *ve = (const uint16_t *)&vv;
            float kf[8], vf[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) { kf[j] = hx_bf16_to_f32(ke[j]); vf[j] = hx_bf16_to_f32(ve[j]); }
            *(uint2 *)(k8 + hx_ktile8_index(slot, c * 8)) = hx_pack8_e4m3(kf);
            const uint2 vp = hx_pack8_e4m3(vf);
            const uint8_t *vb = (const uint8_t *)&vp;
#pragma unroll
            for (int j = 0; j < 8; ++j) v8[hx_vtile8_index(slot, c * 8 + j)] = vb[j];
        } else {
            const uint2 kp = *(const uint2 *)(k8 + hx_ktile8_index(slot, c * 8));
            const uint2 k03 = hx_e4m3x4_to_bf16x4(kp.x), k47 = hx_e4m3x4_to_bf16x4(kp.y);
            *(uint4 *)(k_log + src) = make_uint4(k03.x, k03.y, k47.x, k47.y);
            uint2 vp;
            uint8_t *vb = (uint8_t *)&vp;
#pragma unroll
            for (int j = 0; j < 8; ++j) vb[j] = v8[hx_vtile8_index(slot, c * 8 + j)];
            const uint2 v03 = hx_e4m3x4_to_bf16x4(vp.x), v47 = hx_e4m3x4_to_bf16x4(vp.y);
            *(uint4 *)(v_log + src) = make_uint4(v03.x, v03.y, v47.x, v47.y);
        }
        return;
    }
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
#define HX_KV_LAUNCH(DD, GG, F8)                                                                               \
    hipLaunchKernelGGL((kv_scatter_kernel<DD, GG, F8>), grid, block, 0, st, pool_layer, kv->block_bytes,      \
                       kv->tile_bytes, (uint16_t *)k, (uint16_t *)v, seq_start, table, max_blocks, batch,     \
                       total_tokens, n_kv)
#define HX_KV_LAUNCH_D(DD)                                                                                     \
    do {                                                                                                       \
        if (kv->fp8) { if (gather) HX_KV_LAUNCH(DD, true, true); else HX_KV_LAUNCH(DD, false, true); }        \
        else         { if (gather) HX_KV_LAUNCH(DD, true, false); else HX_KV_LAUNCH(DD, false, false); }      \
    } while (0)
    if (D == 128) HX_KV_LAUNCH_D(128);
    else          HX_KV_LAUNCH_D(64);
#undef HX_KV_LAUNCH_D
#undef HX_KV_LAUNCH
    HX_CHECK_LAUNCH("kv_scatter");
    return HX_OK;
}

// ---- bias + RoPE + append -------------------------------------------------------------------------------
// The q/k/v projection arrives as `splits` fp32 partial results [split][batch][qkv_dim] (summed here in
// split order), the bias is added, q and k heads are rotated by the position's angles (pairs (i, i + D/2)),
// q is written as the packed bf16 B operand of the attention kernel, k and v are rounded to bf16 (or, for an 8-bit
// cache, from fp32 straight to E4M3) and stored
// at (block_table[b][pos/16], pos%16); the block id comes from the per-step table written by step_setup_kernel.
// One thread per work item of 16 values: for q and k heads, 8 consecutive d of the lower half and the 8
// matching d of the upper half (both ends of the rotation, two 16-byte stores); for v, 16 consecutive d.
// grid (batch, ceil(items / 128)), 128 threads.  Query rows g >= G of the packed operand are never written:
// they only feed accumulator columns that nobody reads.
template <int D, bool FP8>
__global__ __launch_bounds__(128) void rope_append_kernel(const float *__restrict__ ypart, int splits,
                                                          size_t split_stride, const uint16_t *__restrict__ bias,
                                                          int has_bias, const float *__restrict__ cs,
                                                          const int32_t *__restrict__ positions,
                                                          const int32_t *__restrict__ blk_new,
                                                          char *pool_layer, size_t block_bytes, size_t tile_bytes,
                                                          uint16_t *__restrict__ qp, int n_q, int n_kv, int G,
                                                          int max_batch, size_t block_stride) {
    constexpr int HALF = D / 2;
    constexpr int RPH = HALF / 8;                         // rotation items per head
    const int b = blockIdx.x;
    if (blockIdx.z) {               // further row blocks of a wide prompt call: same layout, block_stride bytes apart
        const size_t off = (size_t)blockIdx.z * block_stride;
        ypart = (const float *)((const char *)ypart + off);
        cs = (const float *)((const char *)cs + off);
        blk_new = (const int32_t *)((const char *)blk_new + off);
        qp = (uint16_t *)((char *)qp + off);
        positions += (size_t)blockIdx.z * gridDim.x;
    }
    const int item = blockIdx.y * blockDim.x + threadIdx.x;
    const int rot_items = (n_q + n_kv) * RPH;
    const int v_items = n_kv * (D / 16);
    if (item >= rot_items + v_items) return;
    const int qkv_dim = (n_q + 2 * n_kv) * D;
    const int pos = positions[b];
    const int32_t blk = blk_new[b];                     // block of position pos, looked up once per step
    const int slot = pos & 15;

    auto gather8 = [&](int col, float *out) {            // sum of the split partials + bias, 8 consecutive columns
        // every partial is requested before the first is used; they are added in split order
        f32x4_t ya[HX_MAX_SPLITS], yc[HX_MAX_SPLITS];
#pragma unroll
        for (int sp = 0; sp < HX_MAX_SPLITS; ++sp) {
            const float *src = ypart + min(sp, splits - 1) * split_stride + (size_t)b * qkv_dim + col;
            ya[sp] = *(const f32x4_t *)src;
            yc[sp] = *(const f32x4_t *)(src + 4);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) out[j] = 0.f;
#pragma unroll
        for (int sp = 0; sp < HX_MAX_SPLITS; ++sp) {
            if (sp < splits) {
#pragma unroll
                for (int j = 0; j < 4; ++j) { out[j] += ya[sp][j]; out[4 + j] += yc[sp][j]; }
            }
        }
        if (has_bias) {
            const uint4 raw = *(const uint4 *)(bias + col);
            const uint16_t *b16 = (const uint16_t *)&raw;
#pragma unroll
            for (int j = 0; j < 8; ++j) out[j] += hx_bf16_to_f32(b16[j]);
        }
    };
    auto pack8 = [](const float *v) {
        uint4 pk;
        pk.x = hx_cvt_pk_bf16(v[0], v[1]); pk.y = hx_cvt_pk_bf16(v[2], v[3]);
        pk.z = hx_cvt_pk_bf16(v[4], v[5]); pk.w = hx_cvt_pk_bf16(v[6], v[7]);
        return pk;
    };

    if (item < rot_items) {
        const int head = item / RPH, i0 = (item % RPH) * 8;
        float lo[8], hi[8], r0[8], r1[8];
        gather8(head * D + i0, lo);
        gather8(head * D + HALF + i0, hi);
        const float *cosv = cs + (size_t)b * HALF + i0;
        const float *sinv = cs + (size_t)max_batch * HALF + (size_t)b * HALF + i0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float c = cosv[j], sn = sinv[j];
            r0[j] = lo[j] * c - hi[j] * sn;
            r1[j] = hi[j] * c + lo[j] * sn;
        }
        if (head < n_q) {
            const int kvh = head / G, g = head % G;
            uint16_t *dst = qp + ((size_t)b * n_kv + kvh) * (D / 32) * 512;
            const int d0 = i0, d1 = i0 + HALF;
            *(uint4 *)(dst + (d0 >> 5) * 512 + ((((d0 >> 3) & 3) * 16 + g) << 3)) = pack8(r0);
            *(uint4 *)(dst + (d1 >> 5) * 512 + ((((d1 >> 3) & 3) * 16 + g) << 3)) = pack8(r1);
        } else {
            const int kvh = head - n_q;
            char *ktile = pool_layer + (size_t)blk * block_bytes + (size_t)kvh * 2 * tile_bytes;
            if (FP8) {                                     // 8-bit cache: fp32 -> E4M3 directly
                *(uint2 *)(ktile + hx_ktile8_index(slot, i0)) = hx_pack8_e4m3(r0);
                *(uint2 *)(ktile + hx_ktile8_index(slot, i0 + HALF)) = hx_pack8_e4m3(r1);
            } else {
                *(uint4 *)((uint16_t *)ktile + hx_ktile_index(slot, i0)) = pack8(r0);
                *(uint4 *)((uint16_t *)ktile + hx_ktile_index(slot, i0 + HALF)) = pack8(r1);
            }
        }
    } else {
        const int vi = item - rot_items;
        const int kvh = vi / (D / 16), d0 = (vi % (D / 16)) * 16;
        uint16_t *vtile = (uint16_t *)(pool_layer + (size_t)blk * block_bytes + (size_t)kvh * 2 * tile_bytes + tile_bytes);
        float v[8];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            gather8((n_q + n_kv) * D + kvh * D + d0 + 8 * h, v);
            if (FP8) {
                const uint2 vp = hx_pack8_e4m3(v);
                const uint8_t *vb = (const uint8_t *)&vp;
#pragma unroll
                for (int j = 0; j < 8; ++j) ((uint8_t *)vtile)[hx_vtile8_index(slot, d0 + 8 * h + j)] = vb[j];
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) vtile[hx_vtile_index(slot, d0 + 8 * h + j)] = hx_f32_to_bf16(v[j]);
            }
        }
    }
}

int hx_launch_rope_append(const hx_engine *e, const hx_kv *kv, int layer, int batch, const float *ypart,
                          int splits, size_t split_stride, const int32_t *positions, hipStream_t st, int blocks,
                          size_t block_stride) {
    const hx_layer_map &lm = e->layers[layer];
    char *pool_layer = kv->pool + (size_t)layer * kv->layer_bytes;
    const uint16_t *bias = (const uint16_t *)(e->weights + lm.bqkv);
    const float *cs = (const float *)(e->ws + e->map.cs);
    uint16_t *qp = (uint16_t *)(e->ws + e->map.qp);
    const int items = (e->cfg.n_q_heads + e->cfg.n_kv_heads) * (e->D / 16) + e->cfg.n_kv_heads * (e->D / 16);
    dim3 grid(batch, (items + 127) / 128, blocks), block(128);
#define HX_ROPE_LAUNCH(DD, F8)                                                                                  \
    hipLaunchKernelGGL((rope_append_kernel<DD, F8>), grid, block, 0, st, ypart, splits, split_stride, bias,    \
                       e->cfg.qkv_bias, cs, positions, (const int32_t *)(e->ws + e->map.blk_new), pool_layer, kv->block_bytes, \
                       kv->tile_bytes, qp, e->cfg.n_q_heads, e->cfg.n_kv_heads, e->G, e->cfg.max_batch, block_stride)
    if (e->D == 128) { if (kv->fp8) HX_ROPE_LAUNCH(128, true); else HX_ROPE_LAUNCH(128, false); }
    else             { if (kv->fp8) HX_ROPE_LAUNCH(64, true);  else HX_ROPE_LAUNCH(64, false); }
#undef HX_ROPE_LAUNCH
    HX_CHECK_LAUNCH("rope_append");
    return HX_OK;
}
