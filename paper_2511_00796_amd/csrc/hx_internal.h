// Internal declarations shared by the translation units of libhexdecode.so (gfx950 only).
//
// Data layouts (all chosen so that one wavefront load instruction -- 64 lanes x 16 bytes --
// covers 1 KiB of contiguous memory and lands directly in matrix-core operand order):
//
//  * packed weight matrix W [K, N] -> [n_tile][k_step][lane 0..63][8 bf16]:
//        element (lane, j) = W[16*k_step + 8*(lane/32) + j][32*n_tile + lane%32]
//    i.e. the A operand (32 rows n x 16 k) of v_mfma_f32_32x32x16_bf16; columns >= N are zero.
//    The gate and up projections share one packed matrix with 16 gate columns followed by the
//    16 matching up columns in every n_tile, so both land in the same lane of the accumulator.
//
//  * packed activations X [M, K] (bf16) -> [k_step][m_group][lane][8 bf16]:
//        element (lane, j) = X[32*m_group + lane%32][16*k_step + 8*(lane/32) + j]
//    i.e. the B operand (16 k x 32 columns m) of the same instruction.
//
//  * packed query of one (sequence, KV head): [kk][lane][8 bf16], kk < head_dim/32:
//        element (lane, j) = q[head = kvh*G + lane%16][32*kk + 8*(lane/16) + j]; lanes with lane%16 >= G are never
//        written or interpreted (they only feed accumulator columns that nobody reads)
//    i.e. the B operand (32 k x 16 columns g) of v_mfma_f32_16x16x32_bf16.
//
//  * KV pool: [layer][block][kv_head][K tile | V tile]; a tile holds 16 tokens x head_dim:
//      K tile [kk][lane][8]:  (lane, j) = K[token lane%16][32*kk + 8*(lane/16) + j]
//                             (A operand, 16 tokens x 32 k, of v_mfma_f32_16x16x32_bf16)
//      V tile [i][lane][8]:   (lane, 4*half + jj) = V[token 4*(lane/16) + jj][32*i + 16*half + lane%16]
//                             (two A operands, 16 rows d x 16 k tokens, of v_mfma_f32_16x16x16_bf16)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <vector>
#include <utility>

#include "../../include/hexdecode.h"

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

#define HX_WAVE 64
#define HX_BLOCK_TOKENS 16
#define HX_MAX_HIDDEN 8192
#define HX_PREFIX_LEN 320    // entries of the per-step block prefix (max_batch 256 + 1, padded to 5 x 64)
#define HX_CHUNK_ROWS 8      // most consecutive prompt rows of one sequence that share a K/V stream (rows x G <= 64 columns)
#define HX_MAX_SPLITS 9       // K-splits of a product whose partials are summed by its consumer kernel

// ---- error reporting (api.hip) -------------------------------------------------------------------
int hx_fail(int code, const char *fmt, ...);
int hx_device_cus();   // compute units of the current device (256 where none can be asked)
#define HX_CHECK_HIP(expr)                                                                         \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess) return hx_fail(HX_E_HIP, "%s: %s", #expr, hipGetErrorString(e_));    \
    } while (0)
#define HX_CHECK_LAUNCH(name)                                                                      \
    do {                                                                                           \
        hipError_t e_ = hipGetLastError();                                                         \
        if (e_ != hipSuccess) return hx_fail(HX_E_HIP, "launch %s: %s", name, hipGetErrorString(e_)); \
    } while (0)

// ---- small device helpers ------------------------------------------------------------------------
__device__ __forceinline__ float hx_bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// fp32 -> E4M3 (nearest even; the conversion instruction of gfx950 follows the OCP format), saturating at +-448:
// 8 values into 8 bytes, value j in byte j
__device__ __forceinline__ uint2 hx_pack8_e4m3(const float *v) {
    float c[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) c[j] = fminf(fmaxf(v[j], -448.0f), 448.0f);
    int w0 = __builtin_amdgcn_cvt_pk_fp8_f32(c[0], c[1], 0, false);
    w0 = __builtin_amdgcn_cvt_pk_fp8_f32(c[2], c[3], w0, true);
    int w1 = __builtin_amdgcn_cvt_pk_fp8_f32(c[4], c[5], 0, false);
    w1 = __builtin_amdgcn_cvt_pk_fp8_f32(c[6], c[7], w1, true);
    return make_uint2((uint32_t)w0, (uint32_t)w1);
}
// 4 E4M3 bytes of one dword -> 4 bf16 (exact), byte j -> element j
typedef __bf16 hx_bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint2 hx_e4m3x4_to_bf16x4(uint32_t w) {
    const hx_bf16x2_t lo = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false);
    const hx_bf16x2_t hi = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true);
    return make_uint2(__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi));
}
// Registers holding operands that were converted for a matrix instruction die with that instruction, so the
// compiler may hand them to the next vector instruction.  In the 8-bit attention kernel an ordinary vector add that
// wrote such registers a few issue slots behind the 16x16x32 matrix instruction reading them gave deterministic wrong
// scores on ragged tiles (gone with every wait forced; gone with the operands held two or more wait states, not with
// one).  Operands that stay live -- the bf16 kernels multiply straight out of their load registers, and what follows
// their products closely are accumulator-register reads, which are harmless -- are not exposed.  These statements keep
// short-lived operands live for four wait states.  The form with `acc` is the one for 16x16x32 products: it also
// takes the products' accumulator as an in-out operand, which orders it behind the last product of the chain (an
// asm statement that only names the operands may be scheduled in front of a product that is still to read them --
// seen in builds with other ring depths, where the add then followed the product directly).
template <int N>
__device__ __forceinline__ void hx_hold_operands(const unsigned int __attribute__((ext_vector_type(4))) (&op)[N]) {
    if constexpr (N == 4) asm volatile("s_nop 3" : : "v"(op[0]), "v"(op[1]), "v"(op[2]), "v"(op[3]));
    else if constexpr (N == 2) asm volatile("s_nop 3" : : "v"(op[0]), "v"(op[1]));
    else static_assert(N == 2 || N == 4, "operand steps of head sizes 64 and 128");
}
template <int N>
__device__ __forceinline__ void hx_hold_operands(const unsigned int __attribute__((ext_vector_type(4))) (&op)[N],
                                                 f32x4_t &acc) {
    if constexpr (N == 4) asm volatile("s_nop 3" : "+v"(acc) : "v"(op[0]), "v"(op[1]), "v"(op[2]), "v"(op[3]));
    else if constexpr (N == 2) asm volatile("s_nop 3" : "+v"(acc) : "v"(op[0]), "v"(op[1]));
    else static_assert(N == 2 || N == 4, "operand steps of head sizes 64 and 128");
}
template <int N>
__device__ __forceinline__ void hx_hold_operands(const unsigned int __attribute__((ext_vector_type(4))) (&op)[N],
                                                 const unsigned int __attribute__((ext_vector_type(4))) (&op2)[N],
                                                 f32x4_t &acc) {
    if constexpr (N == 4)
        asm volatile("s_nop 3" : "+v"(acc) : "v"(op[0]), "v"(op[1]), "v"(op[2]), "v"(op[3]), "v"(op2[0]), "v"(op2[1]),
                     "v"(op2[2]), "v"(op2[3]));
    else if constexpr (N == 2) asm volatile("s_nop 3" : "+v"(acc) : "v"(op[0]), "v"(op[1]), "v"(op2[0]), "v"(op2[1]));
    else static_assert(N == 2 || N == 4, "operand steps of head sizes 64 and 128");
}

// round-to-nearest-even on the upper half of the fp32 pattern (finite inputs)
__device__ __forceinline__ uint16_t hx_f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ uint32_t hx_pack_bf16x2(float lo, float hi) {
    return (uint32_t)hx_f32_to_bf16(lo) | ((uint32_t)hx_f32_to_bf16(hi) << 16);
}

// two fp32 -> packed bf16 pair with the hardware conversion (round-to-nearest-even)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t hx_cvt_pk_bf16(float lo, float hi) {
    f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// m-groups (of 32 rows) of the packed activation buffers for a batch: rounded up to 1, 2, 4 or 8 so that
// producers and the matrix products agree on one layout per batch size
__host__ __device__ __forceinline__ int hx_m_groups(int batch) {
    int g = (batch + 31) / 32;
    return g <= 1 ? 1 : (g <= 2 ? 2 : (g <= 4 ? 4 : 8));
}

// element offset (in bf16) of activation (m, k) inside a packed X buffer with m_groups groups
__host__ __device__ __forceinline__ size_t hx_xp_index(int m, int k, int m_groups) {
    int ks = k >> 4, h = (k >> 3) & 1, j = k & 7;
    return (((size_t)ks * m_groups + (m >> 5)) * 64 + (h * 32 + (m & 31))) * 8 + j;
}

// element offsets (in bf16) inside one K / V tile of 16 tokens x head_dim
__host__ __device__ __forceinline__ int hx_ktile_index(int t, int d) {
    return (d >> 5) * 512 + ((((d >> 3) & 3) * 16 + t) << 3) + (d & 7);
}
__host__ __device__ __forceinline__ int hx_vtile_index(int t, int d) {
    return (d >> 5) * 512 + ((((t >> 2) * 16) + (d & 15)) << 3) + (((d >> 4) & 1) << 2) + (t & 3);
}

// The same tiles with 1-byte elements (8-bit cache): the 8 bytes a lane holds for operand step 2p and the 8 it holds
// for step 2p + 1 sit side by side, so that one 16-byte load per lane (1 KiB per wavefront) fetches two steps:
//   byte index = (step / 2) * 1024 + lane * 16 + (step % 2) * 8 + (byte within the lane's 8), lane and byte as above.
__host__ __device__ __forceinline__ int hx_ktile8_index(int t, int d) {
    return (d >> 6) * 1024 + ((((d >> 3) & 3) * 16 + t) << 4) + (((d >> 5) & 1) << 3) + (d & 7);
}
__host__ __device__ __forceinline__ int hx_vtile8_index(int t, int d) {
    return (d >> 6) * 1024 + ((((t >> 2) * 16) + (d & 15)) << 4) + (((d >> 5) & 1) << 3) + (((d >> 4) & 1) << 2) + (t & 3);
}

// ---- host-side descriptors ------------------------------------------------------------------------

struct hx_matrix {          // one packed weight matrix
    size_t offset;          // byte offset in the weight buffer
    int K, N;               // logical shape
    int k_steps, n_tiles;   // K / 16, ceil(N / 32) (gate|up: intermediate / 16)
};

struct hx_layer_map {
    hx_matrix wqkv, wo, wgu, wd;
    size_t g1, g2, bqkv;    // byte offsets of bf16 vectors
};

struct hx_ws_map {          // byte offsets in the workspace
    size_t x;               // fp32 [max_batch, hidden]            residual stream
    size_t xp;              // bf16 packed [hidden/16][MG][64][8]  normalised activations
    size_t ap;              // bf16 packed [q_dim/16][MG][64][8]   attention output
    size_t mp;              // bf16 packed [inter/16][MG][64][8]   SwiGLU output
    size_t ypart;           // fp32 [max_splits][max_batch][max(qkv_dim, hidden)] product partials
    size_t qp;              // bf16 packed queries [max_batch][n_kv][D/32][64][8]
    size_t cs;              // fp32 [max_batch][D/2] cos, then [max_batch][D/2] sin
    size_t pre, lens, sched;  // int32 attention schedule: block prefix [HX_PREFIX_LEN], lengths [256], {S, Nt}
    size_t blk_new;         // int32 [256] physical block of each sequence's new position (per step)
    size_t part_ml;         // fp32 [slots][32]     running max (16) | sum (16); slots = attn_waves + max_batch*n_kv
    size_t part_o;          // fp32 [slots][G][D]   unnormalised partial outputs
    // prompt chunks (attention_chunk.hip): rows grouped by sequence, partial results of 4 column blocks per slot
    size_t chunk_cont;      // int32 [256]  row r continues row r - 1
    size_t chunk_ginfo;     // int32 [256]  group: first row | rows << 16
    size_t chunk_rgrp;      // int32 [256]  row: group | index in group << 16
    size_t chunk_part_ml;   // fp32 [slots][4][32]
    size_t chunk_part_o;    // fp32 [slots][4][16][D]
    size_t amax_val, amax_idx;  // fp32 / int32 [max_batch][lm n_tiles]   (sampling: best perturbed score and its column)
    size_t samp_z, samp_m, samp_s;  // fp32 [max_batch][lm n_tiles]: scaled logit of the candidate, tile max, tile sum of exp
    size_t scratch_f32;     // fp32 [max_batch][max(hidden, q_dim, inter, qkv_dim)] stage-hook staging
    size_t total;
};

struct hx_engine {
    hx_model_config cfg;
    int G, D, q_dim, kv_dim, qkv_dim;
    int m_groups_max;       // ceil(max_batch / 32)
    int attn_waves;         // wavefronts of the attention kernel (8 per compute unit of the device)
    bool chunk_attention;     // prompt rows of one sequence share a K/V stream (HX_CHUNK_ATTENTION=0 disables)
    int chunk_rows;           // rows per group: min(HX_CHUNK_ROWS, 64 / G)
    char *weights;          // device
    char *ws;               // device
    size_t weights_bytes, ws_bytes;
    hx_layer_map *layers;   // [n_layers], host
    size_t embed, gf;       // byte offsets
    hx_matrix wlm;
    hx_ws_map map;
    float *attn_capture;    // device or NULL
    uint32_t profile_mask;  // kernel classes bracketed by events
    int profile_stride;     // every n-th launch of a selected class is bracketed (1: every launch)
    int64_t profile_seen[HX_K_COUNT];   // launches of each class since hx_profile_enable
    std::vector<std::pair<hipEvent_t, hipEvent_t>> *profile_events;   // [HX_K_COUNT], host
};

struct hx_kv {
    hx_engine *engine;
    char *pool;             // device
    int64_t num_blocks;
    bool fp8;               // 8-bit (E4M3) elements
    size_t tile_bytes;      // 16 * head_dim * element size
    size_t block_bytes;     // n_kv_heads * 2 * tile_bytes
    size_t layer_bytes;     // num_blocks * block_bytes
};

// Device buffers of the attention stage beyond its inputs and outputs: the packed queries, the per-step schedule and
// the split-K partial results.  They live in the engine's workspace (hx_attn_bufs_of) or, for the entry point that
// must not depend on a workspace, in the library's static device array.
struct hx_attn_bufs {
    uint16_t *qp;               // packed queries
    int32_t *pre, *lens, *sched;
    float *part_ml, *part_o;
    uint16_t *ap;               // packed bf16 attention output for the output projection; NULL: not written
};
hx_attn_bufs hx_attn_bufs_of(const hx_engine *e);

// ---- kernel launchers (one per translation unit) ---------------------------------------------------

// kv_cache.hip
int hx_launch_kv_scatter(const hx_kv *kv, int layer, const void *k, const void *v, const int32_t *seq_start,
                         const int32_t *table, int max_blocks, int batch, int64_t total_tokens, bool gather,
                         hipStream_t st);
int hx_launch_rope_append(const hx_engine *e, const hx_kv *kv, int layer, int batch, const float *ypart,
                          int splits, size_t split_stride, const int32_t *positions, hipStream_t st, int blocks = 1,
                          size_t block_stride = 0);

// attention.hip
// bufs: NULL = the engine's workspace
int hx_launch_step_setup(const hx_engine *e, int batch, const int32_t *positions, const int32_t *seq_lens,
                         const int32_t *table, int max_blocks, hipStream_t st,   // table may be NULL when positions is
                         const hx_attn_bufs *bufs = nullptr);                    // (bufs: positions must be NULL)
int hx_launch_attention(const hx_engine *e, const hx_kv *kv, int layer, int batch, const int32_t *seq_lens,
                        const int32_t *table, int max_blocks, hipStream_t st, const hx_attn_bufs *bufs = nullptr);
int hx_launch_combine(const hx_engine *e, int batch, float *attn_f32_out, hipStream_t st, const hx_attn_bufs *bufs = nullptr);

// gemm.hip
int hx_launch_pack_matrix(const hx_engine *e, const hx_matrix *m, const void *src, int64_t rows, int64_t cols,
                          int col_phase /*0 plain, 1 gate, 2 up*/, hipStream_t st);
enum { HX_EPI_PARTIAL = 0, HX_EPI_SWIGLU = 1, HX_EPI_LOGITS = 2, HX_EPI_SAMPLE = 3 };

// parameters of a sampled step (NULL = greedy)
struct hx_sample_params {
    const int32_t *positions;   // device [batch]: enters the generator's counter
    const int32_t *row_ids;     // device [batch] or NULL (row id = index in the batch)
    float inv_temperature;
    uint32_t key0, key1;        // seed, low and high word
    float top_p;                // 1: no truncation; (0, 1): nucleus of that mass
    int32_t *nucleus_sizes;     // device [batch] or NULL: size of each row's kept set (top_p < 1)
};

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11), from its published definition: ten rounds of
// (c0, c1, c2, c3) <- (hi(M1 c2) ^ c1 ^ k0, lo(M1 c2), hi(M0 c0) ^ c3 ^ k1, lo(M0 c0)), key += (W0, W1) per round.
__device__ __forceinline__ void hx_philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                                 uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0; c1 = lo1; c2 = hi0 ^ c3 ^ k1; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// attention_chunk.hip
int hx_launch_chunk_setup(const hx_engine *e, int n_rows, const int32_t *seq_lens, const int32_t *table, int max_blocks,
                          hipStream_t st);
int hx_launch_chunk_attention(const hx_engine *e, const hx_kv *kv, int layer, const int32_t *table, int max_blocks,
                              hipStream_t st, int blocks = 1, size_t block_stride = 0, int rows_per_block = 0);
int hx_launch_chunk_combine(const hx_engine *e, int n_rows, float *attn_f32_out, hipStream_t st, int blocks = 1,
                            size_t block_stride = 0);

// attention_fp8.hip: the decode step's attention over an 8-bit cache
int hx_launch_attention_fp8(const hx_engine *e, const hx_kv *kv, int layer, const int32_t *table, int max_blocks,
                            hipStream_t st, const hx_attn_bufs *bufs = nullptr);

// sampling.hip
int hx_launch_nucleus(const hx_engine *e, int batch, const float *logits, const hx_sample_params *sample,
                      int32_t *tokens_out, float *logprobs_out, hipStream_t st);
int hx_launch_gemm(const hx_engine *e, const hx_matrix *m, int batch, const void *xp, int epilogue,
                   float *y /*partials or logits or NULL*/, void *mp_out, hipStream_t st,
                   const hx_sample_params *sample = nullptr);
// gemm_wide.hip: products over several 256-row blocks at once (prompt rows)
struct hx_wide_plan { int wnt, splits; };        // 32-column tiles per workgroup, K-splits
hx_wide_plan hx_plan_wide(const hx_matrix *m, int row_blocks, bool partial);
int hx_launch_gemm_wide(const hx_engine *e, const hx_matrix *m, int row_blocks, char *ws0, size_t block_stride, size_t xp_off,
                        int epilogue, size_t y_off, size_t mp_off, hx_wide_plan plan, hipStream_t st);

int hx_launch_sample_final(const hx_engine *e, int batch, int32_t *tokens_out, float *logprobs_out, hipStream_t st);
int hx_gemm_splits(const hx_matrix *m, int batch);   // K-splits the planner uses for a product with split partials
int hx_launch_argmax_final(const hx_engine *e, int batch, int32_t *tokens_out, hipStream_t st);

// elementwise.hip
// blocks > 1 (wide prompt calls): the same launch over further 256-row blocks whose workspaces follow at block_stride bytes
int hx_launch_embed_norm(const hx_engine *e, int batch, const int32_t *tokens, size_t gain_off, hipStream_t st, int blocks = 1,
                         size_t block_stride = 0);
int hx_launch_reduce_norm(const hx_engine *e, int batch, const float *ypart, int splits, size_t split_stride,
                          size_t gain_off, hipStream_t st, int blocks = 1, size_t block_stride = 0);
int hx_launch_pack_x(const hx_engine *e, int batch, const float *x, int K, void *xp, hipStream_t st);
int hx_launch_unpack_x(const hx_engine *e, int batch, const void *xp, int K, float *x, hipStream_t st);
int hx_launch_unpack_q(const hx_engine *e, int batch, float *q_out, hipStream_t st);
int hx_launch_pack_q(const hx_engine *e, int batch, const float *q, hipStream_t st, const hx_attn_bufs *bufs = nullptr);
int hx_launch_sum_partials(const hx_engine *e, int batch, const float *ypart, int splits, size_t split_stride,
                           int N, float *y, hipStream_t st);
int hx_launch_norm_only(const hx_engine *e, int batch, const float *x, size_t gain_off, float *y, hipStream_t st);
