/*
 * hexdecode.h -- C ABI of the MI355X rollout decode-step library (libhexdecode.so).
 *
 * What it computes.  The paper splits asynchronous RL into rollout generation, reward and
 * training, and characterises rollout generation as HBM-I/O-bound inference that dominates the
 * workflow (Section 1; Section 3, Observation 1; Section 4.1, the C_I > C_T assumption; Section
 * 5.3, Discussion); its policy models are distilled Qwen-2.5 decoders of 1.5B / 7B / 14B
 * parameters (Section 5.2) whose response lengths are skewed (Section 4.2.2).  The paper gives no
 * kernel-level description, so the operation is the textbook one: ONE autoregressive decode
 * step of a Qwen2-style decoder (RMSNorm, q/k/v projection with bias, rotate-half RoPE,
 * grouped-query attention over a paged KV cache, SwiGLU MLP, LM head, greedy argmax) for a
 * batch of independent sequences with ragged context lengths.
 *
 * Numeric contract.  Weights, KV cache and every matrix-product input are bf16; all arithmetic
 * accumulates in fp32; the residual stream stays fp32.  Activations are rounded to bf16
 * (nearest-even) at the five matrix-product inputs, at the rotated query and at K/V cache
 * writes, nowhere else (softmax probabilities enter the P*V product as a high + low bf16 pair).
 *
 * Conventions for every function.
 *   - extern "C"; returns hx_status: 0 on success, negative on error.  Never throws, never aborts.
 *     hx_last_error() returns a static, thread-local description of the last failure.
 *   - "DEVICE" pointers are HIP device addresses owned by the caller (e.g. torch.empty(...,
 *     device="cuda")); the library never allocates or frees device memory and keeps only the
 *     addresses.  "HOST" pointers are ordinary process memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Kernels are
 *     enqueued on it and the call returns without synchronising; results are valid once the
 *     stream reaches that point.  Scalar arguments are validated on the host before anything is
 *     enqueued; the CONTENT of device arrays (token ids, block ids, lengths) is not validated:
 *     out-of-range content is undefined behaviour.
 *   - One engine / kv handle may be used by one thread at a time; calls on the same engine must
 *     be stream-ordered (they share the workspace).
 */
#ifndef HEXDECODE_H
#define HEXDECODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hx_engine hx_engine; /* host-side handle: model shape, packed-weight map, workspace map */
typedef struct hx_kv hx_kv;         /* host-side handle: view of a caller-owned paged KV pool           */

/* Shape of the decoder and limits of the deployment.  Set struct_size = sizeof(hx_model_config). */
typedef struct {
    uint32_t struct_size;
    int32_t n_layers;
    int32_t hidden;       /* multiple of 32                                         */
    int32_t n_q_heads;    /* multiple of n_kv_heads, at most 16 query heads per KV head */
    int32_t n_kv_heads;
    int32_t head_dim;     /* 64 or 128                                              */
    int32_t intermediate; /* multiple of 16                                         */
    int32_t vocab;
    int32_t block_size;   /* tokens per KV block; must be 16                        */
    int32_t qkv_bias;     /* 1: q/k/v projections carry a bias                      */
    float rms_eps;
    float rope_theta;
    int32_t max_batch;    /* 1..256 sequences per decode step                        */
    int32_t max_seq_len;  /* largest KV length (new token included) of any sequence  */
    int32_t kv_dtype;     /* HX_KV_BF16 or HX_KV_FP8_E4M3: element type of the KV cache */
} hx_model_config;

/* Element type of the paged KV cache.  HX_KV_BF16 is the numeric contract of the decode step.  HX_KV_FP8_E4M3 is a
   variant that halves the bytes the attention kernel streams: K (after RoPE) and V are rounded from fp32 straight to
   the 8-bit format E4M3 of the OCP 8-bit floating point specification (bias 7, largest finite value 448, no
   infinities), nearest-even, magnitudes above 448 saturating, with no scale factor; attention converts them back
   exactly (every E4M3 value is a bf16 value) and proceeds as in the bf16 contract.  prefill_fill rounds the
   caller's bf16 K/V the same way and hx_kv_gather returns the stored values as bf16. */
enum { HX_KV_BF16 = 0, HX_KV_FP8_E4M3 = 1 };

typedef enum {
    HX_OK = 0,
    HX_E_NULL = -1,      /* a required pointer is NULL                               */
    HX_E_CONFIG = -2,    /* unsupported or inconsistent hx_model_config              */
    HX_E_SHAPE = -3,     /* rows/cols/batch/layer/kind do not match the configuration */
    HX_E_ALIGN = -4,     /* a device buffer is not 256-byte aligned                  */
    HX_E_TOO_SMALL = -5, /* a caller buffer is smaller than the size query says      */
    HX_E_RANGE = -6,     /* a scalar argument is out of range                        */
    HX_E_HIP = -7        /* the HIP runtime reported an error (text in hx_last_error) */
} hx_status;

/* Logical tensors of the model, all bf16 row-major [in, out] (vectors: [n]). */
typedef enum {
    HX_T_EMBED = 0, /* [vocab, hidden]  (layer ignored)            */
    HX_T_G1 = 1,    /* [hidden]  gain of the attention-block norm   */
    HX_T_WQKV = 2,  /* [hidden, (n_q_heads + 2 n_kv_heads) head_dim], columns q | k | v */
    HX_T_BQKV = 3,  /* [(n_q_heads + 2 n_kv_heads) head_dim]        */
    HX_T_WO = 4,    /* [n_q_heads head_dim, hidden]                 */
    HX_T_G2 = 5,    /* [hidden]  gain of the MLP-block norm         */
    HX_T_WG = 6,    /* [hidden, intermediate]  gate projection      */
    HX_T_WU = 7,    /* [hidden, intermediate]  up projection        */
    HX_T_WD = 8,    /* [intermediate, hidden]  down projection      */
    HX_T_GF = 9,    /* [hidden]  final gain      (layer ignored)    */
    HX_T_WLM = 10   /* [hidden, vocab]  LM head  (layer ignored)    */
} hx_tensor_kind;

const char *hx_last_error(void);

/* ---- sizes of the caller-provided device buffers (HOST out-pointers) -------------------------- */

/* Bytes of the packed-weight buffer (all tensors above in the library's streaming layout). */
int hx_weights_bytes(const hx_model_config *cfg, size_t *out);
/* Bytes of the workspace: activations, split-K partial results, work list, per-step tables. */
int hx_workspace_bytes(const hx_model_config *cfg, size_t *out);
/* Bytes of a KV pool of `num_blocks` physical blocks (all layers, K and V). */
int hx_kv_bytes(const hx_model_config *cfg, int64_t num_blocks, size_t *out);

/* ---- engine ------------------------------------------------------------------------------------ */

/* Wraps caller-owned DEVICE buffers (256-byte aligned, at least the sizes above).  No device work
   is done.  The buffers must outlive the engine.  *out receives a handle released with
   hx_engine_destroy (which frees host state only).  Several engines of one configuration may wrap the same weights
   buffer, each with a workspace of its own: their calls may then run concurrently on different streams (only
   hx_weights_pack writes the weights; order it against every engine that reads them). */
int hx_engine_create(const hx_model_config *cfg, void *weights_dev, size_t weights_bytes,
                     void *workspace_dev, size_t workspace_bytes, hx_engine **out);
int hx_engine_destroy(hx_engine *engine);

/* Re-packs ONE logical tensor (DEVICE, bf16, row-major [rows, cols], contiguous) into the engine's
   weight buffer: matrices go to the operand order of the matrix-core instructions so that a
   wavefront streams them with contiguous 1-KiB loads; vectors and the embedding are copied.
   HX_T_WG and HX_T_WU of a layer share one interleaved packed matrix; each may be packed
   independently.  `src_dev` may be released once the stream has passed the call.  This is also
   the weight-update path after a policy update (Section 2, weight synchronisation). */
int hx_weights_pack(hx_engine *engine, int tensor_kind, int layer, const void *src_dev,
                    int64_t rows, int64_t cols, void *stream);

/* ---- paged KV cache ------------------------------------------------------------------------------ */

/* The KV cache of rollout generation (the memory-bound inference stage of paper Section 1 and Section 3,
   Observation 1; response lengths are skewed, Section 4.2.2, hence paging).
   Wraps a caller-owned DEVICE pool (256-byte aligned, >= hx_kv_bytes(num_blocks)) as a paged
   cache of `num_blocks` blocks of 16 tokens.  Pool layout: [layer][block][kv_head][K tile | V tile];
   a tile holds the 16 x head_dim bf16 values of one block and KV head in matrix-core operand
   order, so one wavefront load instruction covers 1 KiB of contiguous memory.  The content is
   not initialised.  *out is released with kv_free. */
int kv_alloc(hx_engine *engine, void *kv_dev, size_t kv_bytes, int64_t num_blocks, hx_kv **out);
int kv_free(hx_kv *kv);

/* Fills the cache of sequences whose context already exists (a rollout starts from its prompt: paper Section 1,
   stage (i) of the workflow).  Scatters caller-supplied K and V of ONE layer into the pool.  k_dev / v_dev: DEVICE bf16
   [total_tokens, n_kv_heads, head_dim], the sequences concatenated in batch order;
   seq_start_dev: DEVICE int32 [batch + 1], token offset of each sequence (seq_start[batch] =
   total_tokens); token p of sequence b goes to block block_table[b][p / 16], slot p % 16.
   block_table_dev: DEVICE int32 [batch, max_blocks_per_seq]. */
int prefill_fill(hx_kv *kv, int layer, const void *k_dev, const void *v_dev,
                 const int32_t *seq_start_dev, const int32_t *block_table_dev,
                 int32_t max_blocks_per_seq, int32_t batch, int64_t total_tokens, void *stream);

/* Inverse of prefill_fill (test / checkpoint hook): gathers the cached K and V of ONE layer back
   into logical layout k_out_dev / v_out_dev [total_tokens, n_kv_heads, head_dim] bf16. */
int hx_kv_gather(hx_kv *kv, int layer, void *k_out_dev, void *v_out_dev,
                 const int32_t *seq_start_dev, const int32_t *block_table_dev,
                 int32_t max_blocks_per_seq, int32_t batch, int64_t total_tokens, void *stream);

/* ---- the decode step ------------------------------------------------------------------------------ */

/* The hot path: one step of rollout generation, which the paper characterises as HBM-I/O-bound inference
   dominating the workflow (Section 1; Section 3, Observation 1; Section 5.3, Discussion), for the decoder family of
   Section 5.2.  One autoregressive step for `batch` sequences.  All array arguments are DEVICE pointers.
     tokens      int32 [batch]   id of the token to process for each sequence
     positions   int32 [batch]   its position = number of tokens already cached
     seq_lens    int32 [batch]   keys attended = positions + 1 (the new token attends itself)
     block_table int32 [batch, max_blocks_per_seq]  physical block of each logical block; entries
                                 past ceil(seq_lens/16) are ignored
     logits_out  fp32 [batch, vocab] or NULL (then the logits are not written)
     next_tokens_out int32 [batch]   smallest index attaining the row maximum of the logits
   Side effect: K and V of the new token are written into `kv` at `positions` for every layer.
   The step is deterministic: the same inputs give the same bits.  It allocates nothing, uses no memset and does not
   synchronise the host, so a caller may capture it into a HIP graph -- after one ordinary call with the same batch
   size class, because the first launch of each kernel variant sets its attributes (the same holds for prefill_chunk,
   prefill_rows and the sampling steps). */
int decode_step(hx_engine *engine, hx_kv *kv, int32_t batch, const int32_t *tokens,
                const int32_t *positions, const int32_t *seq_lens, const int32_t *block_table,
                int32_t max_blocks_per_seq, float *logits_out, int32_t *next_tokens_out, void *stream);

/* The same step ending in a temperature sample instead of the arg-max, with the log-probability of the drawn
   token under the sampling distribution.  Rollout generation draws several responses per prompt (paper
   Section 1, stage (i) of the workflow) and the policy update of the GRPO workloads (Section 5) needs the
   behaviour policy's log-probabilities.  Arguments as decode_step, plus:
     temperature  > 0, finite.  z_i = logit_i * (1 / temperature), the reciprocal taken once in fp32.
     seed         key of the counter-based generator Philox4x32-10 (Salmon et al., SC'11): low, high word.
     row_ids      int32 [batch] DEVICE or NULL: id of each sequence in the generator's counter (NULL: its
                  index in the batch).  Vocabulary entry i of a row uses word i % 4 of the block with counter
                  (i / 4, row id, positions[row], 0x53414D50); u = ((word >> 9) + 0.5) * 2^-23.
     tokens_out   int32 [batch]  argmax_i (z_i - log(-log(u_i))), smallest index on ties (Gumbel-max: the
                  token is distributed as softmax(z)); all fp32.
     logprobs_out fp32 [batch]   z_token - log(sum_i exp(z_i)).
   The draw is a pure function of (logits, temperature, seed, row id, position): repeatable bit for bit.
   Errors: HX_E_RANGE for a temperature that is not positive and finite, HX_E_NULL for NULL outputs. */
int decode_step_sample(hx_engine *engine, hx_kv *kv, int32_t batch, const int32_t *tokens,
                       const int32_t *positions, const int32_t *seq_lens, const int32_t *block_table,
                       int32_t max_blocks_per_seq, float temperature, uint64_t seed, const int32_t *row_ids,
                       float *logits_out, int32_t *tokens_out, float *logprobs_out, void *stream);

/* The sampled step with nucleus (top-p) truncation (Holtzman et al., ICLR 2020) -- the paper does not say how
   rollouts are drawn; this is the usual companion of the temperature.  With p = softmax(z), z as in
   decode_step_sample, the kept set is {i : z_i >= tau}, tau the largest value for which the kept mass is at least
   top_p (entries equal to the last kept one are all kept); the token is the Gumbel-max of decode_step_sample
   restricted to the kept set, with the same noise per entry, so it is distributed as p renormalised over the set.
   Arguments as decode_step_sample, plus:
     top_p        in (0, 1].  1 is exactly decode_step_sample (no truncation).
     logits_out   fp32 [batch, vocab]; REQUIRED when top_p < 1 (the selection re-reads the stored logits).
     logprobs_out fp32 [batch]   log of the renormalised probability: z_token - log(sum over the kept set of exp(z_i)).
     nucleus_sizes_out int32 [batch] or NULL: number of kept entries per row (top_p < 1 only).
   Mass is accumulated in 40-bit fixed point, w_i = floor(exp(z_i - max z) * 2^40), with integer additions: the
   kept set is exact in that arithmetic and the step stays deterministic.  A row whose running mass comes within
   ~1e-7 of top_p at the cut may keep one entry more or less than a double-precision evaluation would.
   Errors: HX_E_RANGE for temperature or top_p out of range, HX_E_NULL for missing outputs. */
int decode_step_top_p(hx_engine *engine, hx_kv *kv, int32_t batch, const int32_t *tokens,
                      const int32_t *positions, const int32_t *seq_lens, const int32_t *block_table,
                      int32_t max_blocks_per_seq, float temperature, float top_p, uint64_t seed,
                      const int32_t *row_ids, float *logits_out, int32_t *tokens_out, float *logprobs_out,
                      int32_t *nucleus_sizes_out, void *stream);

/* Prompt processing in chunks: the step for n_rows (<= max_batch) PROMPT TOKENS at once, without LM head -- only the
   K and V of every row enter the cache (rollouts start from a prompt: paper Section 1, stage (i); Section 4.2.2).
   A row is one token of one sequence: tokens[r] at positions[r], attending seq_lens[r] = positions[r] + 1 keys
   through block_table row r -- rows of the same sequence carry copies of that sequence's table row.  Rows of one
   sequence in one call must cover consecutive positions that continue its cache (K and V of all rows are written
   before any row attends, so a row sees the rows before it); chunks of a sequence are submitted in position order.
   The last prompt token is then given to decode_step / decode_step_sample, which yields the first generated token.
   Consecutive rows that continue one another (seq_lens one more, the same table row) are attended in groups of up
   to 8 that share one read of the cache (8 rows with at most 8 query heads per KV head, down to 4 rows with 16), so
   a call should hold long runs of one sequence rather than one row of many; any row order is correct.  Arguments,
   ownership and errors as decode_step. */
int prefill_chunk(hx_engine *engine, hx_kv *kv, int32_t n_rows, const int32_t *tokens, const int32_t *positions,
                  const int32_t *seq_lens, const int32_t *block_table, int32_t max_blocks_per_seq, void *stream);

/* Prompt processing for many rows per call: prefill_chunk for n_rows = a multiple of 256, at most HX_PREFILL_MAX_ROWS,
   with every matrix product taken over ALL rows at once (both operands tiled through LDS), so that the weights are
   read from memory once per call instead of once per 256 rows (paper Section 1, stage (i); Section 4.2.2: a rollout
   starts from its prompt).  Rows, tables and results exactly as prefill_chunk (rows r of block r / 256; K and V of all
   rows of the call enter the cache before any row attends); the attention output capture, if set, is
   [n_layers, n_rows, n_q_heads * head_dim].  The engine must have been created with max_batch = 256 and its hidden,
   intermediate and n_q_heads * head_dim sizes must be multiples of 32.  workspace_dev: DEVICE memory, 256-byte aligned,
   of at least hx_prefill_workspace_bytes(cfg, n_rows) bytes, owned by the caller, overwritten by the call (the
   engine's own workspace is not used; two calls on different streams need different workspaces).  Nothing is allocated
   and the host is not synchronised.  Errors: HX_E_RANGE for n_rows, alignment or a short workspace, HX_E_SHAPE for the
   size conditions, HX_E_NULL.  The remainder of a prompt (fewer than 256 rows) goes through prefill_chunk. */
#define HX_PREFILL_MAX_ROWS 8192
int hx_prefill_workspace_bytes(const hx_model_config *cfg, int32_t max_rows, size_t *bytes_out);
int prefill_rows(hx_engine *engine, hx_kv *kv, int32_t n_rows, const int32_t *tokens, const int32_t *positions,
                 const int32_t *seq_lens, const int32_t *block_table, int32_t max_blocks_per_seq, void *workspace_dev,
                 size_t workspace_bytes, void *stream);

/* Checks the DEVICE-side inputs of a step before it is launched; decode_step itself trusts them (a wrong block id
   or length makes its kernels read or write outside the pool).  Verified per row: 0 <= token < vocab;
   0 <= position < max_seq_len and position < 16 * max_blocks_per_seq; seq_len == position + 1; every block id
   of the first ceil(seq_len / 16) table entries in [0, num_blocks of kv).  Only the argument arrays are read.
   SYNCHRONISES `stream`.  Returns HX_OK, or HX_E_RANGE with the first offending row in hx_last_error(). */
int hx_validate_step_inputs(hx_engine *engine, hx_kv *kv, int32_t batch, const int32_t *tokens,
                            const int32_t *positions, const int32_t *seq_lens, const int32_t *block_table,
                            int32_t max_blocks_per_seq, void *stream);

/* Parity hook: when attn_dev is not NULL every following decode_step also writes the attention
   output of every layer BEFORE its bf16 rounding to attn_dev, DEVICE fp32
   [n_layers, batch, n_q_heads * head_dim] (batch = that step's batch).  NULL switches it off. */
int hx_set_attn_capture(hx_engine *engine, float *attn_dev);

/* ---- single stages (test and measurement hooks; the same kernels decode_step launches) ------------ */

/* Schedule of the split-K attention.  A tile is the K and V of 16 tokens of one KV head; the tiles of the batch,
   in (sequence, KV head, block) order, are cut into hx_attention_waves(engine) equal runs, one per wavefront.
   Outputs are DEVICE int32: prefix_out [batch + 1] = exclusive prefix sum of ceil(seq_lens[b] / 16);
   sched_out [2] = { tiles per run = ceil(total / waves), total tiles = prefix_out[batch] * n_kv_heads }. */
int hx_stage_schedule(hx_engine *engine, int32_t batch, const int32_t *seq_lens, int32_t *prefix_out,
                      int32_t *sched_out, void *stream);
int hx_attention_waves(const hx_engine *engine); /* wavefronts of the attention kernel */

/* Tuning knobs read from the environment (none is needed for correct or fast operation; results stay within the
   same tolerances, only summation order changes):
     HX_ATTN_WAVES=n        wavefronts of the attention kernel, read at hx_engine_create (default 8 per compute unit
                            of the device: 2048 on an MI355X)
     HX_GEMM_SHAPE=wn,wk,s  force tiles per workgroup (4..6, or 4 with wk = 2), k-slices per workgroup and K-splits
     HX_GEMM_MAX_SPLITS=s   upper bound of the planner's K-splits (1..9)
     HX_CHUNK_ATTENTION=0   prefill_chunk attends every row on its own (the decode step's kernel) instead of in groups
                            of consecutive rows, read at hx_engine_create; for comparison                            */

/* How a matrix product of n_tiles 32-column tiles and k_steps 16-row steps is launched for `batch` rows (host logic
   only, no GPU work): tiles per workgroup, k-slices per workgroup, and K-splits whose fp32 partial results the consumer
   kernel adds (only if `partial` != 0; products with a fused epilogue are never split).  HX_E_RANGE for sizes < 1 or
   batch > 256, HX_E_NULL for NULL outputs. */
int hx_plan_product(int32_t n_tiles, int32_t k_steps, int32_t batch, int32_t partial, int32_t *tiles_per_workgroup_out,
                    int32_t *k_slices_out, int32_t *splits_out);

/* bias + RoPE + cache append of one layer: qkv_dev fp32 [batch, qkv_cols] is the projection WITHOUT
   bias (the packed bias of `layer` is added); writes K/V of position positions[b] into `kv` and
   returns the rotated, bf16-rounded query as fp32 in q_out_dev [batch, n_q_heads * head_dim]. */
int hx_stage_rope_append(hx_engine *engine, hx_kv *kv, int layer, int32_t batch, const float *qkv_dev,
                         const int32_t *positions, const int32_t *block_table,
                         int32_t max_blocks_per_seq, float *q_out_dev, void *stream);

/* Attention of one layer over the cache as it stands: q_dev fp32 [batch, n_q_heads * head_dim]
   (rounded to bf16 on entry), out_dev fp32 [batch, n_q_heads * head_dim] before rounding. */
int hx_stage_attention(hx_engine *engine, hx_kv *kv, int layer, int32_t batch, const float *q_dev,
                       const int32_t *seq_lens, const int32_t *block_table,
                       int32_t max_blocks_per_seq, float *out_dev, void *stream);

/* hx_stage_attention for callers that cannot allocate or provide scratch memory: code under graph capture, tight
   serving loops, harnesses that forbid allocation.  Same arguments, same kernels, same results bit for bit, but the
   stage's scratch (packed queries, schedule, split-K partial results) lives in a device array inside the library,
   HX_STATIC_SCRATCH_BYTES per GPU for the life of the process, instead of the engine's workspace, which this call
   never touches; it calls no allocating routine.  The scratch of a call is
       batch * n_kv_heads * head_dim * 32                                              packed queries
     + (wavefronts + batch * n_kv_heads) * (128 + 4 * G * head_dim)                    partial results (G = query heads
     + about 6 KiB of schedule and padding                                              per KV head)
   bytes (9 to 12 MiB for the five benchmark workloads with the default 2048 wavefronts); a call that needs more than
   the array holds fails with HX_E_RANGE and a message giving both numbers.  Every call on a GPU shares that GPU's
   array and finds the previous call's contents in it (nothing needs clearing: each call writes what it reads).
   Calls that overlap on one GPU -- two streams, two threads -- race: the caller must serialise them. */
#define HX_STATIC_SCRATCH_BYTES (16 << 20)
int hx_stage_attention_static(hx_engine *engine, hx_kv *kv, int layer, int32_t batch, const float *q_dev,
                              const int32_t *seq_lens, const int32_t *block_table,
                              int32_t max_blocks_per_seq, float *out_dev, void *stream);

/* RMSNorm with the packed gain `gain_kind` (HX_T_G1 / HX_T_G2 / HX_T_GF): x_dev fp32
   [batch, hidden] -> y_dev fp32 [batch, hidden] holding the bf16-rounded result. */
int hx_stage_rmsnorm(hx_engine *engine, int gain_kind, int layer, int32_t batch, const float *x_dev,
                     float *y_dev, void *stream);

/* One weight-streaming matrix product with the packed tensor `matrix_kind`:
     HX_T_WQKV: y [batch, qkv_cols] = R(x) W (no bias)      HX_T_WO: y [batch, hidden] = R(x) W
     HX_T_WG  : y [batch, intermediate] = R( silu(R(x) Wg) * (R(x) Wu) ) as fp32
     HX_T_WD  : y [batch, hidden] = R(x) W                   HX_T_WLM: y [batch, vocab] = R(x) W
   x_dev fp32 [batch, in] is rounded to bf16 (R) on entry.  For HX_T_WLM, argmax_out_dev (int32
   [batch], may be NULL) receives the greedy token; it must be NULL for the other kinds. */
int hx_stage_linear(hx_engine *engine, int matrix_kind, int layer, int32_t batch, const float *x_dev,
                    float *y_dev, int32_t *argmax_out_dev, void *stream);

/* The same products as prefill_rows runs them (workgroup-tiled, all rows of the call at once): matrix_kind HX_T_WQKV,
   HX_T_WO, HX_T_WG or HX_T_WD as above, n_rows a multiple of 256 up to HX_PREFILL_MAX_ROWS, x_dev fp32 [n_rows, in],
   y_dev fp32 [n_rows, out]; engine, workspace_dev and errors as prefill_rows. */
int hx_stage_linear_rows(hx_engine *engine, int matrix_kind, int layer, int32_t n_rows, const float *x_dev,
                         float *y_dev, void *workspace_dev, size_t workspace_bytes, void *stream);

/* The LM head on caller-supplied activations followed by the nucleus draw of decode_step_top_p (same kernels, same
   argument meaning; top_p in (0, 1), all outputs but nucleus_sizes_out required): x_dev fp32 [batch, hidden] is
   rounded to bf16 on entry, logits_out fp32 [batch, vocab] receives R(x) W. */
int hx_stage_lm_head_top_p(hx_engine *engine, int32_t batch, const float *x_dev, const int32_t *positions,
                           const int32_t *row_ids, float temperature, float top_p, uint64_t seed,
                           float *logits_out, int32_t *tokens_out, float *logprobs_out,
                           int32_t *nucleus_sizes_out, void *stream);

/* ---- per-kernel timing (measurement hook) -------------------------------------------------------------- */

/* Kernel classes of the decode step. */
typedef enum {
    HX_K_ATTENTION = 0, /* split-K attention kernel                      */
    HX_K_COMBINE = 1,   /* split-K combine                               */
    HX_K_GEMM_QKV = 2,
    HX_K_GEMM_O = 3,
    HX_K_GEMM_GATE_UP = 4,
    HX_K_GEMM_DOWN = 5,
    HX_K_GEMM_LM = 6,
    HX_K_NORM = 7,      /* embedding / split-sum + residual + RMSNorm    */
    HX_K_ROPE = 8,      /* bias + RoPE + cache append                    */
    HX_K_SETUP = 9,     /* work list, RoPE angles, final argmax          */
    HX_K_COUNT = 10
} hx_kernel_class;

/* While bit k of `class_mask` is set, every launch of kernel class k made by decode_step is bracketed
   by two HIP events recorded on the step's stream (host objects; no device memory is allocated).
   0 switches timing off.  Bracketing adds a few microseconds per launch, so a throughput measurement
   should time at most the one class it reports. */
int hx_profile_enable(hx_engine *engine, uint32_t class_mask);
/* Brackets only every n-th launch of a selected class (counted from the last hx_profile_enable; default 1 = every
   launch): a pair of events costs the stream about 5 us, which 28 bracketed launches per step would add to a
   throughput measurement.  HX_E_RANGE for n < 1. */
int hx_profile_sample_every(hx_engine *engine, int32_t n);
/* Waits for the recorded events, adds up the elapsed time of class `kernel_class` since the last read,
   releases those events.  HOST out-pointers. */
int hx_profile_read(hx_engine *engine, int kernel_class, double *total_ms_out, int64_t *launches_out);

#ifdef __cplusplus
}
#endif
#endif /* HEXDECODE_H */
