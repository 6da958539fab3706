// Small-M weight-streaming matrix products  Y[M, N] = X[M, K] W[K, N]  (M = batch <= 256).
//
// The weights dominate the bytes, so the kernel is organised around streaming each packed weight
// tile exactly once, straight from HBM into the A operand of v_mfma_f32_32x32x16_bf16 (32 output
// columns n x 16 k per 1-KiB load).  The activations are the B operand (16 k x 32 batch rows per
// m-group); they are small, L2-resident, and shared by the consumer wavefronts of a workgroup through
// a multi-stage LDS copy made by dedicated producer wavefronts.  Each wavefront owns one 32-column n-tile and all batch rows, so the
// accumulator is MG tiles of 32 x 32 fp32.  Along K the product may be split over workgroups; the
// fp32 partial results are summed in split order by the consumer kernel (deterministic).
//
// Epilogues: plain fp32 partials; SiLU(gate) * up -> bf16 packed activations of the down
// projection; logits + per-tile argmax candidates; logits + per-tile sampling candidates and log-sum-exp pieces.
#include "hx_internal.h"
#include <algorithm>
#include <mutex>

// ---- weight packing ------------------------------------------------------------------------------------------
// grid (n_tiles, ceil(k_steps / 4)), 256 threads: one wavefront per (n_tile, k_step).
// col_phase 0: tile column c -> source column 32*nt + c.  col_phase 1 / 2 (gate / up): only lanes
// c < 16 / c >= 16 are written, from source column 16*nt + c%16.
__global__ __launch_bounds__(256) void pack_matrix_kernel(const uint16_t *__restrict__ src, int64_t rows, int64_t cols,
                                                          uint4 *__restrict__ dst, int k_steps, int col_phase) {
    const int nt = blockIdx.x;
    const int ks = blockIdx.y * 4 + (threadIdx.x >> 6);
    if (ks >= k_steps) return;
    const int lane = threadIdx.x & 63;
    const int c = lane & 31, kh = lane >> 5;
    int64_t col;
    if (col_phase == 0) col = (int64_t)32 * nt + c;
    else {
        if ((col_phase == 1) != (c < 16)) return;
        col = (int64_t)16 * nt + (c & 15);
    }
    uint16_t v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        int64_t k = (int64_t)16 * ks + 8 * kh + j;
        v[j] = (col < cols && k < rows) ? src[k * cols + col] : (uint16_t)0;
    }
    uint4 o;
    o.x = v[0] | ((uint32_t)v[1] << 16); o.y = v[2] | ((uint32_t)v[3] << 16);
    o.z = v[4] | ((uint32_t)v[5] << 16); o.w = v[6] | ((uint32_t)v[7] << 16);
    dst[((size_t)nt * k_steps + ks) * 64 + lane] = o;
}

int hx_launch_pack_matrix(const hx_engine *e, const hx_matrix *m, const void *src, int64_t rows, int64_t cols,
                          int col_phase, hipStream_t st) {
    dim3 grid(m->n_tiles, (m->k_steps + 3) / 4), block(256);
    hipLaunchKernelGGL(pack_matrix_kernel, grid, block, 0, st, (const uint16_t *)src, rows, cols,
                       (uint4 *)(e->weights + m->offset), m->k_steps, col_phase);
    HX_CHECK_LAUNCH("pack_matrix");
    return HX_OK;
}

// ---- the streaming product ------------------------------------------------------------------------------------
// Workgroup = WN x WK consumer wavefronts + NP producer wavefronts, one workgroup per compute unit.
// Consumers: WN adjacent n-tiles, each split into WK k-slices that are summed in slice order through LDS at
// the end.  Every consumer keeps RING weight loads (1 KiB each, non-temporal) in flight in a register ring
// and issues no other vector-memory load, so the in-order load counter never makes it wait for anything but
// the tile it is about to use.  Producers stage the activations of the coming chunks (KC k-steps of every
// k-slice, 32 KiB per stage, four stages; two stages of 64 KiB for 8 m-groups) in LDS: through their own
// registers where two chunks fit them, else with the direct L2 -> LDS load; one workgroup barrier per chunk
// hands a stage over.
#ifndef HX_GEMM_RING
#define HX_GEMM_RING 16
#endif

struct GemmArgs {
    const uint4 *wp;      // packed weights
    const uint4 *xp;      // packed activations
    int k_steps, n_tiles, tile0, tile_end, steps_per_split, steps_per_wave;   // n_tiles: whole matrix; [tile0, tile_end): this launch
    int M, N;
    float *y;             // PARTIAL: [splits][M][N]; LOGITS: [M][N] or NULL
    size_t split_stride;  // elements between splits of y
    uint16_t *mp;         // SWIGLU: packed bf16 output
    float *amax_val;      // LOGITS: [M][n_tiles]; SAMPLE: best perturbed score of the tile
    int32_t *amax_idx;
    // SAMPLE only
    const int32_t *positions, *row_ids;
    float inv_t;
    uint32_t key0, key1;
    float *samp_z, *samp_m, *samp_s;   // [M][n_tiles]
};

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4_t hx_stream_load(const uint4 *p) {   // read-once data: non-temporal
    return __builtin_nontemporal_load((const u32x4_t *)p);
}

// s_waitcnt immediate: wait until at most n vector-memory operations are outstanding, nothing else
#define HX_VMCNT(n) (((n) & 15) | (((n) >> 4) << 14) | 0x0F70)

template <int MG, int WK> struct GemmGeom {
    // stages: 4 x 32 KiB; with 8 m-groups 2 x 64 KiB, so that a stage still holds 8 k-steps (one barrier per 8)
    static constexpr int NBUF = MG >= 8 ? 2 : 4;
    static constexpr int STAGE_KB = MG >= 8 ? 64 : 32;
    static constexpr int KC0 = STAGE_KB / (WK * MG);
    static constexpr int KC = KC0 > 8 ? 8 : (KC0 < 1 ? 1 : KC0);   // k-steps per LDS chunk
    static constexpr int SLICE_U4 = KC * MG * 64;                   // uint4 per k-slice per stage
    static constexpr int PVT = WK * KC * MG;                        // 1-KiB copies per stage
    static constexpr int NP = PVT > 16 ? 2 : 1;                     // producer wavefronts
    static constexpr int PVP = PVT / NP;                            // copies per producer per stage
    static constexpr int STAGE_BYTES = WK * SLICE_U4 * 16;
};
template <int MG, int WN, int WK> constexpr int gemm_lds_bytes() {
    constexpr int stages = GemmGeom<MG, WK>::NBUF * GemmGeom<MG, WK>::STAGE_BYTES;
    constexpr int red = (WK - 1) * WN * MG * 4096;
    return stages > red ? stages : red;
}

template <int MG, int WN, int WK, int EPI>
__global__ __launch_bounds__(64 * (WN * WK + GemmGeom<MG, WK>::NP)) void gemm_stream_kernel(
    const uint4 *__restrict__ a_wp, const uint4 *__restrict__ a_xp, int a_k_steps, int a_n_tiles, int a_tile0,
    int a_tile_end, int a_steps_per_split, int a_steps_per_wave, int a_M, int a_N, float *__restrict__ a_y, size_t a_split_stride,
    uint16_t *__restrict__ a_mp, float *__restrict__ a_amax_val, int32_t *__restrict__ a_amax_idx,
    const int32_t *__restrict__ a_positions, const int32_t *__restrict__ a_row_ids, float a_inv_t, uint32_t a_key0,
    uint32_t a_key1, float *__restrict__ a_samp_z, float *__restrict__ a_samp_m, float *__restrict__ a_samp_s) {
    using GG = GemmGeom<MG, WK>;
    // 8 m-groups: a step takes twice as long (matrix-core time), so half the ring covers the same latency and the
    // revolution that fills it is half as long
    constexpr int RING = MG >= 8 ? HX_GEMM_RING / 2 : HX_GEMM_RING;
    constexpr int NBUF = GG::NBUF, LOOK = NBUF - 1;
    constexpr int KC = GG::KC, CPR = RING / KC, SLICE_U4 = GG::SLICE_U4, NC = WN * WK;
    // with at most 8 wavefronts per workgroup each may use 256 registers: enough to read B operands ahead
    constexpr bool PREFETCH_B = (NC + GG::NP <= 8) && MG <= 4;
    // activations staged through producer registers (two sets of PVP x 16 bytes per lane) where those fit
    constexpr bool COPY_VIA_REGISTERS = GG::PVP <= 16;
    static_assert(RING % KC == 0, "ring must hold whole chunks");
    static_assert(LOOK * GG::PVP <= 63, "the stages in flight must fit the load counter");
    extern __shared__ u32x4_t xs[];                      // [NBUF][WK][SLICE_U4]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);       // wave-uniform, kept in a scalar register
    const bool producer = wave >= NC;                    // the last wavefronts only stage activations
    const int wn = producer ? 0 : wave % WN, wk = producer ? 0 : wave / WN;
    const int nt = a_tile0 + blockIdx.x * WN + wn;
    const bool active = !producer && nt < a_tile_end;
    const int split0 = blockIdx.y * a_steps_per_split;
    const int split1 = min(a_k_steps, split0 + a_steps_per_split);
    // every wavefront of the grid runs the same number of chunks: whole ring revolutions.  Steps past the end
    // of a k-slice re-read the slice's last (cached) weight tile and skip the multiply, so the load stream
    // carries no condition and the compiler keeps exactly RING - 1 loads outstanding.
    const int n_chunks = (a_steps_per_wave + RING - 1) / RING * CPR;

    if (producer) {
        // k-slice w of this workgroup covers k-steps [split0 + w*spw, min(split1, +spw)); chunk c of it is a
        // contiguous run of the packed activations.
        // The consumers spend their first ring revolution (CPR virtual chunks) only requesting weight tiles; real chunk
        // c is their virtual chunk c + CPR and lives in stage (c + CPR) % NBUF.
        const u32x4_t *xp4 = (const u32x4_t *)a_xp;
        const int last_u4 = a_k_steps * MG * 64 - 1;
        const int pid = wave - NC;
        auto copy_chunk = [&](int v) {                       // direct L2 -> LDS copy of virtual chunk v
            const int buf = v % NBUF;
            const int c = max(v - CPR, 0);
#pragma unroll
            for (int f = 0; f < GG::PVP; ++f) {
                const int ff = pid * GG::PVP + f;        // copy index in the stage: (k-slice, 1-KiB piece)
                const int w = ff / (KC * MG), i = ff % (KC * MG);
                const int kb = min(split1, split0 + w * a_steps_per_wave);
                const int src = min((kb + c * KC) * MG * 64 + i * 64 + lane, last_u4);
                __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)(xp4 + src),
                                                 (void __attribute__((address_space(3))) *)&xs[(buf * WK + w) * SLICE_U4 + i * 64],
                                                 16, 0, 0);
            }
        };
        const int n_virtual = n_chunks + CPR;
        if constexpr (COPY_VIA_REGISTERS) {
        // The copy goes through registers (global load, then LDS store): measured faster than the direct L2 -> LDS
        // path, which slows the weight stream of the same compute unit down when both run (timing lab: weights alone
        // 27 us, direct copy alone 18 us, both 49 us for 60 workgroups).
        static_assert(!COPY_VIA_REGISTERS || (RING / KC) % 2 == 0, "register sets alternate in pairs of chunks");
        u32x4_t ra[GG::PVP], rb[GG::PVP];
        auto load_chunk = [&](int c, u32x4_t (&r)[GG::PVP]) {
#pragma unroll
            for (int f = 0; f < GG::PVP; ++f) {
                const int ff = pid * GG::PVP + f;
                const int w = ff / (KC * MG), i = ff % (KC * MG);
                const int kb = min(split1, split0 + w * a_steps_per_wave);
                r[f] = xp4[min((kb + c * KC) * MG * 64 + i * 64 + lane, last_u4)];
            }
        };
        auto store_chunk = [&](int c, const u32x4_t (&r)[GG::PVP]) {
            const int buf = (c + CPR) % NBUF;
#pragma unroll
            for (int f = 0; f < GG::PVP; ++f) {
                const int ff = pid * GG::PVP + f;
                const int w = ff / (KC * MG), i = ff % (KC * MG);
                xs[(buf * WK + w) * SLICE_U4 + i * 64 + lane] = r[f];
            }
        };
        // Barrier v ends the consumers' virtual chunk v (one per KC k-steps, CPR of them before the first real chunk:
        // the revolution that fills their weight ring, which needs no activations).  The barriers of that revolution
        // but the last are passed at once, so the consumers have requested their whole ring before they first wait
        // for this wavefront; chunks 0 and 1 are handed over at the last of them, chunk c >= 2 at barrier c + CPR - 2,
        // one chunk ahead of its use.  Chunk c + 2 is requested as soon as chunk c has left its registers; the two
        // register sets alternate statically (n_chunks is even).
        load_chunk(0, ra);
        load_chunk(1, rb);
#pragma unroll
        for (int i = 0; i < CPR - 1; ++i) __syncthreads();
        store_chunk(0, ra);
        if (2 < n_chunks) load_chunk(2, ra);
        for (int c = 1; c < n_chunks - 1; c += 2) {
            store_chunk(c, rb);
            if (c + 2 < n_chunks) load_chunk(c + 2, rb);
            __syncthreads();
            store_chunk(c + 1, ra);
            if (c + 3 < n_chunks) load_chunk(c + 3, ra);
            __syncthreads();
        }
        store_chunk(n_chunks - 1, rb);
        __syncthreads();
        __syncthreads();
        __syncthreads();
        } else {
#pragma unroll
        for (int q = 0; q < LOOK; ++q) copy_chunk(q);
        for (int v = 0; v < n_virtual; ++v) {                    // barrier v ends the consumers' virtual chunk v
            if (v + LOOK < n_virtual) {
                copy_chunk(v + LOOK);                            // into the stage the consumers left at the last barrier
                __builtin_amdgcn_s_waitcnt(HX_VMCNT((LOOK - 1) * GG::PVP)); // stage v + 1 has landed
            } else {
                __builtin_amdgcn_s_waitcnt(HX_VMCNT(0));      // nothing is in flight once the loop ends
            }
            __syncthreads();
        }
        }
        if (WK > 1) __syncthreads();
        return;
    }

    const int kb0 = split0 + wk * a_steps_per_wave;                  // this wavefront's k-slice [kb0, ke)
    const int ke = min(split1, kb0 + a_steps_per_wave);
    const int n_valid = active ? max(0, ke - kb0) : 0;               // steps that are multiplied
    const int kb = min(kb0, a_k_steps - 1);
    const int last = max(0, min(a_k_steps, kb + a_steps_per_wave) - kb - 1);   // last step whose tile may be read
    const uint4 *wrow = a_wp + ((size_t)(active ? nt : a_tile0) * a_k_steps + kb) * 64 + lane;

    f32x16_t acc[MG];
#pragma unroll
    for (int g = 0; g < MG; ++g)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[g][r] = 0.f;

    // The loop starts one revolution early (c0 = -CPR): that revolution multiplies nothing, it only requests the
    // first RING tiles (at once: it does not wait for the activations); from then on step s multiplies the tile
    // requested RING steps earlier and then requests the tile of step s + RING into the same slot.
    // There is no separate prologue, so the only loads outstanding at any wait are the ring's own, in order.
    u32x4_t ring[RING];
#pragma unroll
    for (int r = 0; r < RING; ++r) ring[r] = u32x4_t{0u, 0u, 0u, 0u};

    int c_first = -CPR;
    asm volatile("" : "+s"(c_first));                   // opaque: the ring-filling revolution must not be peeled off the loop
    for (int c0 = c_first; c0 < n_chunks; c0 += CPR) {
#pragma unroll
        for (int cc = 0; cc < CPR; ++cc) {
            const int c = c0 + cc;
            const u32x4_t *xb = &xs[(((c + CPR) % NBUF) * WK + wk) * SLICE_U4 + lane];
            if (PREFETCH_B) {
                // B operands are read from LDS one k-step ahead of the multiplies that use them
                u32x4_t bcur[MG], bnxt[MG];
#pragma unroll
                for (int g = 0; g < MG; ++g) bcur[g] = xb[g * 64];
#pragma unroll
                for (int j = 0; j < KC; ++j) {
                    const int s = c * KC + j;
                    if (j + 1 < KC) {
#pragma unroll
                        for (int g = 0; g < MG; ++g) bnxt[g] = xb[((j + 1) * MG + g) * 64];
                    }
                    if (s >= 0 && s < n_valid) {
                        const bf16x8_t aop = __builtin_bit_cast(bf16x8_t, ring[cc * KC + j]);
#pragma unroll
                        for (int g = 0; g < MG; ++g)
                            acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop, __builtin_bit_cast(bf16x8_t, bcur[g]), acc[g], 0, 0, 0);
                    }
                    // the slot is dead now: request the tile of step s + RING into the same registers
                    ring[cc * KC + j] = hx_stream_load(wrow + (size_t)min(s + RING, last) * 64);
                    if (j + 1 < KC) {
#pragma unroll
                        for (int g = 0; g < MG; ++g) bcur[g] = bnxt[g];
                    }
                }
            } else {
                // too many accumulators to hold two steps of B operands: read them DEPTH operands ahead of the
                // multiply that uses them, in the order (k-step, m-group) in which the stage stores them
                constexpr int DEPTH = 3, ITEMS = KC * MG;
                u32x4_t bq[DEPTH];
#pragma unroll
                for (int t = 0; t < DEPTH; ++t) bq[t] = xb[t * 64];
#pragma unroll
                for (int j = 0; j < KC; ++j) {
                    const int s = c * KC + j;
                    const bf16x8_t aop = __builtin_bit_cast(bf16x8_t, ring[cc * KC + j]);
#pragma unroll
                    for (int g = 0; g < MG; ++g) {
                        const int t = j * MG + g;
                        const u32x4_t bcur = bq[t % DEPTH];
                        if (t + DEPTH < ITEMS) bq[t % DEPTH] = xb[(t + DEPTH) * 64];
                        if (s >= 0 && s < n_valid)
                            acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop, __builtin_bit_cast(bf16x8_t, bcur), acc[g], 0, 0, 0);
                    }
                    ring[cc * KC + j] = hx_stream_load(wrow + (size_t)min(s + RING, last) * 64);
                }
            }
            __syncthreads();
        }
    }

    // sum the k-slices of each n-tile in slice order (the activation stages are free now)
    if (WK > 1) {
        float *red = (float *)xs;
        if (wk > 0 && active) {
            float *dst = red + ((size_t)((wk - 1) * WN + wn) * MG * 16) * 64 + lane;
#pragma unroll
            for (int g = 0; g < MG; ++g)
#pragma unroll
                for (int r = 0; r < 16; ++r) dst[(g * 16 + r) * 64] = acc[g][r];
        }
        __syncthreads();
        if (wk == 0 && active) {
#pragma unroll
            for (int w2 = 1; w2 < WK; ++w2) {
                const float *src = red + ((size_t)((w2 - 1) * WN + wn) * MG * 16) * 64 + lane;
#pragma unroll
                for (int g = 0; g < MG; ++g)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[g][r] += src[(g * 16 + r) * 64];
            }
        }
    }
    if (!active || wk != 0) return;

    // accumulator register r of lane l: column m = 32*g + l%32, row n = 32*nt + 8*(r/4) + 4*(l/32) + r%4
    const int hl = lane >> 5, ml = lane & 31;
    if (EPI == HX_EPI_PARTIAL) {
        float *y = a_y + blockIdx.y * a_split_stride;
#pragma unroll
        for (int g = 0; g < MG; ++g) {
            const int m = 32 * g + ml;
            if (m < a_M) {
#pragma unroll
                for (int j4 = 0; j4 < 4; ++j4) {
                    const int n = 32 * nt + 8 * j4 + 4 * hl;
                    if (n < a_N)
                        *(f32x4_t *)(y + (size_t)m * a_N + n) =
                            f32x4_t{acc[g][4 * j4], acc[g][4 * j4 + 1], acc[g][4 * j4 + 2], acc[g][4 * j4 + 3]};
                }
            }
        }
    } else if (EPI == HX_EPI_SWIGLU) {
        // rows 0..15 of the tile are gate columns 16*nt + p, rows 16..31 the matching up columns
#pragma unroll
        for (int g = 0; g < MG; ++g) {
            const int m = 32 * g + ml;
            if (m < a_M) {
#pragma unroll
                for (int j4 = 0; j4 < 2; ++j4) {
                    float v[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float gt = acc[g][4 * j4 + i], up = acc[g][8 + 4 * j4 + i];
                        v[i] = (gt / (1.0f + expf(-gt))) * up;
                    }
                    uint2 pk;
                    pk.x = hx_cvt_pk_bf16(v[0], v[1]);
                    pk.y = hx_cvt_pk_bf16(v[2], v[3]);
                    *(uint2 *)(a_mp + hx_xp_index(m, 16 * nt + 8 * j4 + 4 * hl, MG)) = pk;
                }
            }
        }
    } else if (EPI == HX_EPI_LOGITS) {
        // logits and the best (value, index) of this lane's 16 columns, ascending column order
#pragma unroll
        for (int g = 0; g < MG; ++g) {
            const int m = 32 * g + ml;
            float best = -INFINITY;
            int best_n = 0x7fffffff;
#pragma unroll
            for (int j4 = 0; j4 < 4; ++j4) {
                const int n = 32 * nt + 8 * j4 + 4 * hl;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float v = acc[g][4 * j4 + i];
                    if (n + i < a_N && v > best) { best = v; best_n = n + i; }
                }
                if (a_y != nullptr && m < a_M && n < a_N)
                    *(f32x4_t *)(a_y + (size_t)m * a_N + n) =
                        f32x4_t{acc[g][4 * j4], acc[g][4 * j4 + 1], acc[g][4 * j4 + 2], acc[g][4 * j4 + 3]};
            }
            const float ov = __shfl_xor(best, 32);
            const int on = __shfl_xor(best_n, 32);
            if (ov > best || (ov == best && on < best_n)) { best = ov; best_n = on; }
            if (hl == 0 && m < a_M) {
                a_amax_val[(size_t)m * a_n_tiles + nt] = best;
                a_amax_idx[(size_t)m * a_n_tiles + nt] = best_n;
            }
        }
    } else {
        // Temperature sample by Gumbel-max, and the pieces of the log-sum-exp: per (row, tile) the best perturbed
        // score y = z + g with its column and its z, the tile's max of z and its sum of exp(z - max).
        // z = logit * (1/T); g = -log(-log(u)); u from one generator block per 4 consecutive columns.
#pragma unroll
        for (int g = 0; g < MG; ++g) {
            const int m = 32 * g + ml;
            const bool row_ok = m < a_M;
            const uint32_t row = row_ok ? (a_row_ids ? (uint32_t)a_row_ids[m] : (uint32_t)m) : 0u;
            const uint32_t pos = row_ok ? (uint32_t)a_positions[m] : 0u;
            float best = -INFINITY, best_z = 0.f, zmax = -INFINITY;
            int best_n = 0x7fffffff;
            float z[16];
#pragma unroll
            for (int j4 = 0; j4 < 4; ++j4) {
                const int n = 32 * nt + 8 * j4 + 4 * hl;
                uint32_t w[4];
                hx_philox4x32_10((uint32_t)(n >> 2), row, pos, 0x53414D50u, a_key0, a_key1, w);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float zi = acc[g][4 * j4 + i] * a_inv_t;
                    z[4 * j4 + i] = (n + i < a_N) ? zi : -INFINITY;
                    const float u = ((float)(w[i] >> 9) + 0.5f) * (1.0f / 8388608.0f);
                    const float y = zi - logf(-logf(u));
                    if (n + i < a_N) {
                        if (y > best) { best = y; best_n = n + i; best_z = zi; }
                        zmax = fmaxf(zmax, zi);
                    }
                }
                if (a_y != nullptr && row_ok && n < a_N)
                    *(f32x4_t *)(a_y + (size_t)m * a_N + n) =
                        f32x4_t{acc[g][4 * j4], acc[g][4 * j4 + 1], acc[g][4 * j4 + 2], acc[g][4 * j4 + 3]};
            }
            // the two half-wavefronts hold the two halves of the tile's 32 columns
            const float tmax = fmaxf(zmax, __shfl_xor(zmax, 32));
            float sum = 0.f;
            if (tmax > -INFINITY) {
#pragma unroll
                for (int i = 0; i < 16; ++i) sum += expf(z[i] - tmax);     // exp(-inf) = 0 for columns past N
            }
            sum += __shfl_xor(sum, 32);
            const float oy = __shfl_xor(best, 32), oz = __shfl_xor(best_z, 32);
            const int on = __shfl_xor(best_n, 32);
            if (oy > best || (oy == best && on < best_n)) { best = oy; best_n = on; best_z = oz; }
            if (hl == 0 && row_ok) {
                const size_t o = (size_t)m * a_n_tiles + nt;
                a_amax_val[o] = best;
                a_amax_idx[o] = best_n;
                a_samp_z[o] = best_z;
                a_samp_m[o] = tmax;
                a_samp_s[o] = sum;
            }
        }
    }
}

// ---- host side: one launch of a given shape -----------------------------------------------------------------------
#define HX_GEMM_ARGS a.wp, a.xp, a.k_steps, a.n_tiles, a.tile0, a.tile_end, a.steps_per_split, a.steps_per_wave, a.M, a.N, a.y, \
                     a.split_stride, a.mp, a.amax_val, a.amax_idx, a.positions, a.row_ids, a.inv_t, a.key0, a.key1, a.samp_z, a.samp_m, \
                     a.samp_s

template <int MG, int WN, int WK, int EPI>
static int launch_one(dim3 grid, hipStream_t st, const GemmArgs &a) {
    constexpr int lds = gemm_lds_bytes<MG, WN, WK>();
    // the opt-in for more than 64 KiB of LDS is per kernel: once per instantiation, whichever thread comes first
    static std::once_flag once;
    static hipError_t configured = hipSuccess;
    std::call_once(once, [] {
        configured = hipFuncSetAttribute((const void *)gemm_stream_kernel<MG, WN, WK, EPI>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    });
    if (configured != hipSuccess) return hx_fail(HX_E_HIP, "hipFuncSetAttribute: %s", hipGetErrorString(configured));
    dim3 block(64 * (WN * WK + GemmGeom<MG, WK>::NP));
    hipLaunchKernelGGL((gemm_stream_kernel<MG, WN, WK, EPI>), grid, block, lds, st, HX_GEMM_ARGS);
    return HX_OK;
}

template <int MG, int WN, int WK>
static int launch_epi(int epilogue, dim3 grid, hipStream_t st, const GemmArgs &a) {
    if (epilogue == HX_EPI_PARTIAL) return launch_one<MG, WN, WK, HX_EPI_PARTIAL>(grid, st, a);
    if (epilogue == HX_EPI_SWIGLU) return launch_one<MG, WN, WK, HX_EPI_SWIGLU>(grid, st, a);
    if (epilogue == HX_EPI_SAMPLE) return launch_one<MG, WN, WK, HX_EPI_SAMPLE>(grid, st, a);
    return launch_one<MG, WN, WK, HX_EPI_LOGITS>(grid, st, a);
}

template <int MG>
static int launch_shape(int wn, int wk, int epilogue, dim3 grid, hipStream_t st, const GemmArgs &a) {
    if (wk == 1) {
        if (wn == 4) return launch_epi<MG, 4, 1>(epilogue, grid, st, a);
        if (wn == 5) return launch_epi<MG, 5, 1>(epilogue, grid, st, a);
        if (wn == 6) return launch_epi<MG, 6, 1>(epilogue, grid, st, a);
    }
    if (wn == 4 && wk == 2) return launch_epi<MG, 4, 2>(epilogue, grid, st, a);
    if constexpr (MG <= 4) {
        // ten n-tiles per workgroup (twelve wavefronts): only for products that run in several rounds (the LM head)
        if (wn == 10 && wk == 1 && epilogue != HX_EPI_PARTIAL) {
            if (epilogue == HX_EPI_SWIGLU) return launch_one<MG, 10, 1, HX_EPI_SWIGLU>(grid, st, a);
            if (epilogue == HX_EPI_SAMPLE) return launch_one<MG, 10, 1, HX_EPI_SAMPLE>(grid, st, a);
            return launch_one<MG, 10, 1, HX_EPI_LOGITS>(grid, st, a);
        }
    }
    return hx_fail(HX_E_RANGE, "unsupported product shape wn=%d wk=%d for %d m-groups", wn, wk, MG);
}

// ---- host side: how to cut one product into launches ---------------------------------------------------------------
// A workgroup occupies a whole compute unit (128 KiB of LDS), so a launch runs in rounds of as many workgroups as
// the device has compute units (hx_device_cus) and a partly filled last round costs a full one.  Measured on MI355X, wn x 1 shapes (wn n-tiles
// sharing one activation stream, 32 KiB stages, a barrier every 8 k-steps) are the fastest.  The planner
// picks wn in {4, 5, 6, 10} -- and, for products whose consumer kernel sums split partials, the number of
// K-splits (at most HX_MAX_SPLITS, at least 16 k-steps each) -- that minimises the time of the busiest compute
// unit: rounds x (wn tiles + 3 tile-times for the round's own copy of the activations, which every workgroup
// draws from the L2 whatever its width) x whole ring revolutions; split products, which run in one round and
// read only a K-slice of the activations, and 256-row products keep a small charge per extra tile instead (five
// consumers on four SIMDs); ties go to the smaller wn and fewer splits.
// Examples: the 1184 tiles of the 7B gate|up matrix make 296 workgroups of 4 (two rounds on 256 compute
// units) but 237 workgroups of 5 (one round); the 4752 tiles of the LM head make five rounds of 4, four of 5 or
// two of 10, measured 253 / 244 / 230 us.  Ten tiles per workgroup are twelve wavefronts (three per SIMD): only
// for products without split partials and up to 128 rows.  HX_GEMM_SHAPE="wn,wk,splits" overrides (tuning).

struct gemm_launch { int wn, wk, splits, tile0, tiles; };

static int plan_product(int n_tiles, int k_steps, int mg, bool partial, gemm_launch *out) {
    const int cus = hx_device_cus();
    gemm_launch best{4, 1, 1, 0, n_tiles};
    double best_cost = 1e300;
    int max_s = partial ? HX_MAX_SPLITS : 1;
    if (const char *cap = getenv("HX_GEMM_MAX_SPLITS")) max_s = partial ? std::max(1, std::min(HX_MAX_SPLITS, atoi(cap))) : 1;
    static const int widths[] = {4, 5, 6, 10};
    for (int wn : widths) {
        if (wn == 10 && (partial || mg > 4)) continue;
        for (int s = 1; s <= max_s; ++s) {
            if (s > 1 && k_steps / s < 16) break;
            const int wgs = ((n_tiles + wn - 1) / wn) * s;
            const int rounds = (wgs + cus - 1) / cus;
            const int sps = (k_steps + s - 1) / s;
            // busiest compute unit: rounds x (wn tiles + the activations) x whole ring revolutions (one more to fill
            // the ring), plus a small charge per split for writing and re-reading its partial tile
            const int revolutions = (sps + HX_GEMM_RING - 1) / HX_GEMM_RING + 1;
            const double width = (partial || mg > 4) ? wn + 0.35 * (wn - 4) : wn + 3.0;   // as measured on each kind
            const double cost = (double)rounds * width * revolutions * (1.0 + 0.02 * (s - 1));
            if (cost < best_cost - 1e-9) { best_cost = cost; best.wn = wn; best.splits = s; }
        }
    }
    int a, b, c;
    const char *ov = getenv("HX_GEMM_SHAPE");
    if (ov && sscanf(ov, "%d,%d,%d", &a, &b, &c) == 3 && c >= 1 && c <= max_s && k_steps / (b * c) >= 1 &&
        ((b == 1 && a >= 4 && a <= 6) || (a == 4 && b == 2))) {
        best.wn = a; best.wk = b; best.splits = c;
    }
    out[0] = best;
    return 1;
}

// The plan of one product, for inspection: tiles per workgroup, k-slices per workgroup, K-splits.
extern "C" int hx_plan_product(int32_t n_tiles, int32_t k_steps, int32_t batch, int32_t partial, int32_t *wn_out,
                               int32_t *wk_out, int32_t *splits_out) {
    if (!wn_out || !wk_out || !splits_out) return hx_fail(HX_E_NULL, "an output pointer is NULL");
    if (n_tiles < 1 || k_steps < 1 || batch < 1 || batch > 256) return hx_fail(HX_E_RANGE, "product %d x %d for batch %d", n_tiles, k_steps, batch);
    gemm_launch plan[2];
    plan_product(n_tiles, k_steps, hx_m_groups(batch), partial != 0, plan);
    *wn_out = plan[0].wn; *wk_out = plan[0].wk; *splits_out = plan[0].splits;
    return HX_OK;
}

int hx_gemm_splits(const hx_matrix *m, int batch) {
    gemm_launch plan[2];
    plan_product(m->n_tiles, m->k_steps, hx_m_groups(batch), true, plan);
    return plan[0].splits;
}

int hx_launch_gemm(const hx_engine *e, const hx_matrix *m, int batch, const void *xp, int epilogue, float *y,
                   void *mp_out, hipStream_t st, const hx_sample_params *sample) {
    if (epilogue == HX_EPI_SAMPLE && !sample) return hx_fail(HX_E_NULL, "sampling parameters missing");
    const int mg = hx_m_groups(batch);
    const bool partial = epilogue == HX_EPI_PARTIAL;
    gemm_launch plan[2];
    const int n_launch = plan_product(m->n_tiles, m->k_steps, mg, partial, plan);
    for (int li = 0; li < n_launch; ++li) {
        const gemm_launch &pl = plan[li];
        GemmArgs a;
        a.wp = (const uint4 *)(e->weights + m->offset);
        a.xp = (const uint4 *)xp;
        a.k_steps = m->k_steps;
        a.n_tiles = m->n_tiles;
        a.tile0 = pl.tile0;
        a.tile_end = pl.tile0 + pl.tiles;
        a.steps_per_split = (m->k_steps + pl.splits - 1) / pl.splits;
        a.steps_per_wave = (a.steps_per_split + pl.wk - 1) / pl.wk;
        a.M = batch;
        a.N = m->N;
        a.y = y;
        a.split_stride = (size_t)batch * m->N;
        a.mp = (uint16_t *)mp_out;
        a.amax_val = (float *)(e->ws + e->map.amax_val);
        a.amax_idx = (int32_t *)(e->ws + e->map.amax_idx);
        a.positions = sample ? sample->positions : nullptr;
        a.row_ids = sample ? sample->row_ids : nullptr;
        a.inv_t = sample ? sample->inv_temperature : 1.0f;
        a.key0 = sample ? sample->key0 : 0u;
        a.key1 = sample ? sample->key1 : 0u;
        a.samp_z = (float *)(e->ws + e->map.samp_z);
        a.samp_m = (float *)(e->ws + e->map.samp_m);
        a.samp_s = (float *)(e->ws + e->map.samp_s);
        dim3 grid((pl.tiles + pl.wn - 1) / pl.wn, pl.splits);
        int rc;
        switch (mg) {
            case 1: rc = launch_shape<1>(pl.wn, pl.wk, epilogue, grid, st, a); break;
            case 2: rc = launch_shape<2>(pl.wn, pl.wk, epilogue, grid, st, a); break;
            case 4: rc = launch_shape<4>(pl.wn, pl.wk, epilogue, grid, st, a); break;
            case 8: rc = launch_shape<8>(pl.wn, pl.wk, epilogue, grid, st, a); break;
            default: return hx_fail(HX_E_RANGE, "batch %d exceeds 256", batch);
        }
        if (rc) return rc;
        HX_CHECK_LAUNCH("gemm_stream");
    }
    return HX_OK;
}

// ---- greedy token: reduce the per-tile candidates of each row ---------------------------------------------------
// grid = batch, 256 threads.  Largest value wins, ties go to the smaller index.
__global__ __launch_bounds__(256) void argmax_final_kernel(const float *__restrict__ val, const int32_t *__restrict__ idx,
                                                           int n_tiles, int32_t *__restrict__ out) {
    __shared__ float sv[256];
    __shared__ int32_t si[256];
    const int m = blockIdx.x, tid = threadIdx.x;
    float best = -INFINITY;
    int32_t bi = 0x7fffffff;
    for (int t = tid; t < n_tiles; t += 256) {
        float v = val[(size_t)m * n_tiles + t];
        int32_t i = idx[(size_t)m * n_tiles + t];
        if (v > best || (v == best && i < bi)) { best = v; bi = i; }
    }
    sv[tid] = best; si[tid] = bi;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (tid < off) {
            float v = sv[tid + off]; int32_t i = si[tid + off];
            if (v > sv[tid] || (v == sv[tid] && i < si[tid])) { sv[tid] = v; si[tid] = i; }
        }
        __syncthreads();
    }
    if (tid == 0) out[m] = si[0];
}

int hx_launch_argmax_final(const hx_engine *e, int batch, int32_t *tokens_out, hipStream_t st) {
    hipLaunchKernelGGL(argmax_final_kernel, dim3(batch), dim3(256), 0, st, (const float *)(e->ws + e->map.amax_val),
                       (const int32_t *)(e->ws + e->map.amax_idx), e->wlm.n_tiles, tokens_out);
    HX_CHECK_LAUNCH("argmax_final");
    return HX_OK;
}

// ---- sampled token and its log-probability: reduce the per-tile pieces of each row -----------------------------
// grid = batch, 256 threads.  Largest perturbed score wins (ties: smaller column); log-sum-exp of the scaled
// logits = M + log(sum_t s_t exp(m_t - M)) with M = max_t m_t; logprob = z_token - that.  Fixed tree: deterministic.
__global__ __launch_bounds__(256) void sample_final_kernel(const float *__restrict__ val, const int32_t *__restrict__ idx,
                                                           const float *__restrict__ zc, const float *__restrict__ tm,
                                                           const float *__restrict__ tsum, int n_tiles,
                                                           int32_t *__restrict__ tok_out, float *__restrict__ lp_out) {
    __shared__ float sv[256], sz[256], sm[256];
    __shared__ int32_t si[256];
    const int m = blockIdx.x, tid = threadIdx.x;
    const size_t base = (size_t)m * n_tiles;
    float best = -INFINITY, bz = 0.f, mx = -INFINITY;
    int32_t bi = 0x7fffffff;
    for (int t = tid; t < n_tiles; t += 256) {
        const float v = val[base + t];
        const int32_t i = idx[base + t];
        if (v > best || (v == best && i < bi)) { best = v; bi = i; bz = zc[base + t]; }
        mx = fmaxf(mx, tm[base + t]);
    }
    sv[tid] = best; si[tid] = bi; sz[tid] = bz; sm[tid] = mx;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (tid < off) {
            const float v = sv[tid + off]; const int32_t i = si[tid + off];
            if (v > sv[tid] || (v == sv[tid] && i < si[tid])) { sv[tid] = v; si[tid] = i; sz[tid] = sz[tid + off]; }
            sm[tid] = fmaxf(sm[tid], sm[tid + off]);
        }
        __syncthreads();
    }
    const float M = sm[0];
    __syncthreads();
    float part = 0.f;
    for (int t = tid; t < n_tiles; t += 256) part += tsum[base + t] * expf(tm[base + t] - M);
    sm[tid] = part;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (tid < off) sm[tid] += sm[tid + off];
        __syncthreads();
    }
    if (tid == 0) {
        tok_out[m] = si[0];
        lp_out[m] = sz[0] - (M + logf(sm[0]));
    }
}

int hx_launch_sample_final(const hx_engine *e, int batch, int32_t *tokens_out, float *logprobs_out, hipStream_t st) {
    hipLaunchKernelGGL(sample_final_kernel, dim3(batch), dim3(256), 0, st, (const float *)(e->ws + e->map.amax_val),
                       (const int32_t *)(e->ws + e->map.amax_idx), (const float *)(e->ws + e->map.samp_z),
                       (const float *)(e->ws + e->map.samp_m), (const float *)(e->ws + e->map.samp_s), e->wlm.n_tiles,
                       tokens_out, logprobs_out);
    HX_CHECK_LAUNCH("sample_final");
    return HX_OK;
}
