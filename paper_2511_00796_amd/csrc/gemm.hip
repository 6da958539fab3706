// Small-M weight-streaming matrix products  Y[M, N] = X[M, K] W[K, N]  (M = batch <= 256).
//
// The weights dominate the bytes, so the kernel is organised around streaming each packed weight
// tile exactly once, straight from HBM into the A operand of v_mfma_f32_32x32x16_bf16 (32 output
// columns n x 16 k per 1-KiB load).  The activations are the B operand (16 k x 32 batch rows per
// m-group); they are small, L2-resident, and shared by the four wavefronts of a workgroup through
// a double-buffered LDS copy.  Each wavefront owns one 32-column n-tile and all batch rows, so the
// accumulator is MG tiles of 32 x 32 fp32.  Along K the product may be split over workgroups; the
// fp32 partial results are summed in split order by the consumer kernel (deterministic).
//
// Epilogues: plain fp32 partials; SiLU(gate) * up -> bf16 packed activations of the down
// projection; logits + per-tile argmax candidates.
#include "hx_internal.h"

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
template <int MG> struct GemmCfg { static constexpr int KC = (MG == 8) ? 4 : 8; };   // k-steps per LDS chunk

struct GemmArgs {
    const uint4 *wp;      // packed weights
    const uint4 *xp;      // packed activations
    int k_steps, n_tiles, steps_per_split;
    int M, N;
    float *y;             // PARTIAL: [splits][M][N]; LOGITS: [M][N] or NULL
    size_t split_stride;  // elements between splits of y
    uint16_t *mp;         // SWIGLU: packed bf16 output
    float *amax_val;      // LOGITS: [M][n_tiles]
    int32_t *amax_idx;
};

template <int MG, int EPI>
__global__ __launch_bounds__(256) void gemm_stream_kernel(GemmArgs a) {
    constexpr int KC = GemmCfg<MG>::KC;
    constexpr int XV = KC * MG / 4;                      // uint4 per thread per staged chunk
    __shared__ uint4 xs[2][KC * MG * 64];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int nt = blockIdx.x * 4 + wave;
    const bool active = nt < a.n_tiles;                  // inactive wavefronts still stage activations
    const int ks0 = blockIdx.y * a.steps_per_split;
    const int ks1 = min(a.k_steps, ks0 + a.steps_per_split);
    const int n_chunks = (ks1 - ks0 + KC - 1) / KC;

    f32x16_t acc[MG];
#pragma unroll
    for (int g = 0; g < MG; ++g)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[g][r] = 0.f;

    const uint4 *wrow = a.wp + ((size_t)(active ? nt : 0) * a.k_steps) * 64 + lane;
    uint4 wcur[KC], wnxt[KC], xr[XV];

    auto load_w = [&](uint4 *w, int ci) {
        const int s0 = ks0 + ci * KC;
#pragma unroll
        for (int s = 0; s < KC; ++s)
            if (active && s0 + s < ks1) w[s] = wrow[(size_t)(s0 + s) * 64];
    };
    auto load_x = [&](int ci) {
        const int s0 = ks0 + ci * KC;
        const int n_u4 = (min(ks1, s0 + KC) - s0) * MG * 64;
        const uint4 *src = a.xp + (size_t)s0 * MG * 64;
#pragma unroll
        for (int i = 0; i < XV; ++i)
            if (tid + i * 256 < n_u4) xr[i] = src[tid + i * 256];
    };
    auto store_x = [&](int ci, int buf) {
        const int s0 = ks0 + ci * KC;
        const int n_u4 = (min(ks1, s0 + KC) - s0) * MG * 64;
#pragma unroll
        for (int i = 0; i < XV; ++i)
            if (tid + i * 256 < n_u4) xs[buf][tid + i * 256] = xr[i];
    };
    auto compute = [&](const uint4 *w, int ci, int buf) {
        const int steps = min(ks1, ks0 + (ci + 1) * KC) - (ks0 + ci * KC);
#pragma unroll
        for (int s = 0; s < KC; ++s) {
            if (s < steps) {
                const bf16x8_t aop = __builtin_bit_cast(bf16x8_t, w[s]);
#pragma unroll
                for (int g = 0; g < MG; ++g) {
                    const bf16x8_t bop = __builtin_bit_cast(bf16x8_t, xs[buf][(s * MG + g) * 64 + lane]);
                    acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop, bop, acc[g], 0, 0, 0);
                }
            }
        }
    };

    if (n_chunks > 0) {
        load_x(0);
        load_w(wcur, 0);
        store_x(0, 0);
        __syncthreads();
        for (int ci = 0; ci < n_chunks; ci += 2) {
            // even chunk: compute from wcur / buffer 0, prefetch into wnxt / buffer 1
            if (ci + 1 < n_chunks) { load_x(ci + 1); load_w(wnxt, ci + 1); }
            if (active) compute(wcur, ci, 0);
            if (ci + 1 < n_chunks) store_x(ci + 1, 1);
            __syncthreads();
            if (ci + 1 >= n_chunks) break;
            // odd chunk
            if (ci + 2 < n_chunks) { load_x(ci + 2); load_w(wcur, ci + 2); }
            if (active) compute(wnxt, ci + 1, 1);
            if (ci + 2 < n_chunks) store_x(ci + 2, 0);
            __syncthreads();
        }
    }
    if (!active) return;

    // accumulator register r of lane l: column m = 32*g + l%32, row n = 32*nt + 8*(r/4) + 4*(l/32) + r%4
    const int hl = lane >> 5, ml = lane & 31;
    if (EPI == HX_EPI_PARTIAL) {
        float *y = a.y + blockIdx.y * a.split_stride;
#pragma unroll
        for (int g = 0; g < MG; ++g) {
            const int m = 32 * g + ml;
            if (m < a.M) {
#pragma unroll
                for (int j4 = 0; j4 < 4; ++j4) {
                    const int n = 32 * nt + 8 * j4 + 4 * hl;
                    if (n < a.N)
                        *(f32x4_t *)(y + (size_t)m * a.N + n) =
                            f32x4_t{acc[g][4 * j4], acc[g][4 * j4 + 1], acc[g][4 * j4 + 2], acc[g][4 * j4 + 3]};
                }
            }
        }
    } else if (EPI == HX_EPI_SWIGLU) {
        // rows 0..15 of the tile are gate columns 16*nt + p, rows 16..31 the matching up columns
#pragma unroll
        for (int g = 0; g < MG; ++g) {
            const int m = 32 * g + ml;
            if (m < a.M) {
#pragma unroll
                for (int j4 = 0; j4 < 2; ++j4) {
                    float v[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float gt = acc[g][4 * j4 + i], up = acc[g][8 + 4 * j4 + i];
                        v[i] = (gt / (1.0f + expf(-gt))) * up;
                    }
                    uint2 pk;
                    pk.x = hx_pack_bf16x2(v[0], v[1]);
                    pk.y = hx_pack_bf16x2(v[2], v[3]);
                    *(uint2 *)(a.mp + hx_xp_index(m, 16 * nt + 8 * j4 + 4 * hl, MG)) = pk;
                }
            }
        }
    } else {
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
                    if (n + i < a.N && v > best) { best = v; best_n = n + i; }
                }
                if (a.y != nullptr && m < a.M && n < a.N)
                    *(f32x4_t *)(a.y + (size_t)m * a.N + n) =
                        f32x4_t{acc[g][4 * j4], acc[g][4 * j4 + 1], acc[g][4 * j4 + 2], acc[g][4 * j4 + 3]};
            }
            const float ov = __shfl_xor(best, 32);
            const int on = __shfl_xor(best_n, 32);
            if (ov > best || (ov == best && on < best_n)) { best = ov; best_n = on; }
            if (hl == 0 && m < a.M) {
                a.amax_val[(size_t)m * a.n_tiles + nt] = best;
                a.amax_idx[(size_t)m * a.n_tiles + nt] = best_n;
            }
        }
    }
}

int hx_launch_gemm(const hx_engine *e, const hx_matrix *m, int batch, const void *xp, int epilogue, float *y,
                   void *mp_out, hipStream_t st) {
    GemmArgs a;
    a.wp = (const uint4 *)(e->weights + m->offset);
    a.xp = (const uint4 *)xp;
    a.k_steps = m->k_steps;
    a.n_tiles = m->n_tiles;
    const int splits = (epilogue == HX_EPI_PARTIAL) ? m->splits : 1;
    a.steps_per_split = (m->k_steps + splits - 1) / splits;
    a.M = batch;
    a.N = m->N;
    a.y = y;
    a.split_stride = (size_t)batch * m->N;
    a.mp = (uint16_t *)mp_out;
    a.amax_val = (float *)(e->ws + e->map.amax_val);
    a.amax_idx = (int32_t *)(e->ws + e->map.amax_idx);
    dim3 grid((m->n_tiles + 3) / 4, splits), block(256);
    const int mg = hx_m_groups(batch);
#define HX_GEMM_CASE(MGV)                                                                                          \
    case MGV:                                                                                                      \
        if (epilogue == HX_EPI_PARTIAL) hipLaunchKernelGGL((gemm_stream_kernel<MGV, HX_EPI_PARTIAL>), grid, block, 0, st, a); \
        else if (epilogue == HX_EPI_SWIGLU) hipLaunchKernelGGL((gemm_stream_kernel<MGV, HX_EPI_SWIGLU>), grid, block, 0, st, a); \
        else hipLaunchKernelGGL((gemm_stream_kernel<MGV, HX_EPI_LOGITS>), grid, block, 0, st, a);                  \
        break;
    switch (mg) {
        HX_GEMM_CASE(1)
        HX_GEMM_CASE(2)
        HX_GEMM_CASE(4)
        HX_GEMM_CASE(8)
        default: return hx_fail(HX_E_RANGE, "batch %d exceeds 256", batch);
    }
#undef HX_GEMM_CASE
    HX_CHECK_LAUNCH("gemm_stream");
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
