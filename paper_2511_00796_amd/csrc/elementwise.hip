// Row-wise kernels between the matrix products: embedding gather, split-sum + residual add + RMSNorm
// (which also rounds to bf16 and writes the packed B operand of the next product), and the small
// pack / unpack helpers used by the single-stage hooks.
#include "hx_internal.h"

// 512 threads x 8 elements cover a row of up to 4096 in one iteration, i.e. one memory round trip for the residual
// and all split partials (measured against 256 threads at hidden 3584: 8.3 instead of 8.8 us per launch, timed with events)
#define HX_NORM_THREADS 512
#define HX_NORM_MAX_IT (HX_MAX_HIDDEN / (HX_NORM_THREADS * 8))   // 8 elements per thread per iteration

__device__ __forceinline__ float block_sum(float v, float *red) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    static_assert(HX_NORM_THREADS == 512, "eight wavefront sums");
    const float t = ((red[0] + red[1]) + (red[2] + red[3])) + ((red[4] + red[5]) + (red[6] + red[7]));
    __syncthreads();
    return t;
}

// MODE 0: x = embed[token]          (start of the step)
// MODE 1: x += sum_s ypart[s]       (after the output / down projection)
// MODE 2: x read only               (norm of a caller-supplied row; nothing stored back to x)
// then u = bf16( x * rsqrt(mean(x^2) + eps) * g ) into the packed buffer xp, or as fp32 into y_f32.
template <int MODE>
__global__ __launch_bounds__(HX_NORM_THREADS) void norm_kernel(float *__restrict__ x, const float *__restrict__ x_in,
                                                              const int32_t *__restrict__ tokens,
                                                              const uint16_t *__restrict__ embed,
                                                              const float *__restrict__ ypart, int splits,
                                                              size_t split_stride, const uint16_t *__restrict__ gain,
                                                              int H, float eps, uint16_t *__restrict__ xp, int m_groups,
                                                              float *__restrict__ y_f32, size_t block_stride) {
    __shared__ float red[8];
    const int b = blockIdx.x;
    if (blockIdx.y) {               // further row blocks of a wide prompt call: same layout, block_stride bytes apart
        const size_t off = (size_t)blockIdx.y * block_stride;
        x = (float *)((char *)x + off);
        if (ypart) ypart = (const float *)((const char *)ypart + off);
        xp = (uint16_t *)((char *)xp + off);
        if (tokens) tokens += (size_t)blockIdx.y * gridDim.x;
    }
    float v[HX_NORM_MAX_IT][8];
    float ss = 0.f;
#pragma unroll
    for (int it = 0; it < HX_NORM_MAX_IT; ++it) {
        const int i0 = (it * HX_NORM_THREADS + threadIdx.x) * 8;
        if (i0 < H) {
            if (MODE == 0) {
                const uint4 raw = *(const uint4 *)(embed + (size_t)tokens[b] * H + i0);
                const uint16_t *e16 = (const uint16_t *)&raw;
#pragma unroll
                for (int j = 0; j < 8; ++j) v[it][j] = hx_bf16_to_f32(e16[j]);
            } else {
                const float *src = (MODE == 1 ? x : x_in) + (size_t)b * H + i0;
                const f32x4_t a = *(const f32x4_t *)src, c = *(const f32x4_t *)(src + 4);
#pragma unroll
                for (int j = 0; j < 4; ++j) { v[it][j] = a[j]; v[it][4 + j] = c[j]; }
                if (MODE == 1) {
                    // all split partials are requested before the first is used (one memory round trip instead
                    // of one per split); they are added in split order
                    f32x4_t ya[HX_MAX_SPLITS], yc[HX_MAX_SPLITS];
#pragma unroll
                    for (int s = 0; s < HX_MAX_SPLITS; ++s) {
                        const float *yp = ypart + min(s, splits - 1) * split_stride + (size_t)b * H + i0;
                        ya[s] = *(const f32x4_t *)yp;
                        yc[s] = *(const f32x4_t *)(yp + 4);
                    }
                    float add[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) add[j] = 0.f;
#pragma unroll
                    for (int s = 0; s < HX_MAX_SPLITS; ++s) {
                        if (s < splits) {
#pragma unroll
                            for (int j = 0; j < 4; ++j) { add[j] += ya[s][j]; add[4 + j] += yc[s][j]; }
                        }
                    }
#pragma unroll
                    for (int j = 0; j < 8; ++j) v[it][j] += add[j];
                }
            }
            if (MODE != 2) {
                float *dst = x + (size_t)b * H + i0;
                *(f32x4_t *)dst = f32x4_t{v[it][0], v[it][1], v[it][2], v[it][3]};
                *(f32x4_t *)(dst + 4) = f32x4_t{v[it][4], v[it][5], v[it][6], v[it][7]};
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) ss += v[it][j] * v[it][j];
        }
    }
    // the gains are requested before the block-wide sum, so their round trip overlaps it
    uint4 graw_all[HX_NORM_MAX_IT];
#pragma unroll
    for (int it = 0; it < HX_NORM_MAX_IT; ++it) {
        const int i0 = (it * HX_NORM_THREADS + threadIdx.x) * 8;
        graw_all[it] = i0 < H ? *(const uint4 *)(gain + i0) : make_uint4(0u, 0u, 0u, 0u);
    }
    ss = block_sum(ss, red);
    const float r = 1.0f / sqrtf(ss / (float)H + eps);
#pragma unroll
    for (int it = 0; it < HX_NORM_MAX_IT; ++it) {
        const int i0 = (it * HX_NORM_THREADS + threadIdx.x) * 8;
        if (i0 < H) {
            const uint4 graw = graw_all[it];
            const uint16_t *g16 = (const uint16_t *)&graw;
            float u[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) u[j] = v[it][j] * r * hx_bf16_to_f32(g16[j]);
            if (y_f32 != nullptr) {
#pragma unroll
                for (int j = 0; j < 8; ++j) y_f32[(size_t)b * H + i0 + j] = hx_bf16_to_f32(hx_f32_to_bf16(u[j]));
            } else {
                uint4 pk;
                pk.x = hx_pack_bf16x2(u[0], u[1]); pk.y = hx_pack_bf16x2(u[2], u[3]);
                pk.z = hx_pack_bf16x2(u[4], u[5]); pk.w = hx_pack_bf16x2(u[6], u[7]);
                *(uint4 *)(xp + hx_xp_index(b, i0, m_groups)) = pk;
            }
        }
    }
}

int hx_launch_embed_norm(const hx_engine *e, int batch, const int32_t *tokens, size_t gain_off, hipStream_t st, int blocks,
                         size_t block_stride) {
    hipLaunchKernelGGL((norm_kernel<0>), dim3(batch, blocks), dim3(HX_NORM_THREADS), 0, st, (float *)(e->ws + e->map.x),
                       (const float *)nullptr, tokens, (const uint16_t *)(e->weights + e->embed),
                       (const float *)nullptr, 0, (size_t)0, (const uint16_t *)(e->weights + gain_off), e->cfg.hidden,
                       e->cfg.rms_eps, (uint16_t *)(e->ws + e->map.xp), hx_m_groups(batch), (float *)nullptr, block_stride);
    HX_CHECK_LAUNCH("embed_norm");
    return HX_OK;
}

int hx_launch_reduce_norm(const hx_engine *e, int batch, const float *ypart, int splits, size_t split_stride,
                          size_t gain_off, hipStream_t st, int blocks, size_t block_stride) {
    hipLaunchKernelGGL((norm_kernel<1>), dim3(batch, blocks), dim3(HX_NORM_THREADS), 0, st, (float *)(e->ws + e->map.x),
                       (const float *)nullptr, (const int32_t *)nullptr, (const uint16_t *)nullptr, ypart, splits,
                       split_stride, (const uint16_t *)(e->weights + gain_off), e->cfg.hidden, e->cfg.rms_eps,
                       (uint16_t *)(e->ws + e->map.xp), hx_m_groups(batch), (float *)nullptr, block_stride);
    HX_CHECK_LAUNCH("reduce_norm");
    return HX_OK;
}

int hx_launch_norm_only(const hx_engine *e, int batch, const float *x, size_t gain_off, float *y, hipStream_t st) {
    hipLaunchKernelGGL((norm_kernel<2>), dim3(batch), dim3(HX_NORM_THREADS), 0, st, (float *)nullptr, x,
                       (const int32_t *)nullptr, (const uint16_t *)nullptr, (const float *)nullptr, 0, (size_t)0,
                       (const uint16_t *)(e->weights + gain_off), e->cfg.hidden, e->cfg.rms_eps, (uint16_t *)nullptr,
                       hx_m_groups(batch), y, (size_t)0);
    HX_CHECK_LAUNCH("norm_only");
    return HX_OK;
}

// ---- stage-hook helpers ------------------------------------------------------------------------------------------
// fp32 [batch, K] -> bf16 packed activations (rounding on entry), and back (as fp32 holding bf16 values)
__global__ void pack_x_kernel(const float *__restrict__ x, int batch, int K, uint16_t *__restrict__ xp, int m_groups) {
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (int64_t)batch * K) return;
    int m = (int)(gid / K), k = (int)(gid % K);
    xp[hx_xp_index(m, k, m_groups)] = hx_f32_to_bf16(x[gid]);
}
__global__ void unpack_x_kernel(const uint16_t *__restrict__ xp, int batch, int K, float *__restrict__ x, int m_groups) {
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (int64_t)batch * K) return;
    int m = (int)(gid / K), k = (int)(gid % K);
    x[gid] = hx_bf16_to_f32(xp[hx_xp_index(m, k, m_groups)]);
}
int hx_launch_pack_x(const hx_engine *e, int batch, const float *x, int K, void *xp, hipStream_t st) {
    int64_t n = (int64_t)batch * K;
    hipLaunchKernelGGL(pack_x_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, x, batch, K, (uint16_t *)xp,
                       hx_m_groups(batch));
    HX_CHECK_LAUNCH("pack_x");
    return HX_OK;
}
int hx_launch_unpack_x(const hx_engine *e, int batch, const void *xp, int K, float *x, hipStream_t st) {
    int64_t n = (int64_t)batch * K;
    hipLaunchKernelGGL(unpack_x_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const uint16_t *)xp, batch,
                       K, x, hx_m_groups(batch));
    HX_CHECK_LAUNCH("unpack_x");
    return HX_OK;
}

// packed queries <-> fp32 [batch, n_q * D]
__global__ void q_pack_kernel(float *__restrict__ q, uint16_t *__restrict__ qp, int batch, int n_q, int n_kv, int G,
                              int D, bool unpack) {
    // one thread per (b, kvh, g in 0..15, d)
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = (int64_t)batch * n_kv * 16 * D;
    if (gid >= total) return;
    int d = (int)(gid % D);
    int g = (int)((gid / D) % 16);
    int kvh = (int)((gid / ((int64_t)D * 16)) % n_kv);
    int b = (int)(gid / ((int64_t)D * 16 * n_kv));
    uint16_t *dst = qp + ((size_t)b * n_kv + kvh) * (D / 32) * 512 + (d >> 5) * 512 + ((((d >> 3) & 3) * 16 + g) << 3) + (d & 7);
    if (g < G) {
        size_t li = ((size_t)b * n_q + kvh * G + g) * D + d;
        if (unpack) q[li] = hx_bf16_to_f32(*dst);
        else *dst = hx_f32_to_bf16(q[li]);
    } else if (!unpack) {
        *dst = 0;
    }
}
int hx_launch_unpack_q(const hx_engine *e, int batch, float *q_out, hipStream_t st) {
    int64_t n = (int64_t)batch * e->cfg.n_kv_heads * 16 * e->D;
    hipLaunchKernelGGL(q_pack_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, q_out,
                       (uint16_t *)(e->ws + e->map.qp), batch, e->cfg.n_q_heads, e->cfg.n_kv_heads, e->G, e->D, true);
    HX_CHECK_LAUNCH("unpack_q");
    return HX_OK;
}
int hx_launch_pack_q(const hx_engine *e, int batch, const float *q, hipStream_t st, const hx_attn_bufs *bufs) {
    int64_t n = (int64_t)batch * e->cfg.n_kv_heads * 16 * e->D;
    hipLaunchKernelGGL(q_pack_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (float *)q,
                       bufs ? bufs->qp : (uint16_t *)(e->ws + e->map.qp), batch, e->cfg.n_q_heads, e->cfg.n_kv_heads, e->G, e->D, false);
    HX_CHECK_LAUNCH("pack_q");
    return HX_OK;
}

// y[m][n] = sum_s ypart[s][m][n], split order
__global__ void sum_partials_kernel(const float *__restrict__ ypart, int splits, size_t split_stride, int64_t n,
                                    float *__restrict__ y) {
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= n) return;
    float s = 0.f;
    for (int sp = 0; sp < splits; ++sp) s += ypart[sp * split_stride + gid];
    y[gid] = s;
}
int hx_launch_sum_partials(const hx_engine *e, int batch, const float *ypart, int splits, size_t split_stride, int N,
                           float *y, hipStream_t st) {
    int64_t n = (int64_t)batch * N;
    hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, ypart, splits,
                       split_stride, n, y);
    HX_CHECK_LAUNCH("sum_partials");
    return HX_OK;
}
