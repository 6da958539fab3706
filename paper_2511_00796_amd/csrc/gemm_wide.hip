// Products for many prompt rows at once: C[R x 256 rows][N] = X W with BOTH operands tiled through LDS, so that a
// weight is read from HBM once per call instead of once per 256 rows (prompt processing, Section 1 stage (i) of the
// rollout; the step before decoding).  The streaming kernel of gemm.hip keeps one weight tile per wavefront in
// registers and is right for up to 256 rows; here a workgroup owns a 256 x 256 (or 256 x 192) tile of the output.
//
// Layouts are the decode step's (hx_internal.h): weights [n_tile][k_step][lane][8], activations of each 256-row block
// [k_step][8 m-groups][lane][8] in that block's workspace.  Both are already in matrix-core operand order, so
// staging is a plain copy of 1-KiB pieces and every LDS read is 16 contiguous bytes per lane (conflict-free).
//
// Workgroup = 4 wavefronts in 2 x 2, each a 128 x 128 sub-tile = 4 x 4 accumulators of 32 x 32 (256 accumulator
// registers: all a wavefront has beside its 256 ordinary ones, which is why there are no producer wavefronts).
// A chunk is 2 k-steps: 16 pieces of X and 16 of W (32 KiB).  Every wavefront copies a quarter of each chunk,
// global -> registers -> LDS: requested three chunks ahead (two register sets), written to LDS one chunk ahead, two
// LDS stages, one barrier per chunk.  The barrier of chunk c + 1 is passed BEFORE the last k-step of chunk c is
// multiplied, so that the first operand reads of the next chunk hide behind those products.  Measured on MI355X
// (7B gate|up, 2048 rows): 45-48 % of the bf16 matrix peak.  The kernel with its copies alone (no arithmetic) takes as
// long as the whole kernel: what bounds it is the rate at which the compute units can draw from the L2 (8-9 TB/s over
// the chip, about 35 GB/s per compute unit when all are busy, however local the traffic: 80 % of the L2 requests of
// this product hit), not the matrix cores (66 % with the copies removed) and not the LDS.  The direct global -> LDS
// path (global_load_lds) was slower; a larger output tile, the only way to draw fewer bytes per flop, spills.
//
// Workgroup numbering: consecutive workgroup ids go to different XCDs, so id -> (xcd, slot); the workgroups of one
// XCD take all row blocks of a few column blocks and walk K in step: each XCD's L2 sees every weight once.
#include "hx_internal.h"
#include <algorithm>
#include <mutex>

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

namespace {

constexpr int WIDE_KC = 2;        // k-steps per chunk
constexpr int wide_lds_bytes(int wnt) { return 2 * WIDE_KC * (8 + wnt) * 1024; }

#define HX_WIDE_LGKM0 0xC07F      /* s_waitcnt lgkmcnt(0) and nothing else */

struct WideArgs {
    const uint4 *wp;              // packed weights of the matrix
    int k_steps, n_tiles, N;
    const char *xp0;              // block 0's packed activations; block b's are block_stride bytes further
    size_t block_stride;
    int R;                        // 256-row blocks
    float *y0;                    // fp32 output of block 0 ([splits][256][N]), same stride between blocks
    int steps_per_split;
    uint16_t *mp0;                // SiLU(gate)*up output of block 0 (packed activations, 8 m-groups)
};

// WNT: 32-column tiles per workgroup: 8 (a 256 x 256 output tile) or 6 (256 x 192, for products that would otherwise
// leave compute units idle)
template <int WNT, int EPI, bool TAIL>
__global__ __launch_bounds__(256) void gemm_wide_kernel(WideArgs a) {
    constexpr int KC = WIDE_KC, TW = WNT / 2, PIECES = KC * (8 + WNT), LPW = PIECES / 4, STAGE_U4 = PIECES * 64;
    extern __shared__ u32x4_t lds[];                    // [2 stages][PIECES][64 lanes]
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int w = blockIdx.x, xcd = w & 7, slot = w >> 3;
    const int b = slot % a.R, nbl = (slot / a.R) * 8 + xcd;
    const int NB = (a.n_tiles + WNT - 1) / WNT;
    if (nbl >= NB) return;                              // whole workgroup, before any barrier
    const int nt0 = nbl * WNT;
    const int k_steps = a.k_steps;
    const int k0 = blockIdx.y * a.steps_per_split, k1 = min(k_steps, k0 + a.steps_per_split);
    const int n_chunks = (k1 - k0 + KC - 1) / KC;
    const uint4 *xp = (const uint4 *)(a.xp0 + (size_t)b * a.block_stride);
    // this wavefront's share of the copies of a chunk: LPW streams, each a wave-uniform pointer that advances by a
    // fixed step per chunk and stops at the matrix' last chunk (requests past the end re-read it: never used)
    const uint4 *ptr[LPW];
    int step[LPW], dsts[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int p = wave * LPW + i;
        if (p < KC * 8) {
            const int kc = p >> 3, mg = p & 7;
            ptr[i] = xp + ((size_t)(k0 + kc) * 8 + mg) * 64; step[i] = KC * 8 * 64; dsts[i] = kc * 8 + mg;
        } else {
            const int q = p - KC * 8, t = q / KC, kc = q % KC;
            const int nt = min(nt0 + t, a.n_tiles - 1);
            ptr[i] = a.wp + ((size_t)nt * k_steps + k0 + kc) * 64; step[i] = KC * 64; dsts[i] = KC * 8 + kc * WNT + t;
        }
    }
    int next_c = 0;                                     // chunk the streams point at
    auto fetch = [&](u32x4_t (&g)[LPW]) {               // global -> registers, then the streams move on
#pragma unroll
        for (int i = 0; i < LPW; ++i) g[i] = *(const u32x4_t *)(ptr[i] + lane);
        ++next_c;
        const int adv = -(int)(k0 + next_c * KC < k_steps);     // all ones while the next chunk exists
#pragma unroll
        for (int i = 0; i < LPW; ++i) ptr[i] += step[i] & adv;
    };
    auto stash = [&](int c, const u32x4_t (&g)[LPW]) {  // registers -> the LDS stage of chunk c
        u32x4_t *st = lds + (c & 1) * STAGE_U4;
#pragma unroll
        for (int i = 0; i < LPW; ++i) st[dsts[i] * 64 + lane] = g[i];
    };
    const int wm = wave >> 1, wn = wave & 1;
    f32x16_t acc[4][TW];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < TW; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    u32x4_t a0[4], b0[TW], a1[4], b1[TW];
    auto load_ops = [&](int c, int kc, u32x4_t (&x)[4], u32x4_t (&wt)[TW]) {
        const u32x4_t *st = lds + (c & 1) * STAGE_U4;
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = st[(kc * 8 + 4 * wm + i) * 64 + lane];
#pragma unroll
        for (int j = 0; j < TW; ++j) wt[j] = st[(KC * 8 + kc * WNT + wn * TW + j) * 64 + lane];
    };
    auto mfmas = [&](int ks, u32x4_t (&x)[4], u32x4_t (&wt)[TW]) {
        if (TAIL && ks >= k1) {                         // the chunk that pads an odd count: multiply by zero
#pragma unroll
            for (int i = 0; i < 4; ++i) x[i] = u32x4_t{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < TW; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, wt[j]),
                                                                    __builtin_bit_cast(bf16x8_t, x[i]), acc[i][j], 0, 0, 0);
    };
    // one chunk: g holds chunk c + 1 on entry and chunk c + 3 on exit
    auto chunk = [&](int c, u32x4_t (&g)[LPW]) {
        // k-step 0: its products; between them the operand reads of k-step 1, chunk c + 1 into its stage (which nobody
        // reads any more: everyone has passed barrier c) and the requests for chunk c + 3
        load_ops(c, 1, a1, b1);
        stash(c + 1, g);
        fetch(g);
        mfmas(k0 + c * KC, a0, b0);
#pragma unroll
        for (int r = 0; r < 4 + TW; ++r) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one matrix instruction,
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);      // one LDS read
        }
#pragma unroll
        for (int r = 0; r < LPW; ++r) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);      // one LDS write,
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);      // one global load
        }
        __builtin_amdgcn_sched_barrier(0);
        // this wavefront has read all it needs of chunk c and has written its share of chunk c + 1.  A bare barrier:
        // the LDS traffic it orders has been waited for explicitly, and no global store is outstanding in the loop.
        __builtin_amdgcn_s_waitcnt(HX_WIDE_LGKM0);
        __builtin_amdgcn_s_barrier();                  // barrier c + 1
        asm volatile("" ::: "memory");
        load_ops(c + 1, 0, a0, b0);
        mfmas(k0 + c * KC + 1, a1, b1);
#pragma unroll
        for (int r = 0; r < 4 + TW; ++r) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 1);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    u32x4_t g0[LPW], g1[LPW];
    fetch(g0);                                          // chunk 0
    fetch(g1);                                          // chunk 1
    stash(0, g0);
    fetch(g0);                                          // chunk 2
    __builtin_amdgcn_s_waitcnt(HX_WIDE_LGKM0);
    __builtin_amdgcn_s_barrier();                      // barrier 0: chunk 0 is in its stage
    asm volatile("" ::: "memory");
    load_ops(0, 0, a0, b0);
    for (int c = 0; c < n_chunks; c += 2) {             // an odd count runs one chunk more, with zero operands (TAIL)
        chunk(c, g1);
        chunk(c + 1, g0);
    }

    // accumulator register r of lane l: batch row m = 32*(4*wm + i) + l%32, column n = 32*nt + 8*(r/4) + 4*(l/32) + r%4
    const int hl = lane >> 5, ml = lane & 31;
    if (EPI == HX_EPI_PARTIAL) {
        float *y = a.y0 + ((size_t)b * a.block_stride) / 4 + (size_t)blockIdx.y * 256 * a.N;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = 32 * (4 * wm + i) + ml;
#pragma unroll
            for (int j = 0; j < TW; ++j) {
                const int nt = nt0 + wn * TW + j;
                if (nt < a.n_tiles) {
#pragma unroll
                    for (int j4 = 0; j4 < 4; ++j4) {
                        const int n = 32 * nt + 8 * j4 + 4 * hl;
                        if (n < a.N)
                            *(f32x4_t *)(y + (size_t)m * a.N + n) =
                                f32x4_t{acc[i][j][4 * j4], acc[i][j][4 * j4 + 1], acc[i][j][4 * j4 + 2], acc[i][j][4 * j4 + 3]};
                    }
                }
            }
        }
    } else {
        // SiLU(gate) * up: rows 0..15 of a tile are gate columns 16*nt + p, rows 16..31 the matching up columns
        uint16_t *mp = a.mp0 + ((size_t)b * a.block_stride) / 2;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = 32 * (4 * wm + i) + ml;
#pragma unroll
            for (int j = 0; j < TW; ++j) {
                const int nt = nt0 + wn * TW + j;
                if (nt < a.n_tiles) {
#pragma unroll
                    for (int j4 = 0; j4 < 2; ++j4) {
                        float v[4];
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const float gt = acc[i][j][4 * j4 + q], up = acc[i][j][8 + 4 * j4 + q];
                            v[q] = (gt / (1.0f + expf(-gt))) * up;
                        }
                        uint2 pk;
                        pk.x = hx_cvt_pk_bf16(v[0], v[1]);
                        pk.y = hx_cvt_pk_bf16(v[2], v[3]);
                        *(uint2 *)(mp + hx_xp_index(m, 16 * nt + 8 * j4 + 4 * hl, 8)) = pk;
                    }
                }
            }
        }
    }
}

template <int WNT, int EPI, bool TAIL>
int launch_wide(dim3 grid, hipStream_t st, const WideArgs &a) {
    static std::once_flag once;
    static hipError_t configured = hipSuccess;
    std::call_once(once, [] {
        configured = hipFuncSetAttribute((const void *)gemm_wide_kernel<WNT, EPI, TAIL>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         wide_lds_bytes(WNT));
    });
    if (configured != hipSuccess) return hx_fail(HX_E_HIP, "hipFuncSetAttribute: %s", hipGetErrorString(configured));
    hipLaunchKernelGGL((gemm_wide_kernel<WNT, EPI, TAIL>), grid, dim3(256), wide_lds_bytes(WNT), st, a);
    return HX_OK;
}

template <int WNT>
int launch_wide_epi(int epilogue, bool tail, dim3 grid, hipStream_t st, const WideArgs &a) {
    if (epilogue == HX_EPI_PARTIAL) return tail ? launch_wide<WNT, HX_EPI_PARTIAL, true>(grid, st, a) : launch_wide<WNT, HX_EPI_PARTIAL, false>(grid, st, a);
    return tail ? launch_wide<WNT, HX_EPI_SWIGLU, true>(grid, st, a) : launch_wide<WNT, HX_EPI_SWIGLU, false>(grid, st, a);
}

}  // namespace

// Tiles per workgroup and, for a product whose consumer sums partials, K-splits: the time of the busiest compute unit
// (rounds x tiles per workgroup x k-steps per split), with a charge per extra split for writing and re-reading its
// partial (measured: a 256 x N fp32 partial per row block is about 4 % of a 3584-deep product) and one per narrower
// tile (it draws more bytes per flop).  Splits hold whole chunks.
hx_wide_plan hx_plan_wide(const hx_matrix *m, int row_blocks, bool partial) {
    const int cus = hx_device_cus();
    hx_wide_plan best{8, 1};
    double best_cost = 1e300;
    for (int wnt : {8, 6}) {
        const int NB = (m->n_tiles + wnt - 1) / wnt;
        for (int s = 1; s <= (partial ? HX_MAX_SPLITS : 1); ++s) {
            if (s > 1 && m->k_steps / s < 32) break;
            const int wgs = NB * row_blocks * s;
            const int rounds = (wgs + cus - 1) / cus;
            const int sps = ((m->k_steps + s - 1) / s + 1) & ~1;
            const double cost = (double)rounds * wnt * sps * (1.0 + 0.04 * (s - 1)) * (1.0 + 0.03 * (8 - wnt));
            if (cost < best_cost - 1e-9) { best_cost = cost; best.wnt = wnt; best.splits = s; }
        }
    }
    return best;
}

// One wide product over `row_blocks` blocks of 256 rows.  xp_off / y_off / mp_off: byte offsets of the packed input,
// the fp32 output ([splits][256][N]) and the SiLU*mul output inside each block's workspace; ws0 = block 0's
// workspace, block_stride bytes between blocks.
int hx_launch_gemm_wide(const hx_engine *e, const hx_matrix *m, int row_blocks, char *ws0, size_t block_stride, size_t xp_off,
                        int epilogue, size_t y_off, size_t mp_off, hx_wide_plan plan, hipStream_t st) {
    int splits = plan.splits;
    const int wnt = plan.wnt;
    if (wnt != 8 && wnt != 6) return hx_fail(HX_E_RANGE, "%d tiles per workgroup: no such wide product", wnt);
    if (m->k_steps % WIDE_KC) return hx_fail(HX_E_SHAPE, "wide products need K to be a multiple of 32, not %d", m->k_steps * 16);
    if (epilogue != HX_EPI_PARTIAL && epilogue != HX_EPI_SWIGLU) return hx_fail(HX_E_RANGE, "epilogue %d has no wide product", epilogue);
    if (epilogue == HX_EPI_SWIGLU) splits = 1;
    if (block_stride % 16) return hx_fail(HX_E_RANGE, "block stride %zu is not a multiple of 16", block_stride);
    WideArgs a;
    a.wp = (const uint4 *)(e->weights + m->offset);
    a.k_steps = m->k_steps; a.n_tiles = m->n_tiles; a.N = m->N;
    a.xp0 = ws0 + xp_off; a.block_stride = block_stride; a.R = row_blocks;
    a.y0 = (float *)(ws0 + y_off);
    a.mp0 = (uint16_t *)(ws0 + mp_off);
    a.steps_per_split = ((m->k_steps + splits - 1) / splits + 1) & ~1;
    const int NB = (m->n_tiles + wnt - 1) / wnt;
    dim3 grid(((NB + 7) / 8) * 8 * row_blocks, splits);
    bool tail = false;                                  // some split has an odd number of chunks
    for (int s = 0; s < splits; ++s) {
        const int k0 = s * a.steps_per_split, k1 = std::min(m->k_steps, k0 + a.steps_per_split);
        if (k1 <= k0) return hx_fail(HX_E_RANGE, "%d splits leave split %d of %d k-steps empty", splits, s, m->k_steps);
        if (((k1 - k0) / WIDE_KC) & 1) tail = true;
    }
    const int rc = wnt == 8 ? launch_wide_epi<8>(epilogue, tail, grid, st, a) : launch_wide_epi<6>(epilogue, tail, grid, st, a);
    if (rc) return rc;
    HX_CHECK_LAUNCH("gemm_wide");
    return HX_OK;
}
