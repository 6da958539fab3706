// Split-K flash-decoding attention over the paged cache: the per-step schedule that cuts the ragged
// batch into equal shares of K/V tiles, the attention kernel, and the combine kernel that merges the
// partial results.
//
// Work decomposition ("stream-K").  A tile is the K and V of 16 tokens of one KV head.  All tiles of the
// batch are lined up in (sequence, KV head, block) order and cut into W equal runs of S = ceil(Nt / W)
// tiles, one run per wavefront, W = 8 per compute unit.
// Every wavefront therefore streams the same
// number of bytes whatever the length mix, all of them are resident at once and finish together, and a
// run is long (about 1 MiB at the 7B shape), so start-up latency is paid once.  A run that crosses from
// one (sequence, KV head) pair into the next emits one partial result per pair it touches; run w and pair
// p write slot w + p, which is unique and makes the slots of a pair contiguous (w0 + p .. w1 + p).
//
// One wavefront serves all G query heads of its KV head at once, so every K and V byte is read exactly once:
//     S^T[token, g] = K_tile[token, :] . q[g, :]        v_mfma_f32_16x16x32_bf16 (A = K tile, B = packed q)
//     O^T[d, g]    += V_tile^T[d, token] . P^T[token, g] v_mfma_f32_16x16x16_bf16 (A = V tile, B = P)
// The accumulator layout of the first product (lane = query head g, 4 registers = 4 tokens) is
// exactly the B-operand layout of the second, so the probabilities never cross lanes; only the
// running maximum is exchanged between the four 16-lane groups with two wavefront shuffles per
// tile, and the running sum is reduced once at the end.  K/V tiles are stored in operand order
// in the pool, so they go from HBM to registers with contiguous 1-KiB loads and need no LDS.
#include "hx_internal.h"

#define HX_NEG_BIG (-1.0e30f)

// ---- per-step setup: schedule + RoPE angles ----------------------------------------------------------------
// block 0: sched[0] = S (tiles per wavefront), sched[1] = Nt (tiles in all), pre[b] = blocks of the sequences
// before b (pre[b] = total for b >= batch, HX_PREFIX_LEN entries), lens[b] = seq_lens[b] (0 for b >= batch).
// blocks 1..batch: cos/sin of pos * theta^(-2i/D), evaluated in double, stored fp32; and the physical block that
// holds the new position (one look-up per step instead of one per layer in the append kernel).
__global__ __launch_bounds__(256) void step_setup_kernel(int batch, int n_kv, int n_waves,
                                                         const int32_t *__restrict__ positions,
                                                         const int32_t *__restrict__ seq_lens,
                                                         const int32_t *__restrict__ table, int max_blocks,
                                                         int32_t *__restrict__ pre, int32_t *__restrict__ lens,
                                                         int32_t *__restrict__ sched, int32_t *__restrict__ blk_new,
                                                         float *__restrict__ cs, int half, double theta, int max_batch) {
    if (blockIdx.x == 0) {
        if (seq_lens == nullptr) return;
        __shared__ int32_t scan[256];
        const int b = threadIdx.x;
        const int T = b < batch ? seq_lens[b] : 0;
        const int cnt = (T + 15) >> 4;
        scan[b] = cnt;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {       // inclusive Hillis-Steele scan
            int v = (b >= off) ? scan[b - off] : 0;
            __syncthreads();
            scan[b] += v;
            __syncthreads();
        }
        const int total = scan[255];
        pre[b] = scan[b] - cnt;                          // b >= batch: cnt = 0, so pre[b] = total
        lens[b] = T;
        for (int i = 256 + b; i < HX_PREFIX_LEN; i += 256) pre[i] = total;
        if (b == 0) {
            const long long nt = (long long)total * n_kv;
            sched[0] = (int)((nt + n_waves - 1) / n_waves);
            sched[1] = (int)nt;
        }
    } else if (positions != nullptr) {
        int b = blockIdx.x - 1;
        if (threadIdx.x == 0 && table != nullptr) blk_new[b] = table[(size_t)b * max_blocks + (positions[b] >> 4)];
        double pos = (double)positions[b];
        for (int i = threadIdx.x; i < half; i += blockDim.x) {
            double ang = pos * pow(theta, -(double)i / (double)half);
            cs[(size_t)b * half + i] = (float)cos(ang);
            cs[(size_t)max_batch * half + (size_t)b * half + i] = (float)sin(ang);
        }
    }
}

hx_attn_bufs hx_attn_bufs_of(const hx_engine *e) {
    char *ws = e->ws;
    return hx_attn_bufs{(uint16_t *)(ws + e->map.qp), (int32_t *)(ws + e->map.pre), (int32_t *)(ws + e->map.lens),
                        (int32_t *)(ws + e->map.sched), (float *)(ws + e->map.part_ml), (float *)(ws + e->map.part_o),
                        (uint16_t *)(ws + e->map.ap)};
}

int hx_launch_step_setup(const hx_engine *e, int batch, const int32_t *positions, const int32_t *seq_lens,
                         const int32_t *table, int max_blocks, hipStream_t st, const hx_attn_bufs *bufs) {
    char *ws = e->ws;
    const hx_attn_bufs own = hx_attn_bufs_of(e);
    if (bufs && positions) return hx_fail(HX_E_RANGE, "the schedule-only set-up takes no positions");
    const hx_attn_bufs &a = bufs ? *bufs : own;
    // without positions only block 0 runs: the per-row blocks would write the engine's RoPE tables
    hipLaunchKernelGGL(step_setup_kernel, dim3(positions ? batch + 1 : 1), dim3(256), 0, st, batch, e->cfg.n_kv_heads, e->attn_waves,
                       positions, seq_lens, table, max_blocks, a.pre, a.lens, a.sched, (int32_t *)(ws + e->map.blk_new),
                       (float *)(ws + e->map.cs), e->D / 2, (double)e->cfg.rope_theta, e->cfg.max_batch);
    HX_CHECK_LAUNCH("step_setup");
    return HX_OK;
}

// ---- split-K attention -----------------------------------------------------------------------------------
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// One K/V tile in registers: D/32 K operands then D/32 V operands, 16 bytes per lane each.
// K/V are read exactly once per step: non-temporal loads keep them from displacing reusable lines.
template <int D>
__device__ __forceinline__ void load_tile(u32x4_t (&r)[D / 16], const char *tile, int lane) {
    const u32x4_t *p = (const u32x4_t *)tile + lane;
#pragma unroll
    for (int i = 0; i < D / 16; ++i) r[i] = __builtin_nontemporal_load(p + i * 64);
}

// State of one (sequence, KV head) pair while its tiles stream through.
template <int D>
struct AttnState {
    f32x4_t o[D / 16];
    float m;   // running maximum of the scaled scores (base-2 domain), same in the 4 lane groups
    float l;   // this lane's share of the running sum
};

// Streams `nblk` (1..128) consecutive blocks of one pair: tokens [t0, t1), t0 a multiple of 16.  blk_lo / blk_hi
// hold the physical ids: lane i of blk_lo = block i, lane i of blk_hi = block 64 + i.
// PF = tiles in flight (register ring).  The loop has no prologue and no conditional load: it starts PF tiles
// early (those iterations see only masked-out tokens and zero operands) and every iteration requests the tile
// PF ahead into the slot it has just finished with; past the end of the run the request goes to the packed
// query (small, cache-resident, finite), so the load stream is unconditional and the compiler keeps exactly
// PF - 1 tiles outstanding behind every wait.
template <int D, int PF>
__device__ __forceinline__ void stream_tiles(AttnState<D> &st, const bf16x8_t (&qop)[D / 32], const char *pool_layer,
                                             size_t block_bytes, size_t head_off, const char *qtile, int32_t blk_lo,
                                             int32_t blk_hi, int nblk, int t0, int t1, float scale_log2e, int lane) {
    const int qd = lane >> 4;
    u32x4_t ring[PF][D / 16];
#pragma unroll
    for (int s = 0; s < PF; ++s)
#pragma unroll
        for (int i = 0; i < D / 16; ++i) ring[s][i] = u32x4_t{0u, 0u, 0u, 0u};

    const int n_rounds = (nblk + PF - 1) / PF + 1;
    for (int rd = 0; rd < n_rounds; ++rd) {
#pragma unroll
        for (int s = 0; s < PF; ++s) {
            const int i = (rd - 1) * PF + s;                   // tile of this iteration; < 0 while the ring fills
            const int tok0 = t0 + i * 16 + qd * 4;             // this lane's 4 tokens
            // scores of 16 tokens x 16 query heads
            f32x4_t sc = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < D / 32; ++kk)
                sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ring[s][kk]), qop[kk], sc, 0, 0, 0);
            {
                // The K operands of the slot die with these products, so the compiler may hand their registers to the
                // next vector instruction (at head size 64 it did: the mask arithmetic of a ragged tile, a few
                // instructions behind the product that was still to read them).  Keep them live past the products
                // (hx_hold_operands) at both head sizes.
                u32x4_t kheld[D / 32];
#pragma unroll
                for (int kk = 0; kk < D / 32; ++kk) kheld[kk] = ring[s][kk];
                hx_hold_operands(kheld, sc);
            }
            float s4[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) s4[r] = (tok0 + r >= t0 && tok0 + r < t1) ? sc[r] * scale_log2e : -INFINITY;
            // V of positions that do not exist must not reach the product as NaN/Inf
            u32x4_t vv[D / 32];
#pragma unroll
            for (int q = 0; q < D / 32; ++q) vv[q] = ring[s][D / 32 + q];
            if (i < 0 || t0 + (i + 1) * 16 > t1) {             // wave-uniform: a tile with missing tokens
                const int valid = (i < 0) ? 0 : (t1 - tok0);
                const uint32_t m01 = valid >= 2 ? 0xffffffffu : (valid == 1 ? 0x0000ffffu : 0u);
                const uint32_t m23 = valid >= 4 ? 0xffffffffu : (valid == 3 ? 0x0000ffffu : 0u);
#pragma unroll
                for (int q = 0; q < D / 32; ++q) { vv[q].x &= m01; vv[q].y &= m23; vv[q].z &= m01; vv[q].w &= m23; }
            }
            float mx = fmaxf(fmaxf(s4[0], s4[1]), fmaxf(s4[2], s4[3]));
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(st.m, mx);
            const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
            float p[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) p[r] = __builtin_amdgcn_exp2f(s4[r] - m_new);
            st.l = st.l * alpha + ((p[0] + p[1]) + (p[2] + p[3]));
            st.m = m_new;
#pragma unroll
            for (int nn = 0; nn < D / 16; ++nn) st.o[nn] *= alpha;
            // P enters the matrix core as bf16; split it into a high and a low bf16 part so that the
            // product keeps ~16 significant bits of every probability
            uint2 ph, pl;
            ph.x = hx_cvt_pk_bf16(p[0], p[1]);
            ph.y = hx_cvt_pk_bf16(p[2], p[3]);
            pl.x = hx_cvt_pk_bf16(p[0] - __uint_as_float(ph.x << 16), p[1] - __uint_as_float(ph.x & 0xffff0000u));
            pl.y = hx_cvt_pk_bf16(p[2] - __uint_as_float(ph.y << 16), p[3] - __uint_as_float(ph.y & 0xffff0000u));
            const s16x4_t pop_hi = __builtin_bit_cast(s16x4_t, ph);
            const s16x4_t pop_lo = __builtin_bit_cast(s16x4_t, pl);
#pragma unroll
            for (int q = 0; q < D / 32; ++q) {
                uint2 lo = make_uint2(vv[q].x, vv[q].y), hi = make_uint2(vv[q].z, vv[q].w);
                st.o[2 * q] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, lo), pop_hi, st.o[2 * q], 0, 0, 0);
                st.o[2 * q + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, hi), pop_hi, st.o[2 * q + 1], 0, 0, 0);
            }
#pragma unroll
            for (int q = 0; q < D / 32; ++q) {
                uint2 lo = make_uint2(vv[q].x, vv[q].y), hi = make_uint2(vv[q].z, vv[q].w);
                st.o[2 * q] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, lo), pop_lo, st.o[2 * q], 0, 0, 0);
                st.o[2 * q + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, hi), pop_lo, st.o[2 * q + 1], 0, 0, 0);
            }
            // the slot is free: request tile i + PF into it (or the query once the run is exhausted)
            const int nx = i + PF;
            const int32_t blk = (nx < 64) ? __builtin_amdgcn_readlane(blk_lo, nx & 63) : __builtin_amdgcn_readlane(blk_hi, nx & 63);
            const char *src = (nx < nblk) ? pool_layer + (size_t)blk * block_bytes + head_off : qtile;
            load_tile<D>(ring[s], src, lane);
        }
    }
}

template <int D, int PF>
__global__ __launch_bounds__(64) void attn_splitk_kernel(const char *__restrict__ pool_layer, size_t block_bytes,
                                                         const uint16_t *__restrict__ qp,
                                                         const int32_t *__restrict__ table, int max_blocks,
                                                         const int32_t *__restrict__ pre,
                                                         const int32_t *__restrict__ lens,
                                                         const int32_t *__restrict__ sched, int n_kv, int G,
                                                         float scale_log2e, float *__restrict__ part_ml,
                                                         float *__restrict__ part_o) {
    const int w = blockIdx.x;
    const int lane = threadIdx.x;
    const int S = sched[0], Nt = sched[1];
    int f = w * S;
    const int f1 = min(Nt, f + S);
    if (f >= f1) return;
    const int g = lane & 15, qd = lane >> 4;

    // the whole schedule sits in registers: lane l holds pre[l + 64 i] and lens[l + 64 i]
    int32_t pr[HX_PREFIX_LEN / 64], ln[4];
#pragma unroll
    for (int i = 0; i < HX_PREFIX_LEN / 64; ++i) pr[i] = pre[lane + 64 * i];
#pragma unroll
    for (int i = 0; i < 4; ++i) ln[i] = lens[lane + 64 * i];
    auto pick = [&](const int32_t *regs, int n, int idx) -> int32_t {   // regs[idx / 64] of lane idx % 64
        int32_t v = 0;
#pragma unroll
        for (int i = 0; i < HX_PREFIX_LEN / 64; ++i)
            if (i < n && (idx >> 6) == i) v = __builtin_amdgcn_readlane(regs[i], idx & 63);
        return v;
    };

    while (f < f1) {                                     // one iteration per (sequence, KV head) pair touched
        // sequence of tile f: the last b with pre[b] * n_kv <= f
        int cnt = 0;
#pragma unroll
        for (int i = 0; i < HX_PREFIX_LEN / 64; ++i) cnt += __popcll(__ballot((long long)pr[i] * n_kv <= (long long)f));
        const int b = __builtin_amdgcn_readfirstlane(cnt) - 1;
        const int pb = pick(pr, HX_PREFIX_LEN / 64, b);
        const int T = pick(ln, 4, b);
        const int nblk_b = (T + 15) >> 4;
        const int local = f - pb * n_kv;
        const int kvh = local / nblk_b;
        const int blk0 = local - kvh * nblk_b;
        const int n = min(f1 - f, nblk_b - blk0);        // tiles of this pair in this run
        const size_t head_off = (size_t)kvh * 2 * (16 * D * 2);

        // packed query: B operand of the score product
        const char *qtile = (const char *)(qp + ((size_t)b * n_kv + kvh) * (D / 32) * 512);
        bf16x8_t qop[D / 32];
        {
            const uint4 *q4 = (const uint4 *)qtile + lane;
#pragma unroll
            for (int kk = 0; kk < D / 32; ++kk) qop[kk] = __builtin_bit_cast(bf16x8_t, q4[kk * 64]);
        }
        AttnState<D> st;
#pragma unroll
        for (int nn = 0; nn < D / 16; ++nn) st.o[nn] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        st.m = HX_NEG_BIG;
        st.l = 0.f;

        for (int done = 0; done < n; done += 128) {      // at most 128 block ids fit the two id registers
            const int nsub = min(128, n - done);
            const int32_t *row = table + (size_t)b * max_blocks + blk0 + done;
            int32_t blk_lo = (lane < nsub) ? row[lane] : 0;
            int32_t blk_hi = (64 + lane < nsub) ? row[64 + lane] : 0;
            const int t0 = (blk0 + done) * 16;
            // Everything requested so far must have landed before the tile loop is entered: its waits count
            // outstanding loads, and a load still in flight on entry would make every wait in the loop drain
            // the tile ring to match.
#pragma unroll
            for (int kk = 0; kk < D / 32; ++kk) asm volatile("" : "+v"(qop[kk]));
            asm volatile("" : "+v"(blk_lo), "+v"(blk_hi));
            stream_tiles<D, PF>(st, qop, pool_layer, block_bytes, head_off, qtile, blk_lo, blk_hi, nsub, t0,
                                min(T, t0 + nsub * 16), scale_log2e, lane);
        }

        // total of the running sum over the four lane groups
        float l = st.l;
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        const size_t slot = (size_t)w + (size_t)b * n_kv + kvh;
        if (qd == 0) {
            part_ml[slot * 32 + g] = st.m;
            part_ml[slot * 32 + 16 + g] = l;
        }
        if (g < G) {
            float *po = part_o + (slot * G + g) * D;
#pragma unroll
            for (int nn = 0; nn < D / 16; ++nn) *(f32x4_t *)(po + nn * 16 + qd * 4) = st.o[nn];
        }
        f += n;
    }
}

// ---- combine ---------------------------------------------------------------------------------------------
// o = sum_c 2^(m_c - M) o_c / sum_c 2^(m_c - M) l_c over the partial results of the pair (sequence, KV head):
// the runs w0..w1 that cover its tiles, found from the schedule, in slots w + pair.
// One wavefront per (sequence, query head).  Maximum and denominator: lane i takes partials i, i+64, ..., reduced by
// a fixed shuffle tree.  Numerator: lane = (phase 0..3, d8 0..15); phase p takes partials p, p+4, ... in order, then
// the four phases are summed by a fixed shuffle tree (deterministic).  Lanes of phase 0
// write the bf16-rounded result into the packed activation buffer of the output projection and, if asked,
// the unrounded fp32 values.  D = 64 uses lanes d8 < 8 only.
template <int D>
__global__ __launch_bounds__(256) void attn_combine_kernel(int batch, int n_q, int n_kv, int G,
                                                           const int32_t *__restrict__ pre,
                                                           const int32_t *__restrict__ lens,
                                                           const int32_t *__restrict__ sched,
                                                           const float *__restrict__ part_ml,
                                                           const float *__restrict__ part_o,
                                                           uint16_t *__restrict__ ap, int m_groups,
                                                           float *__restrict__ attn_f32) {
    const int bh = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (bh >= batch * n_q) return;
    const int lane = threadIdx.x & 63, d8 = lane & 15, ph = lane >> 4;
    const bool has_d = d8 < D / 8;
    const int b = bh / n_q, h = bh % n_q;
    const int kvh = h / G, g = h % G;
    const int S = sched[0];
    const int nblk_b = (lens[b] + 15) >> 4;
    const int start = pre[b] * n_kv + kvh * nblk_b;      // tiles of this pair: [start, start + nblk_b)
    const int pair = b * n_kv + kvh;
    const int s0 = start / S + pair, s1 = (start + nblk_b - 1) / S + pair;   // its slots, inclusive
    // More than 8 partials per pair (a short batch of long sequences has a hundred): maximum and denominator take one
    // partial per lane, 64 at a time; the weighted sum of the o vectors four partials per 16-lane group and iteration,
    // all requested before the first is used.
    const int n = s1 - s0 + 1;
    float M = HX_NEG_BIG, den = 0.f;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    if (n <= 8) {                   // the usual case (a few partials per pair): each 16-lane group takes every fourth
        for (int it = s0 + ph; it <= s1; it += 4) M = fmaxf(M, part_ml[(size_t)it * 32 + g]);
        M = fmaxf(M, __shfl_xor(M, 16));
        M = fmaxf(M, __shfl_xor(M, 32));
        for (int it = s0 + ph; it <= s1; it += 4) {
            const float w = __builtin_amdgcn_exp2f(part_ml[(size_t)it * 32 + g] - M);
            den += w * part_ml[(size_t)it * 32 + 16 + g];
            if (has_d) {
                const float *po = part_o + ((size_t)it * G + g) * D + d8 * 8;
                const f32x4_t a = *(const f32x4_t *)po, c = *(const f32x4_t *)(po + 4);
                acc[0] += w * a[0]; acc[1] += w * a[1]; acc[2] += w * a[2]; acc[3] += w * a[3];
                acc[4] += w * c[0]; acc[5] += w * c[1]; acc[6] += w * c[2]; acc[7] += w * c[3];
            }
        }
        den += __shfl_xor(den, 16);
        den += __shfl_xor(den, 32);
    } else {
        for (int i = lane; i < n; i += 64) M = fmaxf(M, part_ml[(size_t)(s0 + i) * 32 + g]);
#pragma unroll
        for (int sh = 1; sh < 64; sh <<= 1) M = fmaxf(M, __shfl_xor(M, sh));
        for (int i = lane; i < n; i += 64) {
            const float *ml = part_ml + (size_t)(s0 + i) * 32;
            den += __builtin_amdgcn_exp2f(ml[g] - M) * ml[16 + g];
        }
#pragma unroll
        for (int sh = 1; sh < 64; sh <<= 1) den += __shfl_xor(den, sh);
        for (int it = s0 + ph; it <= s1; it += 16) {
            float w[4];
            f32x4_t a[4], c[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int iu = min(it + 4 * u, s1);                   // past the end: re-read the last, weight 0
                w[u] = part_ml[(size_t)iu * 32 + g];
                if (has_d) {
                    const float *po = part_o + ((size_t)iu * G + g) * D + d8 * 8;
                    a[u] = *(const f32x4_t *)po; c[u] = *(const f32x4_t *)(po + 4);
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float wu = it + 4 * u <= s1 ? __builtin_amdgcn_exp2f(w[u] - M) : 0.f;
                if (has_d) {
                    acc[0] += wu * a[u][0]; acc[1] += wu * a[u][1]; acc[2] += wu * a[u][2]; acc[3] += wu * a[u][3];
                    acc[4] += wu * c[u][0]; acc[5] += wu * c[u][1]; acc[6] += wu * c[u][2]; acc[7] += wu * c[u][3];
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        acc[j] += __shfl_xor(acc[j], 16);
        acc[j] += __shfl_xor(acc[j], 32);
    }
    if (ph != 0 || !has_d) return;
    const float inv = 1.0f / den;
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] *= inv;
    if (attn_f32) {
        float *dst = attn_f32 + ((size_t)b * n_q + h) * D + d8 * 8;
        *(f32x4_t *)dst = f32x4_t{acc[0], acc[1], acc[2], acc[3]};
        *(f32x4_t *)(dst + 4) = f32x4_t{acc[4], acc[5], acc[6], acc[7]};
    }
    if (ap == nullptr) return;
    uint4 pk;
    pk.x = hx_cvt_pk_bf16(acc[0], acc[1]); pk.y = hx_cvt_pk_bf16(acc[2], acc[3]);
    pk.z = hx_cvt_pk_bf16(acc[4], acc[5]); pk.w = hx_cvt_pk_bf16(acc[6], acc[7]);
    *(uint4 *)(ap + hx_xp_index(b, h * D + d8 * 8, m_groups)) = pk;
}

int hx_launch_attention(const hx_engine *e, const hx_kv *kv, int layer, int batch, const int32_t *seq_lens,
                        const int32_t *table, int max_blocks, hipStream_t st, const hx_attn_bufs *bufs) {
    const char *pool_layer = kv->pool + (size_t)layer * kv->layer_bytes;
    const hx_attn_bufs own = hx_attn_bufs_of(e);
    const hx_attn_bufs &a = bufs ? *bufs : own;
    const int n_kv = e->cfg.n_kv_heads;
    const float scale_log2e = (float)(1.4426950408889634 / sqrt((double)e->D));
    (void)seq_lens; (void)batch;
    dim3 grid(e->attn_waves), block(64);
#define HX_ATTN_ARGS                                                                                             \
    pool_layer, kv->block_bytes, (const uint16_t *)a.qp, table, max_blocks, (const int32_t *)a.pre,              \
        (const int32_t *)a.lens, (const int32_t *)a.sched, n_kv, e->G, scale_log2e, a.part_ml, a.part_o
    if (e->D == 128) hipLaunchKernelGGL((attn_splitk_kernel<128, 3>), grid, block, 0, st, HX_ATTN_ARGS);
    else             hipLaunchKernelGGL((attn_splitk_kernel<64, 4>), grid, block, 0, st, HX_ATTN_ARGS);
#undef HX_ATTN_ARGS
    HX_CHECK_LAUNCH("attn_splitk");
    return HX_OK;
}

int hx_launch_combine(const hx_engine *e, int batch, float *attn_f32_out, hipStream_t st, const hx_attn_bufs *bufs) {
    const hx_attn_bufs own = hx_attn_bufs_of(e);
    const hx_attn_bufs &a = bufs ? *bufs : own;
    const int n_kv = e->cfg.n_kv_heads, n_q = e->cfg.n_q_heads;
    const int m_groups = hx_m_groups(batch);
    dim3 cgrid((batch * n_q + 3) / 4), cblock(256);
#define HX_COMB_ARGS                                                                                             \
    batch, n_q, n_kv, e->G, (const int32_t *)a.pre, (const int32_t *)a.lens, (const int32_t *)a.sched,            \
        (const float *)a.part_ml, (const float *)a.part_o, a.ap, m_groups, attn_f32_out
    if (e->D == 128) hipLaunchKernelGGL((attn_combine_kernel<128>), cgrid, cblock, 0, st, HX_COMB_ARGS);
    else             hipLaunchKernelGGL((attn_combine_kernel<64>), cgrid, cblock, 0, st, HX_COMB_ARGS);
#undef HX_COMB_ARGS
    HX_CHECK_LAUNCH("attn_combine");
    return HX_OK;
}
