// The decode step's split-K attention over an 8-bit (E4M3) cache.
//
// Schedule, work decomposition, products and partial results are those of attention.hip; only the tiles differ.  A
// tile (K and V of 16 tokens of one KV head) holds 1-byte elements in the operand order of the bf16 tile with the bytes
// of two operand steps side by side (hx_ktile8_index / hx_vtile8_index), so it is half as many 1-KiB loads.  Each
// operand is converted to bf16 in registers right before its product -- exactly, every E4M3 value is a bf16 value --
// and from there on the arithmetic is the bf16 kernel's.  The ring holds the raw bytes (4 tiles of 4 KiB in flight at
// head size 128: with the converted operands held in registers past their products, a deeper ring costs more in
// register pressure than it gains; measured 194 us per launch at depth 4, 207 at depth 6, 214 at depth 7).
#include "hx_internal.h"

#define HX_NEG_BIG (-1.0e30f)

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// One tile in registers: D/64 loads of K then D/64 loads of V, 16 bytes per lane each.
template <int D>
__device__ __forceinline__ void load_tile8(u32x4_t (&r)[D / 32], const char *tile, int lane) {
    const u32x4_t *p = (const u32x4_t *)tile + lane;
#pragma unroll
    for (int i = 0; i < D / 32; ++i) r[i] = __builtin_nontemporal_load(p + i * 64);
}

template <int D>
struct AttnState8 {
    f32x4_t o[D / 16];
    float m;   // running maximum of the scaled scores (base-2 domain), same in the 4 lane groups
    float l;   // this lane's share of the running sum
};

// Streams `nblk` (1..128) consecutive blocks of one pair: tokens [t0, t1), t0 a multiple of 16.  As stream_tiles of
// the bf16 kernel: no prologue, no conditional load, PF tiles in flight, requests past the end go to the packed query.
template <int D, int PF>
__device__ __forceinline__ void stream_tiles8(AttnState8<D> &st, const bf16x8_t (&qop)[D / 32], const char *pool_layer,
                                              size_t block_bytes, size_t head_off, const char *qtile, int32_t blk_lo,
                                              int32_t blk_hi, int nblk, int t0, int t1, float scale_log2e, int lane) {
    const int qd = lane >> 4;
    u32x4_t ring[PF][D / 32];
#pragma unroll
    for (int s = 0; s < PF; ++s)
#pragma unroll
        for (int i = 0; i < D / 32; ++i) ring[s][i] = u32x4_t{0u, 0u, 0u, 0u};

    const int n_rounds = (nblk + PF - 1) / PF + 1;
    for (int rd = 0; rd < n_rounds; ++rd) {
#pragma unroll
        for (int s = 0; s < PF; ++s) {
            const int i = (rd - 1) * PF + s;                   // tile of this iteration; < 0 while the ring fills
            const int tok0 = t0 + i * 16 + qd * 4;             // this lane's 4 tokens
            // scores of 16 tokens x 16 query heads; operand step kk = dwords 2 (kk % 2), 2 (kk % 2) + 1 of load kk / 2
            u32x4_t kop[D / 32];
            f32x4_t sc = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < D / 32; ++kk) {
                const u32x4_t raw = ring[s][kk >> 1];
                const uint2 a = hx_e4m3x4_to_bf16x4((kk & 1) ? raw.z : raw.x);
                const uint2 b = hx_e4m3x4_to_bf16x4((kk & 1) ? raw.w : raw.y);
                kop[kk] = u32x4_t{a.x, a.y, b.x, b.y};
                sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kop[kk]), qop[kk], sc, 0, 0, 0);
            }
            hx_hold_operands(kop, sc);                         // converted operands outlive the products that read them
            float s4[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) s4[r] = (tok0 + r >= t0 && tok0 + r < t1) ? sc[r] * scale_log2e : -INFINITY;
            // V: operand step q = dwords 2 (q % 2) (rows d < 16 of the step) and 2 (q % 2) + 1 (rows d >= 16) of load
            // D/64 + q / 2; a dword holds this lane's 4 tokens, one byte each.  Bytes of positions that do not
            // exist may hold anything (also NaN codes): they are cleared before the conversion.
            uint32_t vlo[D / 32], vhi[D / 32];
#pragma unroll
            for (int q = 0; q < D / 32; ++q) {
                const u32x4_t raw = ring[s][D / 64 + (q >> 1)];
                vlo[q] = (q & 1) ? raw.z : raw.x;
                vhi[q] = (q & 1) ? raw.w : raw.y;
            }
            if (i < 0 || t0 + (i + 1) * 16 > t1) {             // wave-uniform: a tile with missing tokens
                const int valid = (i < 0) ? 0 : (t1 - tok0);
                const uint32_t keep = valid >= 4 ? 0xffffffffu : (valid <= 0 ? 0u : ((1u << (8 * valid)) - 1u));
#pragma unroll
                for (int q = 0; q < D / 32; ++q) { vlo[q] &= keep; vhi[q] &= keep; }
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
            // probabilities as a high + low bf16 pair, as in the bf16 kernel
            uint2 ph, pl;
            ph.x = hx_cvt_pk_bf16(p[0], p[1]);
            ph.y = hx_cvt_pk_bf16(p[2], p[3]);
            pl.x = hx_cvt_pk_bf16(p[0] - __uint_as_float(ph.x << 16), p[1] - __uint_as_float(ph.x & 0xffff0000u));
            pl.y = hx_cvt_pk_bf16(p[2] - __uint_as_float(ph.y << 16), p[3] - __uint_as_float(ph.y & 0xffff0000u));
            const s16x4_t pop_hi = __builtin_bit_cast(s16x4_t, ph);
            const s16x4_t pop_lo = __builtin_bit_cast(s16x4_t, pl);
            u32x4_t vop[D / 32];                               // x, y: rows d < 16 of the step; z, w: rows d >= 16
#pragma unroll
            for (int q = 0; q < D / 32; ++q) {
                const uint2 lo2 = hx_e4m3x4_to_bf16x4(vlo[q]), hi2 = hx_e4m3x4_to_bf16x4(vhi[q]);
                vop[q] = u32x4_t{lo2.x, lo2.y, hi2.x, hi2.y};
                const s16x4_t lo = __builtin_bit_cast(s16x4_t, make_uint2(vop[q].x, vop[q].y));
                const s16x4_t hi = __builtin_bit_cast(s16x4_t, make_uint2(vop[q].z, vop[q].w));
                st.o[2 * q] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(lo, pop_hi, st.o[2 * q], 0, 0, 0);
                st.o[2 * q + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(hi, pop_hi, st.o[2 * q + 1], 0, 0, 0);
                st.o[2 * q] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(lo, pop_lo, st.o[2 * q], 0, 0, 0);
                st.o[2 * q + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(hi, pop_lo, st.o[2 * q + 1], 0, 0, 0);
            }
            hx_hold_operands(vop);
            // the slot is free: request tile i + PF into it (or the query once the run is exhausted)
            const int nx = i + PF;
            const int32_t blk = (nx < 64) ? __builtin_amdgcn_readlane(blk_lo, nx & 63) : __builtin_amdgcn_readlane(blk_hi, nx & 63);
            const char *src = (nx < nblk) ? pool_layer + (size_t)blk * block_bytes + head_off : qtile;
            load_tile8<D>(ring[s], src, lane);
        }
    }
}

template <int D, int PF>
__global__ __launch_bounds__(64) void attn_splitk_fp8_kernel(const char *__restrict__ pool_layer, size_t block_bytes,
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
        const size_t head_off = (size_t)kvh * 2 * (16 * D);   // K | V of one head: 2 tiles of 16 x D bytes

        const char *qtile = (const char *)(qp + ((size_t)b * n_kv + kvh) * (D / 32) * 512);
        bf16x8_t qop[D / 32];
        {
            const uint4 *q4 = (const uint4 *)qtile + lane;
#pragma unroll
            for (int kk = 0; kk < D / 32; ++kk) qop[kk] = __builtin_bit_cast(bf16x8_t, q4[kk * 64]);
        }
        AttnState8<D> st;
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
            // everything requested so far has landed before the tile loop is entered (its waits count loads)
#pragma unroll
            for (int kk = 0; kk < D / 32; ++kk) asm volatile("" : "+v"(qop[kk]));
            asm volatile("" : "+v"(blk_lo), "+v"(blk_hi));
            stream_tiles8<D, PF>(st, qop, pool_layer, block_bytes, head_off, qtile, blk_lo, blk_hi, nsub, t0,
                                 min(T, t0 + nsub * 16), scale_log2e, lane);
        }

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

int hx_launch_attention_fp8(const hx_engine *e, const hx_kv *kv, int layer, const int32_t *table, int max_blocks,
                            hipStream_t st, const hx_attn_bufs *bufs) {
    const char *pool_layer = kv->pool + (size_t)layer * kv->layer_bytes;
    const hx_attn_bufs own = hx_attn_bufs_of(e);
    const hx_attn_bufs &a = bufs ? *bufs : own;
    const float scale_log2e = (float)(1.4426950408889634 / sqrt((double)e->D));
    dim3 grid(e->attn_waves), block(64);
#define HX_ATTN8_ARGS                                                                                            \
    pool_layer, kv->block_bytes, (const uint16_t *)a.qp, table, max_blocks, (const int32_t *)a.pre,              \
        (const int32_t *)a.lens, (const int32_t *)a.sched, e->cfg.n_kv_heads, e->G, scale_log2e, a.part_ml, a.part_o
    // ring depths: 128: see the header; 64: depth 6 (every depth from 2 to 12 is right since the operand hold is
    // ordered behind the products; the tests cover long runs)
    if (e->D == 128) hipLaunchKernelGGL((attn_splitk_fp8_kernel<128, 4>), grid, block, 0, st, HX_ATTN8_ARGS);
    else             hipLaunchKernelGGL((attn_splitk_fp8_kernel<64, 6>), grid, block, 0, st, HX_ATTN8_ARGS);
#undef HX_ATTN8_ARGS
    HX_CHECK_LAUNCH("attn_splitk_fp8");
    return HX_OK;
}
