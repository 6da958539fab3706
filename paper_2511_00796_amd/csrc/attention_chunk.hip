// Attention for prompt rows (prefill_chunk): consecutive rows of one sequence share one K/V stream.
//
// A row of a prompt chunk is one token; row r of a sequence attends the keys [0, T_r), T_r = T_{r-1} + 1.  The decode
// kernel would stream the whole prefix once per row.  Here up to min(HX_CHUNK_ROWS, 64 / G) consecutive rows of one
// sequence form a GROUP whose (row, query head) pairs are the columns of the score product -- at most 64 columns = 4
// column blocks of 16 (8 rows for G <= 8, 4 rows for G = 16) -- so a K/V tile is loaded once per group and multiplied
// up to four times:
//     S^T[token, (row, g)] = K_tile . q[row, g]          4 x v_mfma_f32_16x16x32_bf16 per column block
//     O^T[d, (row, g)]    += V_tile^T . P^T               as in the decode kernel, per column block
// The causal mask is per column: keys >= T_row are dropped (only the last tiles of a group differ between its rows).
// The schedule is the decode step's with "sequence" replaced by "group" (tiles of a group = ceil(T_last / 16) per KV
// head, cut into equal runs over all wavefronts); a partial result holds 4 column blocks.  Groups are found on the
// device from the arguments: row r continues row r - 1 if seq_lens[r] = seq_lens[r - 1] + 1 and its block-table row
// repeats that of r - 1 over the blocks r - 1 uses; the group reads the cache through the table row of its last row.
#include "hx_internal.h"

#define HX_NEG_BIG (-1.0e30f)
#define HX_CHUNK_CB 4
#define HX_CHUNK_MIN_TILES 2
#define HX_CHUNK_MAX_MIN_TILES 8

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

// ---- which rows continue their predecessor ------------------------------------------------------------------------
// grid = n_rows, 64 threads.  cont[r] = 1 iff row r is the next position of the sequence of row r - 1.
__global__ __launch_bounds__(64) void chunk_rows_kernel(const int32_t *__restrict__ seq_lens,
                                                        const int32_t *__restrict__ table, int max_blocks,
                                                        int32_t *__restrict__ cont) {
    const int r = blockIdx.x, lane = threadIdx.x;
    if (r == 0) {
        if (lane == 0) cont[0] = 0;
        return;
    }
    const int Tp = seq_lens[r - 1], T = seq_lens[r];
    const int nb = (Tp + 15) >> 4;
    bool ok = (T == Tp + 1) && nb <= max_blocks;
    const int32_t *a = table + (size_t)(r - 1) * max_blocks, *b = table + (size_t)r * max_blocks;
    for (int i = lane; i < nb && ok; i += 64) ok = a[i] == b[i];
    const bool all = __all(ok);
    if (lane == 0) cont[r] = all ? 1 : 0;
}

__device__ __forceinline__ void scan_sum_256(int32_t *scan, int r) {     // inclusive, in place; ends synchronised
    for (int off = 1; off < 256; off <<= 1) {
        const int v = (r >= off) ? scan[r - off] : 0;
        __syncthreads();
        scan[r] += v;
        __syncthreads();
    }
}

// ---- groups and their schedule --------------------------------------------------------------------------------------
// One workgroup of 256 threads (thread = row, later thread = group).  Writes the decode schedule's arrays with groups
// in place of sequences -- pre[g] = blocks of the groups before g, lens[g] = keys of the group's last row, sched =
// {tiles per wavefront, tiles} -- plus ginfo[g] = first row | rows << 16 and rgrp[r] = group | index in group << 16.
__global__ __launch_bounds__(256) void chunk_setup_kernel(int n_rows, int n_kv, int n_waves, int group_rows,
                                                          const int32_t *__restrict__ seq_lens,
                                                          const int32_t *__restrict__ cont, int32_t *__restrict__ pre,
                                                          int32_t *__restrict__ lens, int32_t *__restrict__ sched,
                                                          int32_t *__restrict__ ginfo, int32_t *__restrict__ rgrp) {
    __shared__ int32_t scan[256], gfirst[256], gcount[256];
    const int r = threadIdx.x;
    const bool valid = r < n_rows;
    // first row of the run of consecutive rows that holds r: inclusive max-scan of (r starts a run ? r : -1)
    scan[r] = (!valid || r == 0 || !cont[r]) ? r : -1;
    gfirst[r] = 0;
    gcount[r] = 0;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        const int v = (r >= off) ? scan[r - off] : -1;
        __syncthreads();
        scan[r] = max(scan[r], v);
        __syncthreads();
    }
    const int local = (r - scan[r]) % group_rows;             // index of r in its group
    const int gstart = (valid && local == 0) ? 1 : 0;
    __syncthreads();
    scan[r] = gstart;
    __syncthreads();
    scan_sum_256(scan, r);
    const int gid = scan[r] - 1;
    const int n_groups = scan[255];
    __syncthreads();
    if (valid) {
        if (gstart) gfirst[gid] = r;
        atomicMax(&gcount[gid], local + 1);
        rgrp[r] = gid | (local << 16);
    }
    __syncthreads();
    int first = 0, cnt = 0, T = 0;
    if (r < n_groups) {
        first = gfirst[r];
        cnt = gcount[r];
        T = seq_lens[first + cnt - 1];
    }
    const int nb = (T + 15) >> 4;
    scan[r] = nb;
    __syncthreads();
    scan_sum_256(scan, r);
    const int total = scan[255];
    pre[r] = scan[r] - nb;                                    // r >= n_groups: nb = 0, so pre[r] = total
    lens[r] = T;
    ginfo[r] = first | (cnt << 16);
    for (int i = 256 + r; i < HX_PREFIX_LEN; i += 256) pre[i] = total;
    if (r == 0) {
        // A run costs its wavefront a query staging and a partial result of up to 33 KiB, so short schedules are cut
        // into fewer, longer runs than there are wavefronts (the surplus wavefronts exit at once): about 512 runs
        // (two per compute unit) of 2 to 8 tiles.  Measured at the 7B shape, 256 rows of one prompt: 8 is best from
        // position 1024 on, 2-4 for the first chunk of a prompt.
        const long long nt = (long long)total * n_kv;
        const int s_small = min(max((int)((nt + 511) / 512), HX_CHUNK_MIN_TILES), HX_CHUNK_MAX_MIN_TILES);
        sched[0] = max((int)((nt + n_waves - 1) / n_waves), s_small);
        sched[1] = (int)nt;
    }
}

// ---- the attention kernel ---------------------------------------------------------------------------------------------
// loads of 1 KiB per tile: D/16 for bf16 elements, D/32 for the 8-bit cache (tile layouts: hx_internal.h)
template <int NL>
__device__ __forceinline__ void load_tile_c(u32x4_t (&r)[NL], const char *tile, int lane) {
    const u32x4_t *p = (const u32x4_t *)tile + lane;
#pragma unroll
    for (int i = 0; i < NL; ++i) r[i] = __builtin_nontemporal_load(p + i * 64);
}

template <int D>
struct ChunkState {
    f32x4_t o[HX_CHUNK_CB][D / 16];
    float m[HX_CHUNK_CB];   // running maximum per column (same in the 4 lane groups)
    float l[HX_CHUNK_CB];   // this lane's share of the running sum
};

// Streams `nblk` (1..128) consecutive blocks of one (group, KV head) pair: tokens [t0, t0 + 16 nblk).  tcol[cb] = keys
// the lane's column of block cb attends (0 for an unused column), t_first / t_last = the smallest and largest of the
// used ones, n_cb = column blocks in use.  qs = this wavefront's staged query operands.  Ring and load stream as in
// the decode kernel.
template <int D, int PF, bool FP8>
__device__ __forceinline__ void stream_tiles_chunk(ChunkState<D> &st, const u32x4_t *qs, const char *pool_layer,
                                                   size_t block_bytes, size_t head_off, const char *qtile,
                                                   int32_t blk_lo, int32_t blk_hi, int nblk, int t0,
                                                   const int (&tcol)[HX_CHUNK_CB], int n_cb, int t_first, int t_last,
                                                   float scale_log2e, int lane) {
    const int qd = lane >> 4;
    const int t_end = t0 + nblk * 16;
    const int t1v = min(t_last, t_end);                       // V rows from here on may hold anything
    const int t_clean = min(t_first, t_end);                  // tiles that end at or before this need no mask
    int t1c[HX_CHUNK_CB];
#pragma unroll
    for (int cb = 0; cb < HX_CHUNK_CB; ++cb) t1c[cb] = min(tcol[cb], t_end);
    constexpr int NL = FP8 ? D / 32 : D / 16;
    u32x4_t ring[PF][NL];
#pragma unroll
    for (int s = 0; s < PF; ++s)
#pragma unroll
        for (int i = 0; i < NL; ++i) ring[s][i] = u32x4_t{0u, 0u, 0u, 0u};

    const int n_rounds = (nblk + PF - 1) / PF + 1;
    for (int rd = 0; rd < n_rounds; ++rd) {
#pragma unroll
        for (int s = 0; s < PF; ++s) {
            const int i = (rd - 1) * PF + s;                   // tile of this iteration; < 0 while the ring fills
            const int tok0 = t0 + i * 16 + qd * 4;             // this lane's 4 tokens
            const bool edge = i < 0 || t0 + (i + 1) * 16 > t_clean;   // wave-uniform
            // operands of this tile: K steps kop[kk], V steps vv[q] (x, y: rows d < 16 of the step; z, w: rows d >= 16).
            // V of positions that do not exist must not reach the product (it may hold anything, also NaN).
            u32x4_t kop[D / 32], vv[D / 32];
            const bool ragged = i < 0 || t0 + (i + 1) * 16 > t1v;     // wave-uniform
            const int valid = (i < 0) ? 0 : (t1v - tok0);
            if (FP8) {
                // 8-bit cache: bytes -> bf16 (exact), once per tile for all column blocks
                const uint32_t keep = (!ragged || valid >= 4) ? 0xffffffffu : (valid <= 0 ? 0u : ((1u << (8 * valid)) - 1u));
#pragma unroll
                for (int kk = 0; kk < D / 32; ++kk) {
                    const u32x4_t raw = ring[s][kk >> 1];
                    const uint2 a = hx_e4m3x4_to_bf16x4((kk & 1) ? raw.z : raw.x);
                    const uint2 b = hx_e4m3x4_to_bf16x4((kk & 1) ? raw.w : raw.y);
                    kop[kk] = u32x4_t{a.x, a.y, b.x, b.y};
                }
#pragma unroll
                for (int q = 0; q < D / 32; ++q) {
                    const u32x4_t raw = ring[s][D / 64 + (q >> 1)];
                    const uint2 lo = hx_e4m3x4_to_bf16x4(((q & 1) ? raw.z : raw.x) & keep);
                    const uint2 hi = hx_e4m3x4_to_bf16x4(((q & 1) ? raw.w : raw.y) & keep);
                    vv[q] = u32x4_t{lo.x, lo.y, hi.x, hi.y};
                }
            } else {
#pragma unroll
                for (int kk = 0; kk < D / 32; ++kk) kop[kk] = ring[s][kk];
#pragma unroll
                for (int q = 0; q < D / 32; ++q) vv[q] = ring[s][D / 32 + q];
                if (ragged) {
                    const uint32_t m01 = valid >= 2 ? 0xffffffffu : (valid == 1 ? 0x0000ffffu : 0u);
                    const uint32_t m23 = valid >= 4 ? 0xffffffffu : (valid == 3 ? 0x0000ffffu : 0u);
#pragma unroll
                    for (int q = 0; q < D / 32; ++q) { vv[q].x &= m01; vv[q].y &= m23; vv[q].z &= m01; vv[q].w &= m23; }
                }
            }
#pragma unroll
            for (int cb = 0; cb < HX_CHUNK_CB; ++cb) {
                if (cb >= n_cb) continue;                     // wave-uniform: column blocks no row of the group uses
                u32x4_t qb[D / 32];                            // this column block's query operands, from LDS
#pragma unroll
                for (int kk = 0; kk < D / 32; ++kk) qb[kk] = qs[(cb * (D / 32) + kk) * 64 + lane];
                f32x4_t sc = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < D / 32; ++kk)
                    sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kop[kk]),
                                                                 __builtin_bit_cast(bf16x8_t, qb[kk]), sc, 0, 0, 0);
                hx_hold_operands(qb, kop, sc);                 // short-lived operands outlive the products that read them
                float s4[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) s4[r] = sc[r] * scale_log2e;
                if (edge) {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (!(tok0 + r >= t0 && tok0 + r < t1c[cb])) s4[r] = -INFINITY;
                }
                float mx = fmaxf(fmaxf(s4[0], s4[1]), fmaxf(s4[2], s4[3]));
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(st.m[cb], mx);
                const float alpha = __builtin_amdgcn_exp2f(st.m[cb] - m_new);
                float p[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) p[r] = __builtin_amdgcn_exp2f(s4[r] - m_new);
                st.l[cb] = st.l[cb] * alpha + ((p[0] + p[1]) + (p[2] + p[3]));
                // the accumulators are rescaled only when some column's maximum moved (else alpha is exactly 1 in
                // every lane): after the first tiles of a group that is rare, and it saves a multiply per register
                if (__builtin_amdgcn_ballot_w64(m_new != st.m[cb]) != 0ull) {
#pragma unroll
                    for (int nn = 0; nn < D / 16; ++nn) st.o[cb][nn] *= alpha;
                }
                st.m[cb] = m_new;
                // probabilities as a high + low bf16 pair, as in the decode kernel
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
                    st.o[cb][2 * q] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, lo), pop_hi, st.o[cb][2 * q], 0, 0, 0);
                    st.o[cb][2 * q + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, hi), pop_hi, st.o[cb][2 * q + 1], 0, 0, 0);
                }
#pragma unroll
                for (int q = 0; q < D / 32; ++q) {
                    uint2 lo = make_uint2(vv[q].x, vv[q].y), hi = make_uint2(vv[q].z, vv[q].w);
                    st.o[cb][2 * q] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, lo), pop_lo, st.o[cb][2 * q], 0, 0, 0);
                    st.o[cb][2 * q + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, hi), pop_lo, st.o[cb][2 * q + 1], 0, 0, 0);
                }
            }
            if (FP8) hx_hold_operands(vv);                     // converted operands outlive the products that read them
            // the slot is free: request tile i + PF into it (or the query once the run is exhausted)
            const int nx = i + PF;
            const int32_t blk = (nx < 64) ? __builtin_amdgcn_readlane(blk_lo, nx & 63) : __builtin_amdgcn_readlane(blk_hi, nx & 63);
            const char *src = (nx < nblk) ? pool_layer + (size_t)blk * block_bytes + head_off : qtile;
            load_tile_c<NL>(ring[s], src, lane);
        }
    }
}

// grid = wavefronts of the schedule, one wavefront per workgroup, at most 256 registers so that two wavefronts share a
// SIMD and cover each other's latencies.  Partial result of run w and pair p = (group, KV
// head): slot w + p, column block cb at sub-slot 4 * slot + cb: part_ml [sub][max 16 | sum 16], part_o [sub][16][D].
template <int D, int PF, bool FP8>
__global__ __launch_bounds__(64, 2) void attn_chunk_kernel(const char *__restrict__ pool_layer, size_t block_bytes,
                                                        const uint16_t *__restrict__ qp,
                                                        const int32_t *__restrict__ table, int max_blocks,
                                                        const int32_t *__restrict__ pre,
                                                        const int32_t *__restrict__ lens,
                                                        const int32_t *__restrict__ sched,
                                                        const int32_t *__restrict__ ginfo, int n_kv, int G,
                                                        float scale_log2e, float *__restrict__ part_ml,
                                                        float *__restrict__ part_o, size_t block_stride,
                                                        size_t table_block_stride) {
    // query operands of the 4 column blocks; every lane reads back only what it wrote itself
    __shared__ u32x4_t qs[HX_CHUNK_CB * (D / 32) * 64];
    const int w = blockIdx.x;
    const int lane = threadIdx.x;
    if (blockIdx.y) {               // further row blocks of a wide prompt call: each with its own schedule, queries and
        const size_t off = (size_t)blockIdx.y * block_stride;      // partial results, block_stride bytes apart
        qp = (const uint16_t *)((const char *)qp + off);
        pre = (const int32_t *)((const char *)pre + off);
        lens = (const int32_t *)((const char *)lens + off);
        sched = (const int32_t *)((const char *)sched + off);
        ginfo = (const int32_t *)((const char *)ginfo + off);
        part_ml = (float *)((char *)part_ml + off);
        part_o = (float *)((char *)part_o + off);
        table += (size_t)blockIdx.y * table_block_stride;
    }
    const int S = sched[0], Nt = sched[1];
    int f = w * S;
    const int f1 = min(Nt, f + S);
    if (f >= f1) return;
    const int g16 = lane & 15, qd = lane >> 4;

    int32_t pr[HX_PREFIX_LEN / 64];                      // the block prefix sits in registers: lane l holds pre[l + 64 i]
#pragma unroll
    for (int i = 0; i < HX_PREFIX_LEN / 64; ++i) pr[i] = pre[lane + 64 * i];
    auto pick = [&](const int32_t *regs, int n, int idx) -> int32_t {   // regs[idx / 64] of lane idx % 64
        int32_t v = 0;
#pragma unroll
        for (int i = 0; i < HX_PREFIX_LEN / 64; ++i)
            if (i < n && (idx >> 6) == i) v = __builtin_amdgcn_readlane(regs[i], idx & 63);
        return v;
    };

    while (f < f1) {                                     // one iteration per (group, KV head) pair touched
        int cnt_le = 0;
#pragma unroll
        for (int i = 0; i < HX_PREFIX_LEN / 64; ++i) cnt_le += __popcll(__ballot((long long)pr[i] * n_kv <= (long long)f));
        const int gi = __builtin_amdgcn_readfirstlane(cnt_le) - 1;
        const int pb = pick(pr, HX_PREFIX_LEN / 64, gi);
        const int T = lens[gi];                          // keys of the group's last row
        const int info = ginfo[gi];
        const int first = info & 0xffff, rows = info >> 16;
        const int nblk_g = (T + 15) >> 4;
        const int local = f - pb * n_kv;
        const int kvh = local / nblk_g;
        const int blk0 = local - kvh * nblk_g;
        const int n = min(f1 - f, nblk_g - blk0);        // tiles of this pair in this run
        const size_t head_off = (size_t)kvh * 2 * (16 * D * (FP8 ? 1 : 2));   // K | V tiles of one head
        const int trow = first + rows - 1;               // the group reads the cache through its last row's table
        const int n_cb = (rows * G + 15) >> 4;           // column blocks in use

        // stage the query operands: column c = 16 cb + lane % 16 is (row c / G of the group, head c % G)
        const char *qtile = (const char *)(qp + ((size_t)first * n_kv + kvh) * (D / 32) * 512);
        int tcol[HX_CHUNK_CB];
#pragma unroll
        for (int cb = 0; cb < HX_CHUNK_CB; ++cb) {
            const int c = cb * 16 + g16;
            const int rl = c / G, gq = c - rl * G;
            const bool used = rl < rows;
            tcol[cb] = used ? T - (rows - 1 - rl) : 0;
            const uint4 *q4 = (const uint4 *)(qp + ((size_t)(first + (used ? rl : 0)) * n_kv + kvh) * (D / 32) * 512) + (qd * 16 + gq);
#pragma unroll
            for (int kk = 0; kk < D / 32; ++kk) {
                const uint4 v = q4[kk * 64];
                qs[(cb * (D / 32) + kk) * 64 + lane] = used ? u32x4_t{v.x, v.y, v.z, v.w} : u32x4_t{0u, 0u, 0u, 0u};
            }
        }
        ChunkState<D> st;
#pragma unroll
        for (int cb = 0; cb < HX_CHUNK_CB; ++cb) {
#pragma unroll
            for (int nn = 0; nn < D / 16; ++nn) st.o[cb][nn] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            st.m[cb] = HX_NEG_BIG;
            st.l[cb] = 0.f;
        }

        for (int done = 0; done < n; done += 128) {      // at most 128 block ids fit the two id registers
            const int nsub = min(128, n - done);
            const int32_t *row = table + (size_t)trow * max_blocks + blk0 + done;
            int32_t blk_lo = (lane < nsub) ? row[lane] : 0;
            int32_t blk_hi = (64 + lane < nsub) ? row[64 + lane] : 0;
            const int t0 = (blk0 + done) * 16;
            asm volatile("" : "+v"(blk_lo), "+v"(blk_hi));
            stream_tiles_chunk<D, PF, FP8>(st, qs, pool_layer, block_bytes, head_off, qtile, blk_lo, blk_hi, nsub, t0, tcol,
                                      n_cb, T - (rows - 1), T, scale_log2e, lane);
        }

        const size_t slot = (size_t)w + (size_t)gi * n_kv + kvh;
#pragma unroll
        for (int cb = 0; cb < HX_CHUNK_CB; ++cb) {
            if (cb >= n_cb) continue;                    // never read by the combine
            float l = st.l[cb];
            l += __shfl_xor(l, 16);
            l += __shfl_xor(l, 32);
            const size_t sub = slot * HX_CHUNK_CB + cb;
            if (qd == 0) {
                part_ml[sub * 32 + g16] = st.m[cb];
                part_ml[sub * 32 + 16 + g16] = l;
            }
            float *po = part_o + (sub * 16 + g16) * D;
#pragma unroll
            for (int nn = 0; nn < D / 16; ++nn) *(f32x4_t *)(po + nn * 16 + qd * 4) = st.o[cb][nn];
        }
        f += n;
    }
}

// ---- combine ------------------------------------------------------------------------------------------------------------
// As the decode step's combine, with the column of (row, head) looked up through the row's group.
template <int D>
__global__ __launch_bounds__(256) void attn_chunk_combine_kernel(int n_rows, int n_q, int n_kv, int G,
                                                                 const int32_t *__restrict__ pre,
                                                                 const int32_t *__restrict__ lens,
                                                                 const int32_t *__restrict__ sched,
                                                                 const int32_t *__restrict__ rgrp,
                                                                 const float *__restrict__ part_ml,
                                                                 const float *__restrict__ part_o,
                                                                 uint16_t *__restrict__ ap, int m_groups,
                                                                 float *__restrict__ attn_f32, size_t block_stride) {
    const int bh = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (bh >= n_rows * n_q) return;
    if (blockIdx.y) {               // further row blocks of a wide prompt call: same layout, block_stride bytes apart
        const size_t off = (size_t)blockIdx.y * block_stride;
        pre = (const int32_t *)((const char *)pre + off);
        lens = (const int32_t *)((const char *)lens + off);
        sched = (const int32_t *)((const char *)sched + off);
        rgrp = (const int32_t *)((const char *)rgrp + off);
        part_ml = (const float *)((const char *)part_ml + off);
        part_o = (const float *)((const char *)part_o + off);
        ap = (uint16_t *)((char *)ap + off);
        if (attn_f32) attn_f32 += (size_t)blockIdx.y * n_rows * n_q * D;
    }
    const int lane = threadIdx.x & 63, d8 = lane & 15, ph = lane >> 4;
    const bool has_d = d8 < D / 8;
    const int b = bh / n_q, h = bh % n_q;
    const int kvh = h / G, g = h % G;
    const int info = rgrp[b];
    const int gi = info & 0xffff, rl = info >> 16;
    const int c = rl * G + g, cb = c >> 4, col = c & 15;
    const int S = sched[0];
    const int nblk_g = (lens[gi] + 15) >> 4;
    const int start = pre[gi] * n_kv + kvh * nblk_g;     // tiles of this pair: [start, start + nblk_g)
    const int pair = gi * n_kv + kvh;
    const int s0 = start / S + pair, s1 = (start + nblk_g - 1) / S + pair;   // its slots, inclusive
    float M = HX_NEG_BIG;
    for (int it = s0 + ph; it <= s1; it += 4) M = fmaxf(M, part_ml[((size_t)it * HX_CHUNK_CB + cb) * 32 + col]);
    M = fmaxf(M, __shfl_xor(M, 16));
    M = fmaxf(M, __shfl_xor(M, 32));
    float den = 0.f;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    for (int it = s0 + ph; it <= s1; it += 4) {
        const size_t sub = (size_t)it * HX_CHUNK_CB + cb;
        const float w = __builtin_amdgcn_exp2f(part_ml[sub * 32 + col] - M);
        den += w * part_ml[sub * 32 + 16 + col];
        if (has_d) {
            const float *po = part_o + (sub * 16 + col) * D + d8 * 8;
            const f32x4_t a = *(const f32x4_t *)po, c4 = *(const f32x4_t *)(po + 4);
            acc[0] += w * a[0]; acc[1] += w * a[1]; acc[2] += w * a[2]; acc[3] += w * a[3];
            acc[4] += w * c4[0]; acc[5] += w * c4[1]; acc[6] += w * c4[2]; acc[7] += w * c4[3];
        }
    }
    den += __shfl_xor(den, 16);
    den += __shfl_xor(den, 32);
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
    uint4 pk;
    pk.x = hx_cvt_pk_bf16(acc[0], acc[1]); pk.y = hx_cvt_pk_bf16(acc[2], acc[3]);
    pk.z = hx_cvt_pk_bf16(acc[4], acc[5]); pk.w = hx_cvt_pk_bf16(acc[6], acc[7]);
    *(uint4 *)(ap + hx_xp_index(b, h * D + d8 * 8, m_groups)) = pk;
}

// ---- launchers ------------------------------------------------------------------------------------------------------------
int hx_launch_chunk_setup(const hx_engine *e, int n_rows, const int32_t *seq_lens, const int32_t *table, int max_blocks,
                          hipStream_t st) {
    char *ws = e->ws;
    int32_t *cont = (int32_t *)(ws + e->map.chunk_cont);
    hipLaunchKernelGGL(chunk_rows_kernel, dim3(n_rows), dim3(64), 0, st, seq_lens, table, max_blocks, cont);
    HX_CHECK_LAUNCH("chunk_rows");
    hipLaunchKernelGGL(chunk_setup_kernel, dim3(1), dim3(256), 0, st, n_rows, e->cfg.n_kv_heads, e->attn_waves, e->chunk_rows, seq_lens,
                       (const int32_t *)cont, (int32_t *)(ws + e->map.pre), (int32_t *)(ws + e->map.lens),
                       (int32_t *)(ws + e->map.sched), (int32_t *)(ws + e->map.chunk_ginfo),
                       (int32_t *)(ws + e->map.chunk_rgrp));
    HX_CHECK_LAUNCH("chunk_setup");
    return HX_OK;
}

int hx_launch_chunk_attention(const hx_engine *e, const hx_kv *kv, int layer, const int32_t *table, int max_blocks,
                              hipStream_t st, int blocks, size_t block_stride, int rows_per_block) {
    const char *pool_layer = kv->pool + (size_t)layer * kv->layer_bytes;
    char *ws = e->ws;
    const float scale_log2e = (float)(1.4426950408889634 / sqrt((double)e->D));
    dim3 grid(e->attn_waves, blocks), block(64);
#define HX_CHUNK_ARGS                                                                                            \
    pool_layer, kv->block_bytes, (const uint16_t *)(ws + e->map.qp), table, max_blocks,                          \
        (const int32_t *)(ws + e->map.pre), (const int32_t *)(ws + e->map.lens),                                 \
        (const int32_t *)(ws + e->map.sched), (const int32_t *)(ws + e->map.chunk_ginfo), e->cfg.n_kv_heads,     \
        e->G, scale_log2e, (float *)(ws + e->map.chunk_part_ml), (float *)(ws + e->map.chunk_part_o), block_stride,   \
        (size_t)rows_per_block * max_blocks
    if (kv->fp8) {
        if (e->D == 128) hipLaunchKernelGGL((attn_chunk_kernel<128, 2, true>), grid, block, 0, st, HX_CHUNK_ARGS);
        else             hipLaunchKernelGGL((attn_chunk_kernel<64, 3, true>), grid, block, 0, st, HX_CHUNK_ARGS);
    } else {
        if (e->D == 128) hipLaunchKernelGGL((attn_chunk_kernel<128, 2, false>), grid, block, 0, st, HX_CHUNK_ARGS);
        else             hipLaunchKernelGGL((attn_chunk_kernel<64, 3, false>), grid, block, 0, st, HX_CHUNK_ARGS);
    }
#undef HX_CHUNK_ARGS
    HX_CHECK_LAUNCH("attn_chunk");
    return HX_OK;
}

int hx_launch_chunk_combine(const hx_engine *e, int n_rows, float *attn_f32_out, hipStream_t st, int blocks, size_t block_stride) {
    char *ws = e->ws;
    const int n_kv = e->cfg.n_kv_heads, n_q = e->cfg.n_q_heads;
    const int m_groups = hx_m_groups(n_rows);
    dim3 cgrid((n_rows * n_q + 3) / 4, blocks), cblock(256);
#define HX_CCOMB_ARGS                                                                                            \
    n_rows, n_q, n_kv, e->G, (const int32_t *)(ws + e->map.pre), (const int32_t *)(ws + e->map.lens),            \
        (const int32_t *)(ws + e->map.sched), (const int32_t *)(ws + e->map.chunk_rgrp),                         \
        (const float *)(ws + e->map.chunk_part_ml), (const float *)(ws + e->map.chunk_part_o),                   \
        (uint16_t *)(ws + e->map.ap), m_groups, attn_f32_out, block_stride
    if (e->D == 128) hipLaunchKernelGGL((attn_chunk_combine_kernel<128>), cgrid, cblock, 0, st, HX_CCOMB_ARGS);
    else             hipLaunchKernelGGL((attn_chunk_combine_kernel<64>), cgrid, cblock, 0, st, HX_CCOMB_ARGS);
#undef HX_CCOMB_ARGS
    HX_CHECK_LAUNCH("attn_chunk_combine");
    return HX_OK;
}
