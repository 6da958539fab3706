// Nucleus (top-p) sampling of one step's logits (Holtzman et al., ICLR 2020), after temperature scaling:
// keep the most probable entries whose mass reaches top_p -- all entries with z_i >= tau, tau the largest
// threshold for which mass{z_i >= tau} >= top_p * total, so entries equal to the last kept one are kept --
// and draw from the kept set by Gumbel-max with the noise of the temperature sampler.
//
// One workgroup per row.  tau is found by a radix select on the 32-bit order-preserving key of z, most
// significant digit first (11, 11, 10 bits): each pass builds a histogram of probability MASS per digit among the
// entries that match the digits chosen so far, and walks it from the largest z down to the digit where the
// running mass reaches the target.  Mass is 40-bit fixed point, w_i = floor(exp(z_i - max z) * 2^40), added with
// integer LDS atomics: the sums are exact, so the kept set does not depend on the order of the additions and the
// kernel is deterministic.  A last pass draws among the kept entries.  Four reads of the row (from the memory-side
// cache: the LM head has just written it).
#include "hx_internal.h"

#define HX_NUC_THREADS 1024
#define HX_NUC_BINS 2048
#define HX_NUC_SCALE 1099511627776.0f   // 2^40

// ascending key order = descending z; -0 and +0 share a key
__device__ __forceinline__ uint32_t nucleus_key(float z) {
    const uint32_t b = __float_as_uint(z + 0.0f);
    return ~(b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u));
}

__device__ __forceinline__ void load_group(const float *__restrict__ x, int V, int q, bool vec, float (&v)[4]) {
    if (vec) {
        const f32x4_t t = *(const f32x4_t *)(x + 4 * (size_t)q);
        v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = (4 * q + i < V) ? x[4 * (size_t)q + i] : 0.f;
    }
}

__global__ __launch_bounds__(HX_NUC_THREADS) void nucleus_kernel(
    const float *__restrict__ logits, int V, const float *__restrict__ tile_max, int n_tiles,
    const int32_t *__restrict__ positions, const int32_t *__restrict__ row_ids, float inv_t, float top_p, uint32_t key0,
    uint32_t key1, int32_t *__restrict__ tok_out, float *__restrict__ lp_out, int32_t *__restrict__ size_out) {
    __shared__ unsigned long long hist[HX_NUC_BINS];
    __shared__ unsigned long long scan[HX_NUC_THREADS];
    __shared__ float redf[HX_NUC_THREADS / 64];
    __shared__ int32_t redi[HX_NUC_THREADS / 64], redc[HX_NUC_THREADS / 64];
    __shared__ float redz[HX_NUC_THREADS / 64];
    __shared__ unsigned long long sh_before, sh_mass;
    __shared__ uint32_t sh_digit;

    const int m = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *x = logits + (size_t)m * V;
    const bool vec = (V & 3) == 0;                // rows then start on 16-byte boundaries
    const int n_groups = (V + 3) >> 2;

    // max z from the LM head's per-tile maxima of the raw logits (scaling by 1/T > 0 is monotone)
    float mx = -INFINITY;
    for (int t = tid; t < n_tiles; t += HX_NUC_THREADS) mx = fmaxf(mx, tile_max[(size_t)m * n_tiles + t]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if (lane == 0) redf[wave] = mx;
    __syncthreads();
    mx = redf[0];
#pragma unroll
    for (int w = 1; w < HX_NUC_THREADS / 64; ++w) mx = fmaxf(mx, redf[w]);
    const float zmax = mx * inv_t;
    __syncthreads();

    uint32_t prefix = 0;                          // digits chosen so far (the high bits of tau's key)
    unsigned long long before = 0, target = 0;    // mass of the entries above the chosen digits; mass to reach
    int shift = 32;
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
        const int bits = pass < 2 ? 11 : 10;
        const int hi_shift = shift;               // entries must match prefix in the bits above hi_shift
        shift -= bits;
        for (int i = tid; i < HX_NUC_BINS; i += HX_NUC_THREADS) hist[i] = 0ull;
        __syncthreads();
        for (int q = tid; q < n_groups; q += HX_NUC_THREADS) {
            float v[4];
            load_group(x, V, q, vec, v);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (4 * q + i >= V) continue;
                const float z = v[i] * inv_t;
                const uint32_t key = nucleus_key(z);
                if (pass == 0 || (key >> hi_shift) == prefix) {
                    const unsigned long long w = (unsigned long long)(expf(z - zmax) * HX_NUC_SCALE);
                    if (w) atomicAdd(&hist[(key >> shift) & ((1u << bits) - 1u)], w);
                }
            }
        }
        __syncthreads();
        // inclusive scan of the bins in key order, two bins per thread
        const unsigned long long h0 = hist[2 * tid], h1 = hist[2 * tid + 1];
        unsigned long long incl = h0 + h1;
        scan[tid] = incl;
        __syncthreads();
#pragma unroll 1
        for (int off = 1; off < HX_NUC_THREADS; off <<= 1) {
            const unsigned long long add = tid >= off ? scan[tid - off] : 0ull;
            __syncthreads();
            incl += add;
            scan[tid] = incl;
            __syncthreads();
        }
        if (pass == 0) {
            // every entry was counted: the total fixes the target, at least one unit and at most everything
            const unsigned long long total = scan[HX_NUC_THREADS - 1];
            const double want = ceil((double)top_p * (double)total);
            target = want < 1.0 ? 1ull : (unsigned long long)want;
            if (target > total) target = total;
        }
        const unsigned long long excl = incl - (h0 + h1);
        if (before + excl < target && target <= before + incl) {       // exactly one thread
            const bool first = before + excl + h0 >= target;
            sh_digit = 2 * tid + (first ? 0 : 1);
            sh_before = before + excl + (first ? 0ull : h0);
            sh_mass = before + excl + h0 + (first ? 0ull : h1);         // through the chosen bin
        }
        __syncthreads();
        prefix = (prefix << bits) | sh_digit;
        before = sh_before;
    }
    const uint32_t key_tau = prefix;
    const unsigned long long mass = sh_mass;      // of all entries with key <= key_tau, i.e. z >= tau

    // the draw: largest z_i - log(-log(u_i)) among the kept entries, smaller index on ties
    const uint32_t row = row_ids ? (uint32_t)row_ids[m] : (uint32_t)m;
    const uint32_t pos = (uint32_t)positions[m];
    float best = -INFINITY, best_z = 0.f;
    int32_t best_i = 0x7fffffff, count = 0;
    for (int q = tid; q < n_groups; q += HX_NUC_THREADS) {
        float v[4];
        load_group(x, V, q, vec, v);
        bool any = false;
        bool keep[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            keep[i] = (4 * q + i < V) && nucleus_key(v[i] * inv_t) <= key_tau;
            any |= keep[i];
        }
        if (!any) continue;
        uint32_t w[4];
        hx_philox4x32_10((uint32_t)q, row, pos, 0x53414D50u, key0, key1, w);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (!keep[i]) continue;
            ++count;
            const float z = v[i] * inv_t;
            const float u = ((float)(w[i] >> 9) + 0.5f) * (1.0f / 8388608.0f);
            const float y = z - logf(-logf(u));
            if (y > best) { best = y; best_i = 4 * q + i; best_z = z; }   // a thread's indices ascend
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float oy = __shfl_xor(best, off), oz = __shfl_xor(best_z, off);
        const int32_t oi = __shfl_xor(best_i, off);
        if (oy > best || (oy == best && oi < best_i)) { best = oy; best_i = oi; best_z = oz; }
        count += __shfl_xor(count, off);
    }
    if (lane == 0) { redf[wave] = best; redi[wave] = best_i; redz[wave] = best_z; redc[wave] = count; }
    __syncthreads();
    if (tid == 0) {
#pragma unroll 1
        for (int w = 1; w < HX_NUC_THREADS / 64; ++w) {
            if (redf[w] > best || (redf[w] == best && redi[w] < best_i)) { best = redf[w]; best_i = redi[w]; best_z = redz[w]; }
            count += redc[w];
        }
        tok_out[m] = best_i;
        lp_out[m] = (float)((double)best_z - ((double)zmax + log((double)mass * (1.0 / 1099511627776.0))));
        if (size_out) size_out[m] = count;
    }
}

int hx_launch_nucleus(const hx_engine *e, int batch, const float *logits, const hx_sample_params *sample,
                      int32_t *tokens_out, float *logprobs_out, hipStream_t st) {
    hipLaunchKernelGGL(nucleus_kernel, dim3(batch), dim3(HX_NUC_THREADS), 0, st, logits, e->cfg.vocab,
                       (const float *)(e->ws + e->map.amax_val), e->wlm.n_tiles, sample->positions, sample->row_ids,
                       sample->inv_temperature, sample->top_p, sample->key0, sample->key1, tokens_out, logprobs_out,
                       sample->nucleus_sizes);
    HX_CHECK_LAUNCH("nucleus");
    return HX_OK;
}
