// AdaCurDKV head-wise budgets (Section 3.2, "Adaptive budget allocation"), for
// gfx950: a layer keeps H*k tokens in all, the top normalised scores across its
// heads, except that every head is guaranteed its own best floor(alpha*k) tokens
// (sinks first).  Only the per-head COUNTS are needed here; feeding them to the
// per-head selection then yields the layer-wide set.
//
// With c_h(t) = number of non-sink tokens of head h that rank above a threshold
// t (ties in (head, token) order), head h keeps max(g, c_h(t)) non-sink tokens,
// g being the guaranteed number, and the threshold is where
//     sum_h max(0, c_h(t) - g) = R,      R = H*(k - s') - H*g.
// The counting functions c_h come from per-head histograms of the order-
// preserving keys, refined level by level from the most significant bits
// (12 + 12 + 8 bits for 8 heads), one streaming pass over the layer's scores
// (H*n floats, resident in L2 / Infinity Cache) per level.  No token order is
// needed: equal keys at the final threshold are allotted head by head.
//
// One 1024-thread workgroup per layer.

#include "select_device.h"

namespace curdkv {

constexpr int kAdaThreads = 1024;
constexpr int kAdaWaves = kAdaThreads / 64;
constexpr int kAdaU = 8;                          // scores per thread per chunk

struct AdaShared {
    uint32_t wave_tot[kAdaWaves];
    unsigned long long best;                      // first position (bins counted from the top) reaching R
};

__global__ __launch_bounds__(kAdaThreads) void adaptive_budget_kernel(
    const float* __restrict__ scores, int64_t n, int H, int bits, int32_t k, int32_t sp, int32_t g,
    long long R, int32_t* __restrict__ budgets) {
    extern __shared__ uint32_t dyn[];
    const int NBmax = 1 << bits;
    uint32_t* hist = dyn;                          // [H][NB]
    uint32_t* above = dyn + (size_t)H * NBmax;     // [H] keys above the prefix decided so far
    uint32_t* wave_excl = above + H;               // [H][kAdaWaves]
    __shared__ AdaShared sm;

    const int layer = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* base = scores + (size_t)layer * H * n;
    int32_t* out = budgets + (size_t)layer * H;

    if (k <= sp) {                                 // budget inside the sink block: nothing to allot
        for (int h = tid; h < H; h += kAdaThreads) out[h] = k;
        return;
    }
    if (R <= 0) {                                  // everything is covered by the safeguard
        for (int h = tid; h < H; h += kAdaThreads) out[h] = sp + g;
        return;
    }
    for (int h = tid; h < H; h += kAdaThreads) above[h] = 0;

    const int64_t total = (int64_t)H * n;
    int decided = 0;
    uint32_t prefix = 0;
    int NB = NBmax, B = bits;
    while (decided < 32) {
        B = bits < 32 - decided ? bits : 32 - decided;
        NB = 1 << B;
        const int shift = 32 - decided - B;
        const uint32_t dmask = (uint32_t)NB - 1u;
        for (int i = tid; i < H * NB; i += kAdaThreads) hist[i] = 0;
        if (tid == 0) sm.best = ~0ull;
        __syncthreads();

        // ---- one pass over the layer: per-head histogram of the next B key bits ----------
        {
            // thread-strided over the flat [H*n] array; (h, j) follows the flat index
            int64_t f = tid;
            int h = (int)(f / n);
            int64_t j = f - (int64_t)h * n;
            float cur[kAdaU], nxt[kAdaU];
            auto load = [&](float (&v)[kAdaU], int64_t f0) {
#pragma unroll
                for (int u = 0; u < kAdaU; ++u) {
                    const int64_t ff = f0 + (int64_t)u * kAdaThreads;
                    v[u] = ff < total ? base[ff] : 0.f;
                }
            };
            load(cur, f);
            for (; f < total; f += (int64_t)kAdaU * kAdaThreads) {
                const int64_t fn = f + (int64_t)kAdaU * kAdaThreads;
                if (fn < total) load(nxt, fn);
#pragma unroll
                for (int u = 0; u < kAdaU; ++u) {
                    if (f + (int64_t)u * kAdaThreads < total && j >= sp) {
                        const uint32_t key = order_key(cur[u]);
                        if (decided == 0 || (key >> (32 - decided)) == prefix)
                            atomicAdd(&hist[(size_t)h * NB + ((key >> shift) & dmask)], 1u);
                    }
                    j += kAdaThreads;
                    while (j >= n) { j -= n; ++h; }
                }
#pragma unroll
                for (int u = 0; u < kAdaU; ++u) cur[u] = nxt[u];
            }
        }
        __syncthreads();

        // ---- find the bin where sum_h max(0, c_h - g) reaches R -----------------------------
        const int per = NB >= kAdaThreads ? NB / kAdaThreads : 1;       // bins per thread, from the top
        unsigned long long E[4] = {0, 0, 0, 0};
        for (int h = 0; h < H; ++h) {
            uint32_t c[4], tot = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int pos = tid * per + i;
                c[i] = (i < per && pos < NB) ? hist[(size_t)h * NB + (NB - 1 - pos)] : 0u;
                tot += c[i];
            }
            uint32_t incl = tot;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t t = __shfl_up(incl, off, 64);
                if (lane >= off) incl += t;
            }
            if (lane == 63) sm.wave_tot[wave] = incl;
            __syncthreads();
            uint32_t before = 0;
            for (int w = 0; w < wave; ++w) before += sm.wave_tot[w];
            if (lane == 0) wave_excl[h * kAdaWaves + wave] = before;
            uint32_t run = above[h] + before + incl - tot;      // keys of head h in higher bins
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                run += c[i];
                if (i < per && run > (uint32_t)g) E[i] += run - (uint32_t)g;
            }
            __syncthreads();                                    // wave_tot is reused by the next head
        }
        {
            unsigned long long mine = ~0ull;
#pragma unroll
            for (int i = 3; i >= 0; --i) {
                const int pos = tid * per + i;
                if (i < per && pos < NB && E[i] >= (unsigned long long)R) mine = (unsigned long long)pos;
            }
            if (mine != ~0ull) atomicMin(&sm.best, mine);
        }
        __syncthreads();
        const int best = (int)sm.best;                          // exists: the lowest bin reaches R
        // ---- keys above the chosen bin join `above`; done by the wave that owns the bin ------
        if (wave == best / per / 64) {
            for (int h = 0; h < H; ++h) {
                uint32_t c[4], tot = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int pos = tid * per + i;
                    c[i] = (i < per && pos < NB) ? hist[(size_t)h * NB + (NB - 1 - pos)] : 0u;
                    tot += c[i];
                }
                uint32_t incl = tot;
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    const uint32_t t = __shfl_up(incl, off, 64);
                    if (lane >= off) incl += t;
                }
                if (tid == best / per) {
                    uint32_t run = wave_excl[h * kAdaWaves + wave] + incl - tot;
                    for (int i = 0; i < best - tid * per; ++i) run += c[i];
                    above[h] += run;
                }
            }
        }
        prefix = (B == 32) ? (uint32_t)(NB - 1 - best) : ((prefix << B) | (uint32_t)(NB - 1 - best));
        decided += B;
        __syncthreads();
    }

    // ---- exact threshold reached: above[h] keys beat it, hist[h][bin] keys equal it ----------
    if (tid == 0) {
        const int bin = (int)(prefix & ((uint32_t)NB - 1u));
        long long rest = R;
        for (int h = 0; h < H; ++h)
            if (above[h] > (uint32_t)g) rest -= (long long)(above[h] - (uint32_t)g);
        for (int h = 0; h < H; ++h) {
            const long long cp = above[h], eq = hist[(size_t)h * NB + bin];
            const long long kept = cp > g ? cp : g;             // before any tied key is allotted
            long long open_eq = cp + eq - kept;                  // tied keys the safeguard does not cover
            if (open_eq < 0) open_eq = 0;
            const long long take = open_eq < rest ? open_eq : rest;
            rest -= take;
            out[h] = (int32_t)(sp + kept + take);
        }
    }
}

// bits per level so that H histograms fit in 128 KB of LDS
static int level_bits(int H) {
    int bits = 12;
    while (bits > 3 && ((size_t)H << bits) * 4 > 128 * 1024) --bits;
    return bits;
}

hipError_t configure_adaptive(curdkv_ctx* ctx) {
    const int dyn = ctx->lds_limit - 8 * 1024;
    if (dyn <= 48 * 1024) return hipSuccess;
    return hipFuncSetAttribute((const void*)adaptive_budget_kernel,
                               hipFuncAttributeMaxDynamicSharedMemorySize, dyn);
}

hipError_t launch_adaptive(const curdkv_ctx* ctx, const float* scores, int64_t n, int32_t k,
                           int32_t sp, int32_t g, long long R, int32_t* budgets, hipStream_t stream) {
    const int H = ctx->cfg.kv_heads;
    const int bits = level_bits(H);
    const size_t lds = (((size_t)H << bits) + (size_t)H + (size_t)H * kAdaWaves) * 4;
    adaptive_budget_kernel<<<dim3((unsigned)ctx->cfg.layers), kAdaThreads, lds, stream>>>(
        scores, n, H, bits, k, sp, g, R, budgets);
    return hipGetLastError();
}

}  // namespace curdkv
