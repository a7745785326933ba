// Device code of the per-head selection: the sink, top-k and union steps of
// Algorithm 1, for gfx950.  Shared by the stand-alone selection kernel and the fused kernel.
//
// A workgroup of THREADS threads handles one (layer, group) with n <= THREADS*KPT.
// Thread t holds the order-preserving 32-bit keys of tokens t, t + THREADS,
// t + 2*THREADS, ... in registers for the whole selection, so every pass is
// straight-line code with no loads.  A most-significant-digit radix select finds
// the key T of the (k-s)-th largest candidate and how many keys equal to T are
// still needed; an ordered compaction then lists, in ascending token order, the
// sinks, every candidate above T and the first `need` candidates equal to T,
// which realises "larger score first, then smaller index" exactly.
//
// The radix digits are taken from (key - kmin), starting at the highest bit in
// which the head's keys differ at all.  Scores of one head span a few binades,
// so digits taken from the raw bit pattern would pile almost every key into two
// or three bins and serialise the LDS atomics; relative to the head's own range
// the first digit already spreads the keys over up to 256 bins.
//
// The compaction works on bitmaps: one ballot per row of THREADS tokens gives a
// 64-token word of "above T" and of "equal to T" flags; one wave trims the tied
// flags to the first `need`, scans the popcounts into output positions, and then
// each word's set bits are listed.  The indices are collected in an LDS staging
// array so that the caller can write them out, or gather by them, with coalesced
// accesses.
#pragma once

#include "curdkv_internal.h"

namespace curdkv {

constexpr int kHistRep = 8;                       // replicated bins to thin out LDS atomic collisions

__device__ __forceinline__ uint32_t order_key(float x) {
    x = x + 0.0f;                                 // -0 -> +0
    const uint32_t b = __float_as_uint(x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// The normalisation step of Algorithm 1 applied on the fly: v -> v / (sum of the head), the sum being the
// per-block partial sums added in index order in double; 1/n when the sum is 0.
// The arithmetic is the one of the stand-alone normalisation kernel.
struct HeadScale {
    float inv, uniform;
    bool zero, on;
    __device__ __forceinline__ float operator()(float v) const {
        return !on ? v : (zero ? uniform : v * inv);
    }
};
__device__ __forceinline__ HeadScale head_scale(const float* __restrict__ partial, int blocks, int64_t n) {
    HeadScale h;
    h.on = blocks > 0;
    double tot = 0.0;
    for (int i = 0; i < blocks; ++i) tot += (double)partial[i];
    h.zero = !(tot > 0.0);
    h.inv = h.zero ? 0.f : (float)(1.0 / tot);
    h.uniform = (float)(1.0 / (double)n);
    return h;
}

template <int THREADS, int KPT>
struct SelectShared {
    static constexpr int kWaves = THREADS / 64;
    uint32_t hist[256 * kHistRep];
    uint32_t bin_count[256];
    unsigned long long gmask[KPT * kWaves];       // bitmaps over the tokens, one 64-token word per (row, wave)
    unsigned long long emask[KPT * kWaves];
    uint32_t wpos[KPT * kWaves];                  // output position of a word's first kept token
    uint32_t wave_a[kWaves], wave_b[kWaves];
    uint32_t digit, want;
};

// x[it]: key of token it*THREADS + tid (any value for tokens >= n).  Writes the k
// selected token indices, ascending, to stage[0..k) (positions >= cap go straight
// to out_global instead).  All threads of the workgroup must call it; it ends
// with a barrier, after which stage[] is complete.  0 <= k <= n, 0 <= s <= n,
// n <= THREADS*KPT < 65536.
template <int THREADS, int KPT>
__device__ __forceinline__ void select_core(uint32_t (&x)[KPT], int32_t n, int32_t s, int32_t k,
                                            SelectShared<THREADS, KPT>& sm, int32_t* stage,
                                            int32_t cap, int32_t* out_global) {
    constexpr int kWaves = THREADS / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    auto put = [&](uint32_t pos, int32_t j) {
        if (pos < (uint32_t)cap) stage[pos] = j; else out_global[pos] = j;
    };

    const int32_t sinks = s < k ? s : k;           // budget inside the sink block: tokens 0..k-1
    for (int32_t j = tid; j < sinks; j += THREADS) put(j, j);
    const int32_t m = k - s;                       // picks among tokens [s, n)
    const uint32_t span = (uint32_t)(n - s);
    if (m <= 0) { __syncthreads(); return; }
    if ((uint32_t)m >= span) {                     // everything is kept
        for (int32_t j = s + tid; j < n; j += THREADS) put(j, j);
        __syncthreads();
        return;
    }

    // ---- range [kmin, kmax] of the candidates -----------------------------------
    const uint32_t jt = (uint32_t)(tid - s);       // token - s of row 0, wraps for sinks
    auto cand = [&](int it) -> bool { return jt + (uint32_t)(it * THREADS) < span; };
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
    for (int it = 0; it < KPT; ++it)
        if (cand(it)) { kmin = x[it] < kmin ? x[it] : kmin; kmax = x[it] > kmax ? x[it] : kmax; }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const uint32_t a = __shfl_xor(kmin, off, 64), b = __shfl_xor(kmax, off, 64);
        kmin = a < kmin ? a : kmin;
        kmax = b > kmax ? b : kmax;
    }
    if (lane == 0) { sm.wave_a[wave] = kmin; sm.wave_b[wave] = kmax; }
    for (int i = tid; i < 256 * kHistRep; i += THREADS) sm.hist[i] = 0;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        kmin = sm.wave_a[w] < kmin ? sm.wave_a[w] : kmin;
        kmax = sm.wave_b[w] > kmax ? sm.wave_b[w] : kmax;
    }
    // From here on x = key - kmin for candidates and all-ones for everything else
    // (sinks, tokens beyond n).  Scores are non-negative, so a candidate's x stays
    // below 2^31 and the all-ones value never matches a prefix or the threshold:
    // the passes below need no per-token candidate test.
    constexpr uint32_t kNotCand = 0xFFFFFFFFu;
#pragma unroll
    for (int it = 0; it < KPT; ++it) x[it] = cand(it) ? x[it] - kmin : kNotCand;

    // ---- radix select on x: T = the m-th largest among the candidates ----------------
    const uint32_t range = kmax - kmin;
    int rem = range ? 32 - __clz(range) : 0;       // bits of x not yet decided
    rem = rem > 31 ? 31 : rem;                     // only reachable with negative scores (not supported)
    uint32_t fixed = 0;                            // decided high part: x >> rem
    uint32_t want = (uint32_t)m;
    uint32_t* myhist = sm.hist + (lane & (kHistRep - 1));
    while (rem > 0) {
        const int w = rem < 8 ? rem : 8;
        const int shift = rem - w;
        const uint32_t dmask = (1u << w) - 1u;
#pragma unroll
        for (int it = 0; it < KPT; ++it)
            if ((x[it] >> rem) == fixed)
                atomicAdd(&myhist[((x[it] >> shift) & dmask) * kHistRep], 1u);
        __syncthreads();
        for (int b = tid; b < 256; b += THREADS) {
            uint32_t c = 0;
#pragma unroll
            for (int r = 0; r < kHistRep; ++r) { c += sm.hist[b * kHistRep + r]; sm.hist[b * kHistRep + r] = 0; }
            sm.bin_count[b] = c;
        }
        __syncthreads();
        if (wave == 0) {
            // lane L looks at bins 255-4L .. 252-4L (descending); find the bin where the
            // count from the top reaches `want`
            uint32_t c[4], tot = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) { c[i] = sm.bin_count[255 - 4 * lane - i]; tot += c[i]; }
            uint32_t incl = tot;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t t = __shfl_up(incl, off, 64);
                if (lane >= off) incl += t;
            }
            uint32_t run = incl - tot;             // keys in higher bins
            if (run < want && want <= incl) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (want <= run + c[i]) { sm.digit = 255 - 4 * lane - i; sm.want = want - run; break; }
                    run += c[i];
                }
            }
        }
        __syncthreads();
        fixed = (fixed << w) | sm.digit;
        want = sm.want;
        rem = shift;
        // digit/want are next written after two more barriers; the histogram is already clear
    }
    const uint32_t T = fixed;                      // in x space
    const uint32_t need = want;                    // keys equal to T still to be kept (>= 1)

    // ---- ordered compaction through bitmaps ----------------------------------------------
    // Word w = it*kWaves + wave of a bitmap covers tokens 64w .. 64w+63, so one ballot per
    // row is one word.  gmask marks candidates above T, emask candidates equal to T.
    constexpr int kWords = KPT * kWaves;
    const uint32_t above = kNotCand - 1u - T;      // T < x < all-ones  <=>  x - T - 1 < above
#pragma unroll
    for (int it = 0; it < KPT; ++it) {
        const uint64_t bg = __ballot(x[it] - T - 1u < above), be = __ballot(x[it] == T);
        if (lane == 0) { sm.gmask[it * kWaves + wave] = bg; sm.emask[it * kWaves + wave] = be; }
    }
    __syncthreads();
    if (wave == 0) {
        // lane L owns words L*kPer .. L*kPer+kPer-1.  First scan: tied keys before each word,
        // to cut emask down to the first `need` of them; second scan: output position of
        // each word's first kept token.
        constexpr int kPer = (kWords + 63) / 64;
        uint64_t keep[kPer];
        uint32_t ne = 0;
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int w = lane * kPer + i;
            keep[i] = w < kWords ? sm.emask[w] : 0ull;
            ne += (uint32_t)__popcll(keep[i]);
        }
        uint32_t incl = ne;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t t = __shfl_up(incl, off, 64);
            if (lane >= off) incl += t;
        }
        uint32_t eq_before = incl - ne, nk = 0;
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int w = lane * kPer + i;
            uint64_t e = keep[i];
            const uint32_t c = (uint32_t)__popcll(e);
            if (eq_before >= need) e = 0ull;                       // quota already used up
            else if (eq_before + c > need)                         // the word where it runs out
                for (uint32_t drop = eq_before + c - need; drop; --drop) e &= ~(1ull << (63 - __clzll((long long)e)));
            eq_before += c;
            keep[i] = (w < kWords ? sm.gmask[w] : 0ull) | e;
            nk += (uint32_t)__popcll(keep[i]);
        }
        incl = nk;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t t = __shfl_up(incl, off, 64);
            if (lane >= off) incl += t;
        }
        uint32_t pos = (uint32_t)s + incl - nk;
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const int w = lane * kPer + i;
            if (w < kWords) { sm.gmask[w] = keep[i]; sm.wpos[w] = pos; }
            pos += (uint32_t)__popcll(keep[i]);
        }
    }
    __syncthreads();
    // a thread lists the kept tokens of a quarter word (16 tokens), ascending.  Quarter words
    // rather than words bound the walk when the kept tokens are neighbours (sink-like prefixes,
    // recent windows): 60 neighbours in one word cost one thread, and everybody waiting for
    // it, 5 us.
    for (int q = tid; q < kWords * 4; q += THREADS) {
        const int w = q >> 2, part = q & 3;
        const uint64_t word = sm.gmask[w];
        uint32_t m = (uint32_t)(word >> (16 * part)) & 0xFFFFu;
        uint32_t pos = sm.wpos[w] + (uint32_t)__popcll(word & ((1ull << (16 * part)) - 1ull));
        while (m) {
            const int bit = __ffs(m) - 1;
            m &= m - 1;
            // positions stay below k by construction; the comparison keeps a write inside
            // the group's slice whatever the keys were
            if (pos < (uint32_t)k) put(pos, w * 64 + 16 * part + bit);
            ++pos;
        }
    }
    __syncthreads();
}

}  // namespace curdkv
