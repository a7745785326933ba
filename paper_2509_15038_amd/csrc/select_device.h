// Device code of the per-head selection: the sink, top-k and union steps of
// Algorithm 1, for gfx950.  Shared by the stand-alone selection kernels, the fused
// kernel and the head-wise budget allocation.
//
// A workgroup of THREADS threads handles one (layer, group) with n <= THREADS*KPT.
// Thread t holds the order-preserving 32-bit keys of tokens t, t + THREADS,
// t + 2*THREADS, ... in registers for the whole selection, so every pass over the
// keys is straight-line code with no loads.  The task is to find the key T of the
// (k-s)-th largest candidate and how many keys equal to T are still needed; an
// ordered compaction then lists, in ascending token order, the sinks, every
// candidate above T and the first `need` candidates equal to T, which realises
// "larger score first, then smaller index" exactly.
//
// Finding T, usual case: one histogram over 4096 bins that are a fixed, monotone
// function of the key (bin12: seven exponent bits and five mantissa bits of a score
// below 2, i.e. 32 bins per binade whatever the head's range is), a scan of the
// bins from the top to the bin that holds T, then one more pass over the keys that
// marks every candidate in a higher bin as kept and copies the few candidates
// inside the bin (typically a fraction of a percent of the head) to a list in LDS.
// The remaining 18 key bits are resolved on that list alone, three 6-bit digits,
// and the list's members are then marked "above T" or "equal to T".  The keys in
// registers are walked twice in all.
//
// Finding T, general case (the bin holds more keys than the list takes, e.g. a
// head whose scores are all equal, or scores of 2 and above, which all share the
// last bin): most-significant-digit radix select over the keys in registers, 8
// bits at a time, on key - kmin starting at the highest bit in which the head's
// keys differ at all.
//
// The compaction works on bitmaps: one 64-token word per (row, wave) of "above T"
// and of "equal to T" flags; one wave trims the tied flags to the first `need`,
// scans the popcounts into output positions, and then each word's set bits are
// listed.  The indices are collected in an LDS staging array so that the caller
// can write them out, or gather by them, with coalesced accesses.
#pragma once

#include "curdkv_internal.h"

namespace curdkv {

constexpr int kHistRep = 8;                       // general case: replicated bins to thin out LDS atomic collisions
constexpr int kBins12 = 4096;
constexpr int kBinShift = 18;                     // key bits below the bin number (for bins other than the last)

__device__ __forceinline__ uint32_t order_key(float x) {
    x = x + 0.0f;                                 // -0 -> +0
    const uint32_t b = __float_as_uint(x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Bin of a key: monotone non-decreasing in the key for non-negative scores.  Scores in
// [0, 2) get their exponent and top five mantissa bits; everything from 2 upwards shares
// bin 4095.  Always in [0, 4095], whatever the key.
__device__ __forceinline__ uint32_t bin12(uint32_t key) {
    const uint32_t b = (key & 0x7FFFFFFFu) >> kBinShift;
    return b < (uint32_t)(kBins12 - 1) ? b : (uint32_t)(kBins12 - 1);
}

// The normalisation step of Algorithm 1 applied on the fly: v -> v / (sum of the head), the
// sum being the per-block partial sums added in index order in double; 1/n when the sum
// is 0.  The arithmetic is the one of the stand-alone normalisation kernel.
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

// A threshold the caller already knows (the head-wise budget allocation finds one per layer):
// keep every candidate whose key, without its top bit, is above key31, and the first `need`
// candidates equal to it.  key31 = 0xFFFFFFFF: not known, search for it.
struct Threshold {
    uint32_t key31;
    uint32_t need;
};
constexpr uint32_t kNoThreshold = 0xFFFFFFFFu;

// What find_bin_from_top reports (in LDS).
struct BinFound {
    uint32_t bin;                                 // the bin in which the running count from the top reaches `want`
    uint32_t rank;                                // the rank wanted inside that bin, counted from its top (>= 1)
    uint32_t count;                               // keys in that bin
};

// Scans BINS counts (a multiple of THREADS) from the top bin downwards and finds the bin in
// which the running count reaches `want` (1 <= want <= total count).  All THREADS threads
// call it; wave_tot is LDS scratch of THREADS/64 words.  Ends with a barrier, after which
// *found may be read.
template <int THREADS, int BINS>
__device__ __forceinline__ void find_bin_from_top(const uint32_t* hist, uint32_t want,
                                                  uint32_t* wave_tot, BinFound* found) {
    constexpr int kPer = BINS / THREADS;           // bins per thread, descending
    static_assert(kPer >= 1 && kPer * THREADS == BINS, "bins must be a multiple of the threads");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t c[kPer], tot = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        c[i] = hist[BINS - 1 - (tid * kPer + i)];
        tot += c[i];
    }
    uint32_t incl = tot;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_up(incl, off, 64);
        if (lane >= off) incl += t;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = 0;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
    uint32_t run = before + incl - tot;            // keys in higher bins
    if (run < want && want <= run + tot) {
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            if (want <= run + c[i]) {
                found->bin = (uint32_t)(BINS - 1 - (tid * kPer + i));
                found->rank = want - run;
                found->count = c[i];
                break;
            }
            run += c[i];
        }
    }
    __syncthreads();
}

template <int THREADS, int KPT>
struct SelectShared {
    static constexpr int kWaves = THREADS / 64;
    uint32_t hist[kBins12];                       // bin12 histogram; later the digit histograms (general case: 256 x kHistRep)
    unsigned long long gmask[KPT * kWaves];       // bitmaps over the tokens, one 64-token word per (row, wave)
    unsigned long long emask[KPT * kWaves];
    uint32_t wpos[KPT * kWaves];                  // output position of a word's first kept token
    uint32_t bin_count[256];                      // general case: bins summed over their replicas
    uint32_t wave_a[kWaves], wave_b[kWaves];
    BinFound found;
    uint32_t digit, want, list_count;
};

// The bin12 histogram of the candidates (tokens s <= j < n) of the keys in registers into
// sm.hist.  All threads call it; sm.hist is complete after the barrier it ends with.
template <int THREADS, int KPT>
__device__ __forceinline__ void build_hist12(const uint32_t (&x)[KPT], int32_t n, int32_t s,
                                             SelectShared<THREADS, KPT>& sm) {
    const int tid = threadIdx.x;
    for (int i = tid; i < kBins12; i += THREADS) sm.hist[i] = 0;
    __syncthreads();
    const uint32_t span = (uint32_t)(n - s);
    const uint32_t jt = (uint32_t)(tid - s);       // token - s of row 0, wraps for sinks
#pragma unroll
    for (int it = 0; it < KPT; ++it)
        if (jt + (uint32_t)(it * THREADS) < span) atomicAdd(&sm.hist[bin12(x[it])], 1u);
    __syncthreads();
}

// General case of the threshold search: radix select over the keys in registers.  Fills
// sm.gmask / sm.emask with the "above T" / "equal to T" flags of the candidates and returns
// how many keys equal to T are still to be kept.  x is overwritten.  Ends with a barrier.
template <int THREADS, int KPT>
__device__ __forceinline__ uint32_t threshold_by_radix(uint32_t (&x)[KPT], int32_t n, int32_t s, int32_t m,
                                                       SelectShared<THREADS, KPT>& sm) {
    constexpr int kWaves = THREADS / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t span = (uint32_t)(n - s);
    const uint32_t jt = (uint32_t)(tid - s);
    auto cand = [&](int it) -> bool { return jt + (uint32_t)(it * THREADS) < span; };
    // ---- range [kmin, kmax] of the candidates -----------------------------------
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
    // Word w = it*kWaves + wave of a bitmap covers tokens 64w .. 64w+63, so one ballot per
    // row is one word.
    const uint32_t above = kNotCand - 1u - T;      // T < x < all-ones  <=>  x - T - 1 < above
#pragma unroll
    for (int it = 0; it < KPT; ++it) {
        const uint64_t bg = __ballot(x[it] - T - 1u < above), be = __ballot(x[it] == T);
        if (lane == 0) { sm.gmask[it * kWaves + wave] = bg; sm.emask[it * kWaves + wave] = be; }
    }
    __syncthreads();
    return want;                                   // keys equal to T still to be kept (>= 1)
}

// Resolves the 18 key bits below the bin number on a list of (key, token) pairs in LDS:
// pairs[2i] = key, pairs[2i+1] = token of the i-th of `count` candidates, all of bin `bin`
// (< 4095).  `want` = rank of the threshold among them, from the top.  Three 6-bit digits;
// hist64 is LDS scratch of 64 zeroed words (left zeroed), digit/want_s LDS words.  Returns
// the threshold as (key & 0x7FFFFFFF) and, through *need, how many keys equal to it are still
// to be kept.  All THREADS threads call it; ends with a barrier.
template <int THREADS>
__device__ __forceinline__ uint32_t threshold_on_list(const int32_t* pairs, uint32_t count, uint32_t bin,
                                                      uint32_t want, uint32_t* hist64, uint32_t* digit,
                                                      uint32_t* want_s, uint32_t* need) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t fixed = bin;                          // decided high part of (key & 0x7FFFFFFF): >> rem
    for (int rem = kBinShift; rem > 0; rem -= 6) {
        const int shift = rem - 6;
        for (uint32_t i = tid; i < count; i += THREADS) {
            const uint32_t key = (uint32_t)pairs[2 * i] & 0x7FFFFFFFu;
            if ((key >> rem) == fixed) atomicAdd(&hist64[(key >> shift) & 63u], 1u);
        }
        __syncthreads();
        if (wave == 0) {                           // lane L looks at digit 63 - L
            const uint32_t c = hist64[63 - lane];
            uint32_t incl = c;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t t = __shfl_up(incl, off, 64);
                if (lane >= off) incl += t;
            }
            if (incl - c < want && want <= incl) { *digit = 63 - lane; *want_s = want - (incl - c); }
            hist64[63 - lane] = 0;
        }
        __syncthreads();
        fixed = (fixed << 6) | *digit;
        want = *want_s;
        // digit/want_s are next written after another barrier
    }
    *need = want;
    return fixed;
}

// x[it]: key of token it*THREADS + tid (any value for tokens >= n).  Writes the k
// selected token indices, ascending, to stage[0..k) (positions >= cap go straight
// to out_global instead).  stage[] is also used as working memory before that.  All
// threads of the workgroup must call it; it ends with a barrier, after which stage[]
// is complete.  0 <= k <= n, 0 <= s <= n, n <= THREADS*KPT < 65536, cap >= 0.
// `given`: the threshold, where the caller knows it (then k - s must be the number of
// candidates above it plus given.need); the search is skipped.
template <int THREADS, int KPT>
__device__ __forceinline__ void select_core(uint32_t (&x)[KPT], int32_t n, int32_t s, int32_t k,
                                            SelectShared<THREADS, KPT>& sm, int32_t* stage,
                                            int32_t cap, int32_t* out_global,
                                            Threshold given = Threshold{kNoThreshold, 0u}) {
    constexpr int kWaves = THREADS / 64;
    constexpr int kWords = KPT * kWaves;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    auto put = [&](uint32_t pos, int32_t j) {
        if (pos < (uint32_t)cap) stage[pos] = j; else out_global[pos] = j;
    };

    const int32_t sinks = s < k ? s : k;           // budget inside the sink block: tokens 0..k-1
    const int32_t m = k - s;                       // picks among tokens [s, n)
    const uint32_t span = (uint32_t)(n - s);
    if (m <= 0) {
        for (int32_t j = tid; j < sinks; j += THREADS) put(j, j);
        __syncthreads();
        return;
    }
    if ((uint32_t)m >= span) {                     // everything is kept
        for (int32_t j = tid; j < n; j += THREADS) put(j, j);
        __syncthreads();
        return;
    }

    uint32_t need;
    if (given.key31 != kNoThreshold) {
        // ---- the threshold is known: flags straight from the keys -------------------------------
        const uint32_t jt = (uint32_t)(tid - s);
#pragma unroll
        for (int it = 0; it < KPT; ++it) {
            const bool cd = jt + (uint32_t)(it * THREADS) < span;
            const uint32_t k31 = x[it] & 0x7FFFFFFFu;
            const uint64_t bg = __ballot(cd && k31 > given.key31), be = __ballot(cd && k31 == given.key31);
            if (lane == 0) { sm.gmask[it * kWaves + wave] = bg; sm.emask[it * kWaves + wave] = be; }
        }
        need = given.need;
        __syncthreads();
    } else {
    // ---- the bin that holds the threshold ------------------------------------------------
    build_hist12<THREADS, KPT>(x, n, s, sm);
    if (tid == 0) sm.list_count = 0;
    find_bin_from_top<THREADS, kBins12>(sm.hist, (uint32_t)m, sm.wave_a, &sm.found);
    const uint32_t bstar = sm.found.bin;
    const uint32_t in_bin = sm.found.count;        // candidates inside that bin (>= 1)
    const uint32_t rank = sm.found.rank;           // of the threshold inside the bin, from the top
    // the list takes (key, token) pairs in stage[]; the last bin has no fixed width
    if (bstar < (uint32_t)(kBins12 - 1) && (int64_t)in_bin * 2 <= (int64_t)cap) {
        const uint32_t jt = (uint32_t)(tid - s);
        for (int i = tid; i < kWords; i += THREADS) sm.emask[i] = 0ull;
        for (int i = tid; i < 64; i += THREADS) sm.hist[i] = 0;
        // ---- candidates in higher bins are kept; those inside the bin go to the list ---------
#pragma unroll
        for (int it = 0; it < KPT; ++it) {
            const bool cd = jt + (uint32_t)(it * THREADS) < span;
            const uint32_t b = bin12(x[it]);
            const uint64_t bg = __ballot(cd && b > bstar);
            if (lane == 0) sm.gmask[it * kWaves + wave] = bg;
            if (cd && b == bstar) {
                const uint32_t slot = atomicAdd(&sm.list_count, 1u);
                if (slot < in_bin) {               // always true; keeps a write inside the list whatever happens
                    stage[2 * slot] = (int32_t)x[it];
                    stage[2 * slot + 1] = it * THREADS + tid;
                }
            }
        }
        __syncthreads();
        const uint32_t T = threshold_on_list<THREADS>(stage, in_bin, bstar, rank, sm.hist, &sm.digit, &sm.want, &need);
        // ---- the list's members join the bitmaps -------------------------------------------------
        for (uint32_t i = tid; i < in_bin; i += THREADS) {
            const uint32_t key = (uint32_t)stage[2 * i] & 0x7FFFFFFFu;
            const uint32_t j = (uint32_t)stage[2 * i + 1];
            if (key > T) atomicOr(&sm.gmask[j >> 6], 1ull << (j & 63u));
            else if (key == T) atomicOr(&sm.emask[j >> 6], 1ull << (j & 63u));
        }
        __syncthreads();
    } else {
        need = threshold_by_radix<THREADS, KPT>(x, n, s, m, sm);
    }
    }

    // ---- ordered compaction through the bitmaps ------------------------------------------
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
    __syncthreads();                               // the list in stage[] is no longer needed either
    for (int32_t j = tid; j < sinks; j += THREADS) put(j, j);
    // a thread lists the kept tokens of a quarter word (16 tokens), ascending.  Quarter words
    // rather than words bound the walk when the kept tokens are neighbours (sink-like prefixes,
    // recent windows): 60 neighbours in one word cost one thread, and everybody waiting for
    // it, 5 us.
    for (int q = tid; q < kWords * 4; q += THREADS) {
        const int w = q >> 2, part = q & 3;
        const uint64_t word = sm.gmask[w];
        uint32_t mm = (uint32_t)(word >> (16 * part)) & 0xFFFFu;
        uint32_t pos = sm.wpos[w] + (uint32_t)__popcll(word & ((1ull << (16 * part)) - 1ull));
        while (mm) {
            const int bit = __ffs(mm) - 1;
            mm &= mm - 1;
            // positions stay below k by construction; the comparison keeps a write inside
            // the group's slice whatever the keys were
            if (pos < (uint32_t)k) put(pos, w * 64 + 16 * part + bit);
            ++pos;
        }
    }
    __syncthreads();
}

}  // namespace curdkv
