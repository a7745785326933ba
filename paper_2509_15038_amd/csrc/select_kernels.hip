// Selection kernels: the sink, top-k and union steps of Algorithm 1, for gfx950.
// One 1024-thread workgroup per (layer, group).  The method is described in
// select_device.h; this file holds the kernels and their launcher.

#include "select_device.h"

namespace curdkv {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelStaticReserve = 32 * 1024;            // LDS kept for the kernels' static arrays
// ---------------------------------------------------------------------------
// Streaming variant for n too large for the register-resident one.  The head's
// scores (a few hundred KB, resident in L2 / Infinity Cache after the scoring
// kernel) are read twice when the head fits one bitmap block (n <= 131072):
//   1. bin12 histogram of the candidates (select_device.h) -> the bin holding the cut;
//   2. candidates in higher bins are flagged in the "kept" bitmap, those inside the
//      bin go to an LDS list of (key, token) pairs on which the remaining key bits are
//      resolved; the list's members then join the bitmaps, and the ordered compaction
//      runs from the bitmaps alone.
// Longer heads, bins too full for the list and scores of 2 and above take the general
// route, three reads:
//   1. histogram of key bits 31..20 -> bin D1 holding the cut;
//   2. for keys in bin D1: histogram of bits 19..10, and the keys themselves are
//      appended to an LDS list; bits 9..0 are then resolved from that list (or by
//      one more read if the list overflowed) -> exact cut key T and the number
//      `need` of keys equal to T still wanted;
//   3. ordered compaction through LDS bitmaps, 131072 tokens at a time, carrying the
//      running output position, so no separate counting pass is needed.
// Loads are issued a chunk ahead of their use.
// ---------------------------------------------------------------------------
constexpr int kStreamU = 16;                              // keys per thread per chunk
constexpr int kStreamChunk = kSelThreads * kStreamU;      // 16384 tokens
constexpr int kStreamBins = 4096;
constexpr int kStreamList = 16384;                        // words of the LDS list: 16384 keys or 8192 (key, token) pairs
constexpr int kStreamSuper = 8 * kStreamChunk;            // tokens per compaction super-chunk (131072)
constexpr int kStreamWords = kStreamSuper / 64;           // bitmap words per super-chunk

struct StreamShared {
    uint32_t hist[kStreamBins];
    uint32_t list[kStreamList];
    unsigned long long gmask[kStreamWords], emask[kStreamWords];   // "above T" / "equal to T" flags
    uint32_t wpos[kStreamWords];                  // output position of a word's first kept token
    uint32_t wave_tot[kSelWaves];
    uint32_t carry[2];
    BinFound found;
    uint32_t list_count, digit, want;
};

__global__ __launch_bounds__(kSelThreads) void select_stream_kernel(float* __restrict__ scores,
                                                                    int64_t n64, int32_t n_sink,
                                                                    const int64_t* __restrict__ offsets,
                                                                    int32_t* __restrict__ indices,
                                                                    const float* __restrict__ partial,
                                                                    int scale_blocks, int write_scaled) {
    __shared__ StreamShared sm;
    // token numbers are 32-bit throughout (n < 2^31); unsigned, because a chunk may reach past n
    const int head = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t n = (uint32_t)n64;
    const int64_t o0 = offsets[head];
    const uint32_t k = (uint32_t)(offsets[head + 1] - o0);
    int32_t* out = indices + o0;
    float* sc = scores + (size_t)head * n;
    const uint32_t s = (uint32_t)n_sink < n ? (uint32_t)n_sink : n;
    const HeadScale scale = head_scale(partial + (size_t)head * kMaxBlocksPerHead, scale_blocks, n64);
    auto scale_all = [&]() {                       // heads that need no selection still get normalised
        if (scale.on && write_scaled)
            for (uint32_t j = tid; j < n; j += kSelThreads) sc[j] = scale(sc[j]);
    };

    if (k == 0) { scale_all(); return; }
    if (k <= s) {                                  // budget inside the sink block: tokens 0..k-1
        for (uint32_t j = tid; j < k; j += kSelThreads) out[j] = (int32_t)j;
        scale_all();
        return;
    }
    for (uint32_t j = tid; j < s; j += kSelThreads) out[j] = (int32_t)j;
    const uint32_t m = k - s;                      // picks among tokens [s, n)
    if (m >= n - s) {                              // everything is kept
        for (uint32_t j = s + tid; j < n; j += kSelThreads) out[j] = (int32_t)j;
        scale_all();
        return;
    }
    const uint32_t chunks = (n + kStreamChunk - 1) / kStreamChunk;

    // one chunk of scores, thread-strided.  With on-the-fly normalisation the first pass
    // scales and writes back; a thread always re-reads its own tokens, so later passes see
    // the scaled values without any fence.  When nobody wants the normalised scores
    // (write_scaled = 0) nothing is written and every pass scales what it loads.
    bool scaling_pass = scale.on;
    auto load_chunk = [&](float (&v)[kStreamU], uint32_t chunk) {
        // a uniform base per chunk plus a small per-thread offset: 32-bit address arithmetic
        float* cp = sc + (size_t)chunk * kStreamChunk;
        const uint32_t left = n - chunk * kStreamChunk;        // tokens from the chunk's first one on
#pragma unroll
        for (int u = 0; u < kStreamU; ++u) {
            const uint32_t o = u * kSelThreads + tid;
            v[u] = o < left ? cp[o] : 0.f;
        }
        if (scaling_pass) {
#pragma unroll
            for (int u = 0; u < kStreamU; ++u) {
                const uint32_t o = u * kSelThreads + tid;
                v[u] = scale(v[u]);
                if (write_scaled && o < left) cp[o] = v[u];
            }
        }
    };
    auto is_cand = [&](uint32_t chunk, int u) -> bool {
        const uint32_t j = chunk * kStreamChunk + u * kSelThreads + tid;
        return j - s < n - s;                      // s <= j < n
    };
    // runs f(key, chunk, u) over every candidate, loads one chunk ahead
    auto for_each_key = [&](auto f) {
        float cur[kStreamU], nxt[kStreamU];
        load_chunk(cur, 0);
        for (uint32_t c = 0; c < chunks; ++c) {
            if (c + 1 < chunks) load_chunk(nxt, c + 1);
#pragma unroll
            for (int u = 0; u < kStreamU; ++u)
                if (is_cand(c, u)) f(order_key(cur[u]));
#pragma unroll
            for (int u = 0; u < kStreamU; ++u) cur[u] = nxt[u];
        }
    };
    // the same without the look-ahead, for the passes of the general route that run rarely
    auto for_each_key_plain = [&](auto f) {
        float cur[kStreamU];
        for (uint32_t c = 0; c < chunks; ++c) {
            load_chunk(cur, c);
#pragma unroll
            for (int u = 0; u < kStreamU; ++u)
                if (is_cand(c, u)) f(order_key(cur[u]));
        }
    };
    auto clear_hist = [&](int bins) {
        for (int i = tid; i < bins; i += kSelThreads) sm.hist[i] = 0;
    };
    // Ordered compaction of one super-chunk from its bitmaps: words [0, words) of gmask
    // ("above T") and emask ("equal to T") cover tokens super_base + 64w .. +63.  One wave
    // trims the tied flags to what is still needed and scans popcounts into output positions
    // (carrying both across super-chunks), then every quarter word lists its set bits.
    uint32_t eq_carry = 0, pos_carry = (uint32_t)s;
    auto compact_super = [&](int words, uint32_t super_base, uint32_t need) {
        if (wave == 0) {
            constexpr int kPer = kStreamWords / 64;
            uint32_t ne = 0;
#pragma unroll 1
            for (int i = 0; i < kPer; ++i) {
                const int w = lane * kPer + i;
                ne += w < words ? (uint32_t)__popcll(sm.emask[w]) : 0u;
            }
            uint32_t incl = ne;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t t = __shfl_up(incl, off, 64);
                if (lane >= off) incl += t;
            }
            uint32_t eq_before = eq_carry + incl - ne, nk = 0;
            const uint32_t eq_total = __shfl(incl, 63, 64);
#pragma unroll 1
            for (int i = 0; i < kPer; ++i) {
                const int w = lane * kPer + i;
                if (w >= words) break;
                uint64_t e = sm.emask[w];
                const uint32_t cnt = (uint32_t)__popcll(e);
                if (eq_before >= need) e = 0ull;                   // quota already used up
                else if (eq_before + cnt > need)                   // the word where it runs out
                    for (uint32_t drop = eq_before + cnt - need; drop; --drop) e &= ~(1ull << (63 - __clzll((long long)e)));
                eq_before += cnt;
                const uint64_t keep = sm.gmask[w] | e;
                sm.gmask[w] = keep;
                nk += (uint32_t)__popcll(keep);
            }
            incl = nk;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t t = __shfl_up(incl, off, 64);
                if (lane >= off) incl += t;
            }
            uint32_t pos = pos_carry + incl - nk;
#pragma unroll 1
            for (int i = 0; i < kPer; ++i) {
                const int w = lane * kPer + i;
                if (w >= words) break;
                sm.wpos[w] = pos;
                pos += (uint32_t)__popcll(sm.gmask[w]);
            }
            if (lane == 63) { sm.carry[0] = eq_carry + eq_total; sm.carry[1] = pos_carry + incl; }
        }
        __syncthreads();
        eq_carry = sm.carry[0];
        pos_carry = sm.carry[1];
        for (int q = tid; q < words * 4; q += kSelThreads) {   // a thread per quarter word (16 tokens)
            const int w = q >> 2, part = q & 3;
            const uint64_t word = sm.gmask[w];
            uint32_t mm = (uint32_t)(word >> (16 * part)) & 0xFFFFu;
            uint32_t pos = sm.wpos[w] + (uint32_t)__popcll(word & ((1ull << (16 * part)) - 1ull));
            while (mm) {
                const int bit = __ffs(mm) - 1;
                mm &= mm - 1;
                // positions stay below k by construction; the comparison keeps a write inside
                // the group's slice even if the scores were changed under the kernel
                if (pos < k) out[pos] = (int32_t)(super_base + (uint32_t)(w * 64 + 16 * part + bit));
                ++pos;
            }
        }
        __syncthreads();                           // the bitmaps are refilled by the next super-chunk
    };

    // ---- a head that fits one bitmap block: two reads ------------------------------------
    if (n <= kStreamSuper) {
        clear_hist(kStreamBins);
        if (tid == 0) sm.list_count = 0;
        __syncthreads();
        for_each_key([&](uint32_t key) { atomicAdd(&sm.hist[bin12(key)], 1u); });
        scaling_pass = scale.on && !write_scaled;  // written back: the later passes read scaled values
        __syncthreads();
        find_bin_from_top<kSelThreads, kStreamBins>(sm.hist, m, sm.wave_tot, &sm.found);
        const uint32_t bstar = sm.found.bin, in_bin = sm.found.count, rank = sm.found.rank;
        if (bstar < (uint32_t)(kBins12 - 1) && in_bin * 2 <= (uint32_t)kStreamList) {
            const int words = (int)(chunks * (kStreamChunk / 64));
            for (int i = tid; i < words; i += kSelThreads) sm.emask[i] = 0ull;
            for (int i = tid; i < 64; i += kSelThreads) sm.hist[i] = 0;
            float cur[kStreamU], nxt[kStreamU];
            load_chunk(cur, 0);
            for (uint32_t c = 0; c < chunks; ++c) {
                if (c + 1 < chunks) load_chunk(nxt, c + 1);
#pragma unroll
                for (int u = 0; u < kStreamU; ++u) {
                    const uint32_t key = order_key(cur[u]);
                    const bool cd = is_cand(c, u);
                    const uint32_t b = bin12(key);
                    const uint64_t bg = __ballot(cd && b > bstar);
                    const int w = (int)(c * (kStreamChunk / 64)) + u * kSelWaves + wave;
                    if (lane == 0) sm.gmask[w] = bg;
                    if (cd && b == bstar) {
                        const uint32_t slot = atomicAdd(&sm.list_count, 1u);
                        if (slot < in_bin) {           // always true; keeps a write inside the list whatever happens
                            sm.list[2 * slot] = key;
                            sm.list[2 * slot + 1] = c * kStreamChunk + u * kSelThreads + tid;
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < kStreamU; ++u) cur[u] = nxt[u];
            }
            __syncthreads();
            uint32_t need;
            const uint32_t T = threshold_on_list<kSelThreads>(reinterpret_cast<const int32_t*>(sm.list), in_bin, bstar, rank,
                                                             sm.hist, &sm.digit, &sm.want, &need);
            for (uint32_t i = tid; i < in_bin; i += kSelThreads) {
                const uint32_t key = sm.list[2 * i] & 0x7FFFFFFFu;
                const uint32_t j = sm.list[2 * i + 1];
                if (key > T) atomicOr(&sm.gmask[j >> 6], 1ull << (j & 63u));
                else if (key == T) atomicOr(&sm.emask[j >> 6], 1ull << (j & 63u));
            }
            __syncthreads();
            compact_super(words, 0, need);
            return;
        }
        __syncthreads();                           // everybody has read the verdict; the general route starts over
    }

    // ---- pass 1: bits 31..20 --------------------------------------------------------
    clear_hist(kStreamBins);
    if (tid == 0) sm.list_count = 0;
    __syncthreads();
    for_each_key([&](uint32_t key) { atomicAdd(&sm.hist[key >> 20], 1u); });
    scaling_pass = scale.on && !write_scaled;      // written back: the later passes read scaled values
    __syncthreads();
    find_bin_from_top<kSelThreads, kStreamBins>(sm.hist, m, sm.wave_tot, &sm.found);
    const uint32_t d1 = sm.found.bin;
    uint32_t want = sm.found.rank;
    __syncthreads();

    // ---- pass 2: bits 19..10 of the keys in bin d1; keep those keys in LDS -------------
    clear_hist(1024);
    __syncthreads();
    for_each_key_plain([&](uint32_t key) {
        if ((key >> 20) == d1) {
            atomicAdd(&sm.hist[(key >> 10) & 1023u], 1u);
            const uint32_t slot = atomicAdd(&sm.list_count, 1u);
            if (slot < (uint32_t)kStreamList) sm.list[slot] = key;
        }
    });
    __syncthreads();
    find_bin_from_top<kSelThreads, 1024>(sm.hist, want, sm.wave_tot, &sm.found);
    const uint32_t d2 = sm.found.bin;
    want = sm.found.rank;
    const uint32_t in_list = sm.list_count;
    __syncthreads();

    // ---- bits 9..0 -------------------------------------------------------------------
    const uint32_t prefix22 = (d1 << 10) | d2;
    clear_hist(1024);
    __syncthreads();
    if (in_list <= (uint32_t)kStreamList) {
        for (uint32_t i = tid; i < in_list; i += kSelThreads) {
            const uint32_t key = sm.list[i];
            if ((key >> 10) == prefix22) atomicAdd(&sm.hist[key & 1023u], 1u);
        }
    } else {
        for_each_key_plain([&](uint32_t key) {
            if ((key >> 10) == prefix22) atomicAdd(&sm.hist[key & 1023u], 1u);
        });
    }
    __syncthreads();
    find_bin_from_top<kSelThreads, 1024>(sm.hist, want, sm.wave_tot, &sm.found);
    const uint32_t T = (prefix22 << 10) | sm.found.bin;
    const uint32_t need = sm.found.rank;           // keys equal to T still to be kept (>= 1)

    // ---- pass 3: ordered compaction through bitmaps, a super-chunk of tokens at a time -------
    // Word w of a bitmap covers tokens 64w .. 64w+63 of the super-chunk; one ballot of a wave
    // over 64 consecutive tokens is one word.
    constexpr uint32_t chunks_per_super = kStreamSuper / kStreamChunk;
    for (uint32_t c0 = 0; c0 < chunks; c0 += chunks_per_super) {
        const uint32_t c1 = c0 + chunks_per_super < chunks ? c0 + chunks_per_super : chunks;
        const uint32_t super_base = c0 * kStreamChunk;
        float cur[kStreamU], nxt[kStreamU];
        load_chunk(cur, c0);
        for (uint32_t c = c0; c < c1; ++c) {
            if (c + 1 < c1) load_chunk(nxt, c + 1);
#pragma unroll
            for (int u = 0; u < kStreamU; ++u) {
                const uint32_t key = order_key(cur[u]);
                const bool cd = is_cand(c, u);
                const uint64_t bg = __ballot(cd && key > T), be = __ballot(cd && key == T);
                const int w = (int)((c - c0) * (kStreamChunk / 64)) + u * kSelWaves + wave;
                if (lane == 0) { sm.gmask[w] = bg; sm.emask[w] = be; }
            }
#pragma unroll
            for (int u = 0; u < kStreamU; ++u) cur[u] = nxt[u];
        }
        const int words = (int)((c1 - c0) * (kStreamChunk / 64));
        __syncthreads();
        compact_super(words, super_base, need);
    }
}

// ---------------------------------------------------------------------------
// Register-resident variant (select_device.h) for n <= 1024 * KPT.  The chosen
// indices are collected in LDS and written out coalesced.
// ---------------------------------------------------------------------------
template <int KPT>
__global__ __launch_bounds__(kSelThreads) void select_reg_kernel(float* __restrict__ scores,
                                                                 int32_t n, int32_t n_sink,
                                                                 const int64_t* __restrict__ offsets,
                                                                 int32_t* __restrict__ indices, int32_t cap,
                                                                 const float* __restrict__ partial,
                                                                 int scale_blocks, int write_scaled,
                                                                 const Threshold* __restrict__ known) {
    extern __shared__ int32_t stage[];             // [cap]
    __shared__ SelectShared<kSelThreads, KPT> sm;
    const int head = blockIdx.x;
    const int tid = threadIdx.x;
    const int64_t o0 = offsets[head];
    const int32_t k = (int32_t)(offsets[head + 1] - o0);
    if (k <= 0 && (scale_blocks <= 0 || !write_scaled)) return;
    int32_t* out = indices + o0;
    float* sc = scores + (size_t)head * n;
    const int32_t s = n_sink < n ? n_sink : n;
    const HeadScale scale = head_scale(partial + (size_t)head * kMaxBlocksPerHead, scale_blocks, n);

    uint32_t x[KPT];
    {
        float v[KPT];
#pragma unroll
        for (int it = 0; it < KPT; ++it) {
            const int32_t j = it * kSelThreads + tid;
            v[it] = j < n ? sc[j] : 0.f;
        }
#pragma unroll
        for (int it = 0; it < KPT; ++it) {
            v[it] = scale(v[it]);
            const int32_t j = it * kSelThreads + tid;
            if (scale.on && write_scaled && j < n) sc[j] = v[it];
            x[it] = order_key(v[it]);
        }
    }
    if (k <= 0) return;
    select_core<kSelThreads, KPT>(x, n, s, k, sm, stage, cap, out, known ? known[head] : Threshold{kNoThreshold, 0u});
    const int32_t staged = k < cap ? k : cap;
    for (int32_t p = tid; p < staged; p += kSelThreads) out[p] = stage[p];
}

template <int KPT>
static hipError_t launch_reg(const curdkv_ctx* ctx, float* scores, int32_t n, int32_t n_sink,
                             const int64_t* d_offsets, int32_t* indices, hipStream_t stream,
                             int scale_blocks, int write_scaled, const Threshold* known) {
    // the staging area takes what the kernel's static LDS leaves, within the dynamic size the
    // kernel was configured for (configure_select); indices beyond it go straight to memory
    const size_t fixed = sizeof(SelectShared<kSelThreads, KPT>) + 256;
    int64_t cap = ((int64_t)ctx->lds_limit - (int64_t)fixed) / 4;
    const int64_t configured = ((int64_t)ctx->lds_limit - kSelStaticReserve) / 4;
    if (cap > configured) cap = configured;
    if (cap > n) cap = n;
    if (cap < 0) cap = 0;
    select_reg_kernel<KPT><<<dim3((unsigned)ctx->heads), kSelThreads, (size_t)cap * 4, stream>>>(
        scores, n, n_sink, d_offsets, indices, (int32_t)cap, ctx->d_partial, scale_blocks, write_scaled, known);
    return hipGetLastError();
}

hipError_t configure_select(curdkv_ctx* ctx) {
    const int dyn = ctx->lds_limit - kSelStaticReserve;   // what the kernels' static LDS leaves
    if (dyn <= 48 * 1024) return hipSuccess;
    hipError_t e;
    e = hipFuncSetAttribute((const void*)select_reg_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, dyn);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void*)select_reg_kernel<8>, hipFuncAttributeMaxDynamicSharedMemorySize, dyn);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void*)select_reg_kernel<16>, hipFuncAttributeMaxDynamicSharedMemorySize, dyn);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void*)select_reg_kernel<32>, hipFuncAttributeMaxDynamicSharedMemorySize, dyn);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute((const void*)select_reg_kernel<36>, hipFuncAttributeMaxDynamicSharedMemorySize, dyn);
}

hipError_t launch_select(const curdkv_ctx* ctx, float* scores, int64_t n, int32_t n_sink,
                         const int64_t* d_offsets, int32_t* indices, hipStream_t stream,
                         int scale_blocks, bool write_scaled, const void* known_thresholds) {
    const Threshold* known = static_cast<const Threshold*>(known_thresholds);
    const int32_t n32 = (int32_t)n;
    const int ws = write_scaled ? 1 : 0;
    if (n <= 4 * kSelThreads) return launch_reg<4>(ctx, scores, n32, n_sink, d_offsets, indices, stream, scale_blocks, ws, known);
    if (n <= 8 * kSelThreads) return launch_reg<8>(ctx, scores, n32, n_sink, d_offsets, indices, stream, scale_blocks, ws, known);
    if (n <= 16 * kSelThreads) return launch_reg<16>(ctx, scores, n32, n_sink, d_offsets, indices, stream, scale_blocks, ws, known);
    if (n <= 32 * kSelThreads) return launch_reg<32>(ctx, scores, n32, n_sink, d_offsets, indices, stream, scale_blocks, ws, known);
    if (n <= 36 * kSelThreads) return launch_reg<36>(ctx, scores, n32, n_sink, d_offsets, indices, stream, scale_blocks, ws, known);
    select_stream_kernel<<<dim3((unsigned)ctx->heads), kSelThreads, 0, stream>>>(
        scores, n, n_sink, d_offsets, indices, ctx->d_partial, scale_blocks, ws);
    return hipGetLastError();
}

}  // namespace curdkv
