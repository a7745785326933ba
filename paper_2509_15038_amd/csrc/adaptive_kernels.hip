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
// preserving keys over the 4096 bins of the selection (bin12, select_device.h):
//   * the histograms are made by the fused kernel while it has a head's keys in
//     registers, or by ada_hist_kernel from scores in memory, one workgroup per
//     (layer, head);
//   * ada_resolve_kernel, again one workgroup per (layer, head): every workgroup
//     scans the H histograms of its layer for the bin in which the sum above reaches
//     R (the same small computation in each of them, which saves a launch and a
//     trip through memory), copies its own head's keys inside that bin (a fraction
//     of a percent of the head) to the workspace and counts itself done; the
//     workgroup that finds itself the last of its layer resolves the remaining key
//     bits on those few keys in LDS, allots keys equal to the threshold head by
//     head, and writes the budgets, their prefix sums and the gather's block table
//     for the layer (every layer keeps H*k rows, so a layer's first row is known).
// Nobody waits for anybody: a workgroup that is not the last simply ends.  Bins
// too full for the lists (a layer of equal scores, say) and scores of 2 and above
// make the last workgroup refine the threshold by reading the layer's scores
// itself, a few bits per pass: slow, and exact all the same.
// No token order is needed anywhere.

#include <mutex>

#include "select_device.h"

namespace curdkv {

constexpr int kAdaThreads = 1024;
constexpr int kAdaWaves = kAdaThreads / 64;
constexpr int kAdaU = 8;                          // scores per thread in flight
constexpr int kAdaOwn = 32;                       // resolve kernel: scores per thread loaded up front
constexpr int kAdaSeg = 2048;                     // in-bin keys a head hands to its layer's last workgroup
constexpr int kAdaList = 4096;                    // (key, head) pairs that workgroup resolves in LDS
constexpr int kAdaDigWords = 8192;                // its per-head digit histograms: H << bits words
constexpr int kAdaMaxHeads = 1024;                // kv_heads the resolve kernel is laid out for

struct AdaWorkspace {                             // device pointers into one allocation
    uint32_t* hist;                               // [heads][4096] bin12 histograms of the candidates
    uint32_t* seg;                                // [heads][kAdaSeg] keys (31 bits) inside the layer's cut bin
    uint32_t* above;                              // [heads] candidates in bins above the cut bin
    uint32_t* inbin;                              // [heads] candidates inside it
    Threshold* known;                             // [heads] what the selection may take over: the layer's threshold
    AdaLayerState* layer;                         // [layers]
};

static constexpr size_t workspace_bytes_for(size_t heads, size_t layers) {
    return heads * (size_t)kBins12 * 4 + heads * (size_t)kAdaSeg * 4 + heads * 16 + layers * sizeof(AdaLayerState);
}

static AdaWorkspace carve(void* base, size_t heads) {
    AdaWorkspace w;
    w.hist = reinterpret_cast<uint32_t*>(base);
    w.seg = w.hist + heads * kBins12;
    w.above = w.seg + heads * kAdaSeg;
    w.inbin = w.above + heads;
    w.known = reinterpret_cast<Threshold*>(w.inbin + heads);
    w.layer = reinterpret_cast<AdaLayerState*>(w.known + heads);
    return w;
}

// a load that sees what other workgroups of this kernel have written (after the fences below)
__device__ __forceinline__ uint32_t load_agent(const uint32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Histogram of a head's candidate keys (tokens sp and up) over the selection's 4096 bins.
__global__ __launch_bounds__(kAdaThreads) void ada_hist_kernel(
    const float* __restrict__ scores, int64_t n, int H, int32_t sp, uint32_t* __restrict__ ws_hist,
    AdaLayerState* __restrict__ layer_state) {
    __shared__ uint32_t hist[kBins12];
    const int head = blockIdx.x;
    const int tid = threadIdx.x;
    const float* sc = scores + (size_t)head * n;
    if (tid == 0 && head % H == 0) {              // a fresh count of finished workgroups for the layer
        layer_state[head / H].done = 0;
        layer_state[head / H].overflow = 0;
    }
    for (int i = tid; i < kBins12; i += kAdaThreads) hist[i] = 0;
    __syncthreads();
    float cur[kAdaU], nxt[kAdaU];
    auto load = [&](float (&v)[kAdaU], int64_t j0) {
#pragma unroll
        for (int u = 0; u < kAdaU; ++u) {
            const int64_t j = j0 + (int64_t)u * kAdaThreads;
            v[u] = j < n ? sc[j] : 0.f;
        }
    };
    load(cur, tid);
    for (int64_t j0 = tid; j0 < n; j0 += (int64_t)kAdaU * kAdaThreads) {
        const int64_t jn = j0 + (int64_t)kAdaU * kAdaThreads;
        if (jn < n) load(nxt, jn);
#pragma unroll
        for (int u = 0; u < kAdaU; ++u) {
            const int64_t j = j0 + (int64_t)u * kAdaThreads;
            if (j >= sp && j < n) atomicAdd(&hist[bin12(order_key(cur[u]))], 1u);
        }
#pragma unroll
        for (int u = 0; u < kAdaU; ++u) cur[u] = nxt[u];
    }
    __syncthreads();
    uint32_t* dst = ws_hist + (size_t)head * kBins12;
    for (int i = tid; i < kBins12; i += kAdaThreads) dst[i] = hist[i];
}

constexpr int kAdaHeadsAtOnce = 8;

struct AdaShared {
    uint32_t wave_tot[kAdaHeadsAtOnce][kAdaWaves];
    unsigned long long best;                      // first position (bins counted from the top) reaching R
    uint32_t count;                               // keys this workgroup has put into its segment
    uint32_t last;                                // this workgroup is the last of its layer
    uint32_t digit;
    uint32_t total_in;                            // keys inside the cut bin, all heads
    uint32_t slow;
};

// bits per refinement level so that H digit histograms fit kAdaDigWords
__device__ __forceinline__ int ada_level_bits(int H) {
    int bits = 6;
    while (bits > 1 && (H << bits) > kAdaDigWords) --bits;
    return bits;
}

__global__ __launch_bounds__(kAdaThreads) void ada_resolve_kernel(
    AdaWorkspace ws, const float* __restrict__ scores, int64_t n, int H, int32_t sp, int32_t g, long long R,
    int32_t k, int32_t* __restrict__ budgets, int64_t* __restrict__ offsets, BlockInfo* __restrict__ block_info,
    int layers) {
    extern __shared__ __align__(16) uint32_t dyn[];
    __shared__ AdaShared sm;
    // Workgroups are dealt to the chip's eight dies (each with an L2 of its own) round-robin by
    // their number, and the H workgroups of a layer all read that layer's H histograms: where
    // the layers come in multiples of eight, a layer's workgroups are numbered so that they
    // share a die, and the histograms cross the fabric once instead of H times.  (Placement
    // only: any numbering is correct.)
    int head = blockIdx.x;
    if (layers % 8 == 0) {
        const int die = head & 7, q = head >> 3;
        head = ((q / H) * 8 + die) * H + q % H;
    }
    const int layer = head / H, my = head - layer * H;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t* lhist = ws.hist + (size_t)layer * H * kBins12;     // the layer's H histograms

    if (tid == 0) { sm.best = ~0ull; sm.count = 0; sm.slow = 0; }

    // ---- the bin in which sum_h max(0, c_h - g) reaches R -------------------------------------
    // Thread t looks at positions 4t .. 4t+3 counted from the top bin (bin = 4095 - position).
    // kAdaHeadsAtOnce heads go through the workgroup-wide prefix sums together.  The loads of
    // the first heads' histograms go out first, then those of this head's own scores, which
    // are wanted further down (the keys inside the layer's cut bin) and arrive while the
    // histograms are being worked on.
    auto load_counts = [&](uint4 (&v)[kAdaHeadsAtOnce], int h0) {
#pragma unroll
        for (int j = 0; j < kAdaHeadsAtOnce; ++j) {
            const int h = h0 + j < H ? h0 + j : H - 1;
            v[j] = *reinterpret_cast<const uint4*>(lhist + (size_t)h * kBins12 + (kBins12 - 4 - 4 * tid));
        }
    };
    uint4 raw[kAdaHeadsAtOnce];
    load_counts(raw, 0);
    const float* sc = scores + (size_t)head * n;
    float* own = reinterpret_cast<float*>(dyn);    // [kAdaOwn * 1024] staged here: registers are short
    const uint32_t n_first = n < (int64_t)kAdaOwn * kAdaThreads ? (uint32_t)n : (uint32_t)(kAdaOwn * kAdaThreads);
    {
        float v[kAdaOwn];
#pragma unroll
        for (int u = 0; u < kAdaOwn; ++u) {
            const uint32_t o = (uint32_t)(u * kAdaThreads + tid);      // 32-bit offsets from a uniform base
            v[u] = o < n_first ? sc[o] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kAdaOwn; ++u) own[u * kAdaThreads + tid] = v[u];
    }
    __syncthreads();
    unsigned long long E[4] = {0, 0, 0, 0};
    uint32_t mine[4] = {0, 0, 0, 0};               // this head's counts at the thread's positions
    for (int h0 = 0; h0 < H; h0 += kAdaHeadsAtOnce) {
        uint32_t c[kAdaHeadsAtOnce][4], tot[kAdaHeadsAtOnce], incl[kAdaHeadsAtOnce];
        if (h0 > 0) load_counts(raw, h0);
#pragma unroll
        for (int j = 0; j < kAdaHeadsAtOnce; ++j) {
            const bool on = h0 + j < H;
            const uint4 v = raw[j];
            c[j][0] = on ? v.w : 0u; c[j][1] = on ? v.z : 0u; c[j][2] = on ? v.y : 0u; c[j][3] = on ? v.x : 0u;
            tot[j] = c[j][0] + c[j][1] + c[j][2] + c[j][3];
            incl[j] = tot[j];
            if (on && h0 + j == my) { mine[0] = c[j][0]; mine[1] = c[j][1]; mine[2] = c[j][2]; mine[3] = c[j][3]; }
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1)
#pragma unroll
            for (int j = 0; j < kAdaHeadsAtOnce; ++j) {
                const uint32_t t = __shfl_up(incl[j], off, 64);
                if (lane >= off) incl[j] += t;
            }
        if (lane == 63) {
#pragma unroll
            for (int j = 0; j < kAdaHeadsAtOnce; ++j) sm.wave_tot[j][wave] = incl[j];
        }
        __syncthreads();
        // exclusive prefix of the wave totals, per head: thread (j, w) of the first
        // kAdaHeadsAtOnce*16 threads scans inside its group of 16 lanes
        if (tid < kAdaHeadsAtOnce * kAdaWaves) {
            const int j = tid / kAdaWaves, w = tid % kAdaWaves;
            const uint32_t own_tot = sm.wave_tot[j][w];
            uint32_t inc = own_tot;
#pragma unroll
            for (int off = 1; off < kAdaWaves; off <<= 1) {
                const uint32_t t = __shfl_up(inc, off, kAdaWaves);
                if (w >= off) inc += t;
            }
            sm.wave_tot[j][w] = inc - own_tot;
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kAdaHeadsAtOnce; ++j) {
            if (h0 + j >= H) break;
            const uint32_t before = sm.wave_tot[j][wave];
            uint32_t run = before + incl[j] - tot[j];              // keys of this head in higher bins
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                run += c[j][i];
                if (run > (uint32_t)g) E[i] += run - (uint32_t)g;
            }
        }
        __syncthreads();                                        // wave_tot is reused by the next heads
    }
    {
        // E grows with the position, so every thread beyond the crossing qualifies: the minimum is
        // taken inside each wave first, one atomic per wave instead of one per thread
        uint32_t first = 0xFFFFFFFFu;
#pragma unroll
        for (int i = 3; i >= 0; --i)
            if (E[i] >= (unsigned long long)R) first = (uint32_t)(tid * 4 + i);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const uint32_t o = __shfl_xor(first, off, 64);
            first = o < first ? o : first;
        }
        if (lane == 0 && first != 0xFFFFFFFFu) atomicMin(&sm.best, (unsigned long long)first);
    }
    __syncthreads();
    // (the lowest bin always reaches R for histograms of n - sp candidates per head; the bound
    // keeps everything below in range whatever the workspace held)
    const int best = sm.best < (unsigned long long)kBins12 ? (int)sm.best : kBins12 - 1;
    const uint32_t bstar = (uint32_t)(kBins12 - 1 - best);

    // ---- this head: candidates above the bin, candidates inside it ------------------------------
    uint32_t above_my, inbin_my;
    {
        uint32_t part = 0, inb = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int pos = tid * 4 + i;
            part += pos < best ? mine[i] : 0u;
            inb += pos == best ? mine[i] : 0u;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) { part += __shfl_xor(part, off, 64); inb += __shfl_xor(inb, off, 64); }
        if (lane == 0) { sm.wave_tot[0][wave] = part; sm.wave_tot[1][wave] = inb; }
        __syncthreads();
        above_my = 0; inbin_my = 0;
#pragma unroll
        for (int w = 0; w < kAdaWaves; ++w) { above_my += sm.wave_tot[0][w]; inbin_my += sm.wave_tot[1][w]; }
    }
    // ---- hand this head's keys inside the bin to the layer -------------------------------------
    if (bstar < (uint32_t)(kBins12 - 1) && inbin_my <= (uint32_t)kAdaSeg) {
        uint32_t* seg = ws.seg + (size_t)head * kAdaSeg;
        auto hand_in = [&](float v, bool cand) {
            const uint32_t key = order_key(v);
            if (cand && bin12(key) == bstar) {
                const uint32_t slot = atomicAdd(&sm.count, 1u);
                if (slot < (uint32_t)kAdaSeg) seg[slot] = key & 0x7FFFFFFFu;
            }
        };
#pragma unroll 8
        for (int u = 0; u < kAdaOwn; ++u) {
            const uint32_t o = (uint32_t)(u * kAdaThreads + tid);
            hand_in(own[o], o >= (uint32_t)sp && o < n_first);
        }
        // heads longer than the staged part: the rest streams through registers
        for (int64_t j0 = (int64_t)kAdaOwn * kAdaThreads; j0 < n; j0 += (int64_t)kAdaU * kAdaThreads) {
            const float* cp = sc + j0;                              // uniform base, 32-bit offsets
            const uint32_t left = n - j0 < (int64_t)kAdaU * kAdaThreads ? (uint32_t)(n - j0) : (uint32_t)(kAdaU * kAdaThreads);
            float v[kAdaU];
#pragma unroll
            for (int u = 0; u < kAdaU; ++u) {
                const uint32_t o = (uint32_t)(u * kAdaThreads + tid);
                v[u] = o < left ? cp[o] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < kAdaU; ++u) {
                const uint32_t o = (uint32_t)(u * kAdaThreads + tid);
                hand_in(v[u], o < left && j0 + o >= sp);
            }
        }
    } else if (tid == 0) {
        atomicOr(&ws.layer[layer].overflow, 1u);
    }
    if (tid == 0) { ws.above[head] = above_my; ws.inbin[head] = inbin_my; }
    // ---- the last workgroup of the layer to get here goes on; the others are done ---------------
    // One thread fences for the workgroup (the barrier orders the others' writes before its
    // fence, and after the count, its second fence before their reads): a fence at device scope
    // is a cache-wide operation on this chip, far too dear to issue from every wave.  What every
    // wave does do is wait until its own stores have been taken by the L2: the barrier by itself
    // does not wait for stores in flight, and the one write-back must cover them all.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (tid == 0) {
        __threadfence();                                        // the workgroup's writes, before the count
        __builtin_amdgcn_s_waitcnt(0);                          // (the write-back itself included)
        const uint32_t old = atomicAdd(&ws.layer[layer].done, 1u);
        sm.last = old == (uint32_t)(H - 1) ? 1u : 0u;
        if (sm.last) __threadfence();                           // the other workgroups' writes, after the count
    }
    __syncthreads();
    if (!sm.last) return;

    // ---- per-head state in LDS ---------------------------------------------------------------------
    const int B0 = ada_level_bits(H);
    uint32_t* dig = dyn;                           // [H << B] digit histograms, then suffix sums
    uint32_t* above = dyn + kAdaDigWords;          // [H] keys above the prefix decided so far
    uint32_t* inbin = above + kAdaMaxHeads;        // [H] keys inside the cut bin; later: keys equal to the threshold
    uint32_t* base = inbin + kAdaMaxHeads;         // [H + 1] start of a head's keys in the list; later: its first row
    uint32_t* list = base + kAdaMaxHeads + 8;      // [kAdaList][2] (key, head)
    for (int h = tid; h < H; h += kAdaThreads) {
        above[h] = load_agent(ws.above + (size_t)layer * H + h);
        inbin[h] = load_agent(ws.inbin + (size_t)layer * H + h);
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t run = 0;
        bool over = bstar == (uint32_t)(kBins12 - 1) || load_agent(&ws.layer[layer].overflow) != 0;
        for (int h = 0; h < H; ++h) {
            base[h] = run;
            over = over || inbin[h] > (uint32_t)kAdaSeg;
            run += inbin[h] <= (uint32_t)kAdaSeg ? inbin[h] : 0u;
        }
        base[H] = run;
        sm.total_in = run;
        sm.slow = (over || run > (uint32_t)kAdaList) ? 1u : 0u;
    }
    __syncthreads();
    const bool slow = sm.slow != 0;
    const uint32_t total_in = sm.total_in;
    if (!slow) {
        // gather the heads' segments into one list; threads are dealt to heads so that all
        // heads' loads are in flight together
        int per_head = kAdaThreads / H;             // H <= 1024
        if (per_head < 1) per_head = 1;
        const int h = tid / per_head, r = tid - h * per_head;
        if (h < H) {
            const uint32_t* seg = ws.seg + ((size_t)layer * H + h) * kAdaSeg;
            const uint32_t cnt = inbin[h], b0 = base[h];
            for (uint32_t i = r; i < cnt; i += per_head) {
                list[2 * (b0 + i)] = load_agent(seg + i);
                list[2 * (b0 + i) + 1] = (uint32_t)h;
            }
        }
        __syncthreads();
    }

    // ---- refine the threshold below the bin: B bits per level -----------------------------------
    // A key takes part while bin12(key) == bstar and its bits above `rem` equal `fixed`.
    int rem = bstar < (uint32_t)(kBins12 - 1) ? kBinShift : 31;
    uint32_t fixed = bstar < (uint32_t)(kBins12 - 1) ? bstar : 0u;
    const float* lsc = scores + (size_t)layer * H * n;
    while (rem > 0) {
        const int B = rem < B0 ? rem : B0;
        const int D = 1 << B;
        const int shift = rem - B;
        for (int i = tid; i < (H << B); i += kAdaThreads) dig[i] = 0;
        __syncthreads();
        if (!slow) {
            for (uint32_t i = tid; i < total_in; i += kAdaThreads) {
                const uint32_t key = list[2 * i], h = list[2 * i + 1];
                if ((key >> rem) == fixed) atomicAdd(&dig[(h << B) | ((key >> shift) & (uint32_t)(D - 1))], 1u);
            }
        } else {
            for (int h = 0; h < H; ++h) {
                const float* hs = lsc + (size_t)h * n;
                for (int64_t j0 = tid; j0 < n; j0 += (int64_t)kAdaU * kAdaThreads) {
                    float v[kAdaU];
#pragma unroll
                    for (int u = 0; u < kAdaU; ++u) {
                        const int64_t j = j0 + (int64_t)u * kAdaThreads;
                        v[u] = j < n ? hs[j] : 0.f;
                    }
#pragma unroll
                    for (int u = 0; u < kAdaU; ++u) {
                        const int64_t j = j0 + (int64_t)u * kAdaThreads;
                        const uint32_t key = order_key(v[u]);
                        const uint32_t k31 = key & 0x7FFFFFFFu;
                        if (j >= sp && j < n && bin12(key) == bstar && (rem >= 31 || (k31 >> rem) == fixed))
                            atomicAdd(&dig[((uint32_t)h << B) | ((k31 >> shift) & (uint32_t)(D - 1))], 1u);
                    }
                }
            }
        }
        __syncthreads();
        // suffix sums per head: dig[h][d] = keys of head h in this prefix with digit >= d.  A wave
        // per head, lane L on digit D-1-L (D <= 64).
        for (int h = wave; h < H; h += kAdaWaves) {
            uint32_t incl = lane < D ? dig[(h << B) | (D - 1 - lane)] : 0u;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t t = __shfl_up(incl, off, 64);
                if (lane >= off) incl += t;
            }
            if (lane < D) dig[(h << B) | (D - 1 - lane)] = incl;
        }
        __syncthreads();
        if (wave == 0) {                            // lane d: does the sum reach R when digits >= d count?
            bool ok = false;
            if (lane < D) {
                unsigned long long e = 0;
                for (int h = 0; h < H; ++h) {
                    const uint32_t c = above[h] + dig[(h << B) | lane];
                    if (c > (uint32_t)g) e += c - (uint32_t)g;
                }
                ok = e >= (unsigned long long)R;
            }
            const unsigned long long m = __ballot(ok);
            if (lane == 0) sm.digit = m ? (uint32_t)(63 - __clzll((long long)m)) : 0u;   // the largest such digit
        }
        __syncthreads();
        const uint32_t digit = sm.digit;
        const bool last_level = shift == 0;
        for (int h = tid; h < H; h += kAdaThreads) {
            const uint32_t ge = dig[(h << B) | digit];
            const uint32_t gt = digit + 1 < (uint32_t)D ? dig[(h << B) | (digit + 1)] : 0u;
            above[h] += gt;
            if (last_level) inbin[h] = ge - gt;    // keys equal to the threshold
        }
        fixed = rem >= 31 ? digit : ((fixed << B) | digit);
        rem = shift;
        __syncthreads();
    }

    // ---- exact threshold reached: above[h] keys beat it, inbin[h] keys equal it -------------------
    if (tid == 0) {
        int32_t* out = budgets + (size_t)layer * H;
        long long rest = R;
        for (int h = 0; h < H; ++h)
            if (above[h] > (uint32_t)g) rest -= (long long)(above[h] - (uint32_t)g);
        if (rest < 0) rest = 0;
        const long long layer_rows = (long long)H * k;
        long long run = 0;
        for (int h = 0; h < H; ++h) {
            const long long cp = above[h], eq = inbin[h];
            const long long kept = cp > g ? cp : g;             // before any tied key is allotted
            long long open_eq = cp + eq - kept;                  // tied keys the safeguard does not cover
            if (open_eq < 0) open_eq = 0;
            const long long take = open_eq < rest ? open_eq : rest;
            rest -= take;
            long long b = sp + kept + take;
            b = b > n ? n : b;
            out[h] = (int32_t)b;
            // a head that keeps more than its safeguard keeps exactly the keys above the layer's
            // threshold and `take` of those equal to it: the selection need not search
            Threshold th;
            th.key31 = cp >= g ? fixed : kNoThreshold;
            th.need = (uint32_t)take;
            ws.known[(size_t)layer * H + h] = th;
            base[h] = (uint32_t)run;                 // the head's first row inside the layer
            run += b;
            if (run > layer_rows) run = layer_rows;  // whatever the counts were, a layer stays inside its rows
        }
        base[H] = (uint32_t)layer_rows;
    }
    if (!offsets) return;
    __syncthreads();
    // ---- prefix sums and the gather's block table for this layer's rows ---------------------------
    const long long row0 = (long long)layer * H * k;
    for (int h = tid; h < H; h += kAdaThreads) offsets[(size_t)layer * H + h] = row0 + base[h];
    if (tid == 0 && layer == layers - 1) offsets[(size_t)layers * H] = row0 + base[H];
    const long long row1 = row0 + (long long)H * k;
    const long long b_first = (row0 + kCompactRowsPerBlock - 1) / kCompactRowsPerBlock;
    for (long long b = b_first + tid; b * kCompactRowsPerBlock < row1; b += kAdaThreads) {
        const uint32_t p = (uint32_t)(b * kCompactRowsPerBlock - row0);     // row inside the layer
        int lo = 0, hi = H - 1;                    // first head whose rows end beyond p (base[H] > p)
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (base[mid + 1] > p) hi = mid; else lo = mid + 1;
        }
        BlockInfo bi;
        bi.head_end = row0 + base[lo + 1];
        bi.head = layer * H + lo;
        bi.pad = 0;
        block_info[b] = bi;
    }
}

__global__ void ada_uniform_kernel(int32_t* __restrict__ budgets, int count, int32_t value) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) budgets[i] = value;
}

// ---- offsets and gather block table from budgets that only exist on the device -------------
// (for the cases in which nothing is allotted layer-wide and every head gets the same budget)
// One workgroup walks the heads in order, 1024 at a time.  Prefix sums are kept within
// [0, total] and the last offset is total, so that whatever the budgets hold, the selection
// and gather kernels that follow stay inside buffers sized for `total` rows.
__device__ __forceinline__ void ada_block_entry(const int64_t* offsets, int heads, int64_t b, BlockInfo* info);

__global__ __launch_bounds__(kAdaThreads) void ada_offsets_kernel(const int32_t* __restrict__ budgets, int heads,
                                                                  int64_t n, int64_t total,
                                                                  int64_t* offsets,      // written, then read back below
                                                                  int64_t blocks_here, BlockInfo* info) {
    __shared__ long long wave_tot[kAdaWaves];
    __shared__ long long carry_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) { carry_s = 0; offsets[0] = 0; }
    __syncthreads();
    for (int base = 0; base < heads; base += kAdaThreads) {
        const int i = base + tid;
        long long b = i < heads ? (long long)budgets[i] : 0;
        b = b < 0 ? 0 : (b > n ? n : b);
        long long incl = b;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const long long t = __shfl_up(incl, off, 64);
            if (lane >= off) incl += t;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        long long before = carry_s;
        for (int w = 0; w < wave; ++w) before += wave_tot[w];
        if (i < heads) {
            const long long end = before + incl;
            offsets[i + 1] = (i == heads - 1 || end > total) ? total : end;
        }
        __syncthreads();
        if (tid == kAdaThreads - 1) carry_s = before + incl;
        __syncthreads();
    }
    // a table of moderate size is filled right here (blocks_here = 0: a launch of its own does it)
    for (int64_t b = tid; b < blocks_here; b += kAdaThreads) ada_block_entry(offsets, heads, b, info);
}

// block b of the gather starts at row b*kCompactRowsPerBlock: the head owning that row is the
// first one whose rows end beyond it
__device__ __forceinline__ void ada_block_entry(const int64_t* offsets, int heads, int64_t b, BlockInfo* info) {
    const int64_t p = b * kCompactRowsPerBlock;
    int lo = 0, hi = heads - 1;                    // offsets[heads] = total > p, so the answer exists
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (offsets[mid + 1] > p) hi = mid; else lo = mid + 1;
    }
    BlockInfo bi;
    bi.head_end = offsets[lo + 1];
    bi.head = lo;
    bi.pad = 0;
    info[b] = bi;
}

__global__ void ada_blocks_kernel(const int64_t* __restrict__ offsets, int heads, int64_t blocks,
                                  BlockInfo* __restrict__ info) {
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b < blocks) ada_block_entry(offsets, heads, b, info);
}

hipError_t launch_adaptive_plan(const curdkv_ctx* ctx, const int32_t* budgets, int64_t n, int64_t total,
                                int64_t* offsets, BlockInfo* block_info, hipStream_t stream) {
    const int64_t blocks = (total + kCompactRowsPerBlock - 1) / kCompactRowsPerBlock;
    // a table of one entry per thread is filled by the offsets kernel itself; a longer one by a
    // launch of its own (one workgroup walking 6552 entries took 10 us, the extra launch 5)
    const bool small = blocks <= kAdaThreads;
    ada_offsets_kernel<<<dim3(1), kAdaThreads, 0, stream>>>(budgets, ctx->heads, n, total, offsets,
                                                           small ? blocks : 0, block_info);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || small) return e;
    ada_blocks_kernel<<<dim3((unsigned)((blocks + 255) / 256)), 256, 0, stream>>>(offsets, ctx->heads, blocks, block_info);
    return hipGetLastError();
}

// dynamic LDS of ada_resolve_kernel: first the head's own scores; then, in the last workgroup
// of a layer, digit histograms, three per-head arrays and the key list
constexpr size_t kAdaLastLds = ((size_t)kAdaDigWords + 3 * (size_t)kAdaMaxHeads + 8 + 2 * (size_t)kAdaList) * 4;
constexpr size_t kAdaOwnLds = (size_t)kAdaOwn * kAdaThreads * 4;
constexpr size_t kAdaResolveLds = kAdaOwnLds > kAdaLastLds ? kAdaOwnLds : kAdaLastLds;

// The layout above holds for every head count the kernel accepts: digit histograms of at least
// one bit per level, and everything inside the 160 KB of a gfx950 workgroup beside the static
// part (AdaShared and the compiler's own few words).
static_assert((kAdaMaxHeads << 1) <= kAdaDigWords, "a level of one bit must fit the digit histograms");
static_assert(kAdaResolveLds + sizeof(AdaShared) + 1024 <= 160 * 1024, "ada_resolve_kernel's LDS");
static_assert(kAdaSeg <= kAdaList, "one head's segment must fit the list");

hipError_t configure_adaptive(curdkv_ctx* ctx) {
    if ((size_t)ctx->lds_limit < kAdaResolveLds + 4096) return hipSuccess;    // the adaptive calls then report an error
    return hipFuncSetAttribute((const void*)ada_resolve_kernel,
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kAdaResolveLds);
}

size_t adaptive_workspace_bytes(const curdkv_ctx* ctx) {
    return workspace_bytes_for((size_t)ctx->heads, (size_t)ctx->cfg.layers);
}

// ---- the same workspace as a static device array, for callers that cannot allocate ----------
// curdkv_adaptive_budgets_noalloc runs the kernels above on this array instead of a buffer
// from hipMalloc.  Every GPU the library is used on holds its own copy, at its own address,
// from the moment the code object is loaded until the process ends.  On the host the array's
// name is only a handle for hipGetSymbolAddress: the address the kernels are given is the one
// that call returns, looked up once per device at curdkv_create.  Nothing in the array has to
// hold a particular value when a call starts: the kernels set what they read.
constexpr int kScratchMaxHeads = 1024;                 // layers * kv_heads the static workspace covers
constexpr size_t kScratchBytes = workspace_bytes_for(kScratchMaxHeads, kScratchMaxHeads);   // 24 MiB + 32 KiB
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kScratchMaxDevices = 64;
static void* g_scratch_ptr[kScratchMaxDevices];        // device address of `scratch`, per device
static std::mutex g_scratch_mutex;

int adaptive_static_max_heads() { return kScratchMaxHeads; }

// Called with `device` current.  Looks the array's device address up on first use.
hipError_t adaptive_static_workspace_init(int device) {
    if (device < 0 || device >= kScratchMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device]) return hipSuccess;
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = ptr;
    return hipSuccess;
}

void* adaptive_static_workspace(int device) {
    if (device < 0 || device >= kScratchMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    return g_scratch_ptr[device];
}

uint32_t* adaptive_hist_buffer(const curdkv_ctx* ctx, void* workspace) {
    return carve(workspace, (size_t)ctx->heads).hist;
}

const void* adaptive_thresholds(const curdkv_ctx* ctx, void* workspace) {
    return carve(workspace, (size_t)ctx->heads).known;
}

AdaLayerState* adaptive_layer_state(const curdkv_ctx* ctx, void* workspace) {
    return carve(workspace, (size_t)ctx->heads).layer;
}

hipError_t launch_adaptive(const curdkv_ctx* ctx, void* workspace, const float* scores, int64_t n, int32_t k,
                           int32_t sp, int32_t g, long long R, int32_t* budgets, hipStream_t stream,
                           bool hist_ready, int64_t* offsets, BlockInfo* block_info, bool* planned) {
    const int H = ctx->cfg.kv_heads, L = ctx->cfg.layers;
    if (planned) *planned = false;
    if (k <= sp || R <= 0) {           // nothing to allot: k each, or all covered by the safeguard
        const int32_t v = k <= sp ? k : sp + g;
        ada_uniform_kernel<<<dim3((unsigned)((ctx->heads + 255) / 256)), 256, 0, stream>>>(budgets, ctx->heads, v);
        return hipGetLastError();
    }
    if ((size_t)ctx->lds_limit < kAdaResolveLds + 4096 || H > kAdaMaxHeads) return hipErrorInvalidConfiguration;
    const AdaWorkspace ws = carve(workspace, (size_t)ctx->heads);
    if (!hist_ready) {
        ada_hist_kernel<<<dim3((unsigned)ctx->heads), kAdaThreads, 0, stream>>>(scores, n, H, sp, ws.hist, ws.layer);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // the kernel keeps a head's first row inside its layer in 32 bits: a layer of 2^32 rows or
    // more gets its offsets and block table from the general kernels instead
    if ((long long)H * k > 0xFFFFFFFFll) offsets = nullptr;
    ada_resolve_kernel<<<dim3((unsigned)ctx->heads), kAdaThreads, kAdaResolveLds, stream>>>(
        ws, scores, n, H, sp, g, R, k, budgets, offsets, offsets ? block_info : nullptr, L);
    if (planned) *planned = offsets != nullptr;
    return hipGetLastError();
}

}  // namespace curdkv
