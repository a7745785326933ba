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
// (12 + 12 + 8 bits for up to 8 heads).  Each level is two launches:
//   * ada_hist_kernel, one workgroup per (layer, head) so that the whole GPU
//     streams the scores: histogram, in LDS, of the next bits of the keys that
//     match the prefix decided so far, written to a workspace;
//   * ada_resolve_kernel, one workgroup per layer: loads the H histograms, finds
//     the bin in which the sum above reaches R, extends the prefix, and at the
//     last level allots keys equal to the threshold head by head and writes the
//     budgets.
// No token order is needed anywhere.

#include <mutex>

#include "select_device.h"

namespace curdkv {

constexpr int kAdaThreads = 1024;
constexpr int kAdaWaves = kAdaThreads / 64;
constexpr int kAdaU = 8;                          // scores per thread per chunk
constexpr int kAdaMaxBins = 4096;

struct AdaLayerState {                            // per layer, in the workspace
    uint32_t prefix;                              // decided high bits of the threshold key
    uint32_t pad;
};

__global__ __launch_bounds__(kAdaThreads) void ada_hist_kernel(
    const float* __restrict__ scores, int64_t n, int H, int32_t sp, int decided, int B,
    const AdaLayerState* __restrict__ state, uint32_t* __restrict__ ws_hist) {
    __shared__ uint32_t hist[kAdaMaxBins];
    const int head = blockIdx.x, layer = head / H;
    const int tid = threadIdx.x;
    const int NB = 1 << B;
    const int shift = 32 - decided - B;
    const uint32_t dmask = (uint32_t)NB - 1u;
    const uint32_t prefix = decided ? state[layer].prefix : 0u;
    const float* sc = scores + (size_t)head * n;
    for (int i = tid; i < NB; i += kAdaThreads) hist[i] = 0;
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
            if (j >= sp && j < n) {
                const uint32_t key = order_key(cur[u]);
                if (decided == 0 || (key >> (32 - decided)) == prefix)
                    atomicAdd(&hist[(key >> shift) & dmask], 1u);
            }
        }
#pragma unroll
        for (int u = 0; u < kAdaU; ++u) cur[u] = nxt[u];
    }
    __syncthreads();
    uint32_t* dst = ws_hist + (size_t)head * kAdaMaxBins;
    for (int i = tid; i < NB; i += kAdaThreads) dst[i] = hist[i];
}

constexpr int kAdaHeadsAtOnce = 8;

struct AdaShared {
    uint32_t wave_tot[kAdaHeadsAtOnce][kAdaWaves];
    unsigned long long best;                      // first position (bins counted from the top) reaching R
};

__global__ __launch_bounds__(kAdaThreads) void ada_resolve_kernel(
    const uint32_t* __restrict__ ws_hist, int H, int decided, int B, int32_t sp, int32_t g, long long R,
    AdaLayerState* __restrict__ state, uint32_t* __restrict__ ws_above, int32_t* __restrict__ budgets) {
    extern __shared__ __align__(16) uint32_t dyn[];
    const int NB = 1 << B;
    uint32_t* hist = dyn;                          // [H][NB]
    uint32_t* above = dyn + (size_t)H * NB;        // [H] keys above the prefix decided so far
    uint32_t* wave_excl = above + H;               // [H][kAdaWaves]
    __shared__ AdaShared sm;

    const int layer = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    {   // the H histograms, 16 bytes per load and eight loads in flight per thread (one load at a
        // time, each waited for, made this copy most of the kernel's 25 us); NB >= 4
        const int quads = (H * NB) >> 2;
        constexpr int kInFlight = 8;
        for (int q0 = tid; q0 < quads; q0 += kInFlight * kAdaThreads) {
            uint4 v[kInFlight];
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const int q = q0 + u * kAdaThreads;
                const int e = (q < quads ? q : q0) << 2;              // element number h*NB + i
                const int h = e >> B, i = e & (NB - 1);
                v[u] = *reinterpret_cast<const uint4*>(ws_hist + ((size_t)layer * H + h) * kAdaMaxBins + i);
            }
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const int q = q0 + u * kAdaThreads;
                if (q < quads) *reinterpret_cast<uint4*>(hist + ((size_t)q << 2)) = v[u];
            }
        }
    }
    for (int h = tid; h < H; h += kAdaThreads) above[h] = decided ? ws_above[(size_t)layer * H + h] : 0u;
    if (tid == 0) sm.best = ~0ull;
    __syncthreads();

    // ---- find the bin where sum_h max(0, c_h - g) reaches R ---------------------------------
    // kAdaHeadsAtOnce heads go through the workgroup-wide prefix sums together, so a layer of
    // eight heads costs one barrier instead of sixteen (the kernel is latency-bound: one
    // workgroup per layer).
    const int per = NB >= kAdaThreads ? NB / kAdaThreads : 1;           // bins per thread, from the top
    unsigned long long E[4] = {0, 0, 0, 0};
    for (int h0 = 0; h0 < H; h0 += kAdaHeadsAtOnce) {
        uint32_t c[kAdaHeadsAtOnce][4], tot[kAdaHeadsAtOnce], incl[kAdaHeadsAtOnce];
#pragma unroll
        for (int j = 0; j < kAdaHeadsAtOnce; ++j) {
            const int h = h0 + j;
            tot[j] = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int pos = tid * per + i;
                c[j][i] = (h < H && i < per && pos < NB) ? hist[(size_t)h * NB + (NB - 1 - pos)] : 0u;
                tot[j] += c[j][i];
            }
            incl[j] = tot[j];
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
#pragma unroll
        for (int j = 0; j < kAdaHeadsAtOnce; ++j) {
            const int h = h0 + j;
            if (h >= H) break;
            uint32_t before = 0;
            for (int w = 0; w < wave; ++w) before += sm.wave_tot[j][w];
            if (lane == 0) wave_excl[h * kAdaWaves + wave] = before;
            uint32_t run = above[h] + before + incl[j] - tot[j];       // keys of head h in higher bins
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                run += c[j][i];
                if (i < per && run > (uint32_t)g) E[i] += run - (uint32_t)g;
            }
        }
        __syncthreads();                                        // wave_tot is reused by the next heads
    }
    {
        // E grows with the position, so every thread beyond the crossing qualifies: the minimum is
        // taken inside each wave first, one atomic per wave instead of one per thread
        uint32_t mine = 0xFFFFFFFFu;
#pragma unroll
        for (int i = 3; i >= 0; --i) {
            const int pos = tid * per + i;
            if (i < per && pos < NB && E[i] >= (unsigned long long)R) mine = (uint32_t)pos;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const uint32_t o = __shfl_xor(mine, off, 64);
            mine = o < mine ? o : mine;
        }
        if (lane == 0 && mine != 0xFFFFFFFFu) atomicMin(&sm.best, (unsigned long long)mine);
    }
    __syncthreads();
    const int best = (int)sm.best;                              // exists: the lowest bin reaches R
    // ---- keys above the chosen bin join `above`; done by the wave that owns the bin ----------
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
    __syncthreads();
    const uint32_t digit = (uint32_t)(NB - 1 - best);
    if (decided + B < 32) {                                     // more levels follow
        if (tid == 0) state[layer].prefix = decided ? ((state[layer].prefix << B) | digit) : digit;
        for (int h = tid; h < H; h += kAdaThreads) ws_above[(size_t)layer * H + h] = above[h];
        return;
    }
    // ---- exact threshold reached: above[h] keys beat it, hist[h][digit] keys equal it ----------
    if (tid == 0) {
        int32_t* out = budgets + (size_t)layer * H;
        long long rest = R;
        for (int h = 0; h < H; ++h)
            if (above[h] > (uint32_t)g) rest -= (long long)(above[h] - (uint32_t)g);
        for (int h = 0; h < H; ++h) {
            const long long cp = above[h], eq = hist[(size_t)h * NB + digit];
            const long long kept = cp > g ? cp : g;             // before any tied key is allotted
            long long open_eq = cp + eq - kept;                  // tied keys the safeguard does not cover
            if (open_eq < 0) open_eq = 0;
            const long long take = open_eq < rest ? open_eq : rest;
            rest -= take;
            out[h] = (int32_t)(sp + kept + take);
        }
    }
}

__global__ void ada_uniform_kernel(int32_t* __restrict__ budgets, int count, int32_t value) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) budgets[i] = value;
}

// ---- offsets and gather block table from budgets that only exist on the device -------------
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

// bits per level so that H histograms fit in 128 KB of LDS
static int level_bits(int H) {
    int bits = 12;
    while (bits > 3 && ((size_t)H << bits) * 4 > 128 * 1024) --bits;
    return bits;
}

hipError_t configure_adaptive(curdkv_ctx* ctx) {
    const int dyn = ctx->lds_limit - 8 * 1024;
    if (dyn <= 48 * 1024) return hipSuccess;
    return hipFuncSetAttribute((const void*)ada_resolve_kernel,
                               hipFuncAttributeMaxDynamicSharedMemorySize, dyn);
}

// Workspace of the allocation for `heads` (layer, group) pairs in `layers` layers: the per-head
// histograms, the per-head counts above the decided prefix, the per-layer prefix.
static constexpr size_t workspace_bytes_for(size_t heads, size_t layers) {
    return heads * kAdaMaxBins * 4 + heads * 4 + layers * sizeof(AdaLayerState);
}

size_t adaptive_workspace_bytes(const curdkv_ctx* ctx) {
    return workspace_bytes_for((size_t)ctx->heads, (size_t)ctx->cfg.layers);
}

// ---- the same workspace as a static device array, for callers that cannot allocate ----------
// curdkv_adaptive_budgets_noalloc runs the kernels above on this array instead of a buffer
// from hipMalloc.  Every GPU the library is used on holds its own copy, at its own address,
// from the moment the code object is loaded until the process ends.  On the host the array's
// name is only a handle for hipGetSymbolAddress: the address the kernels are given is the one
// that call returns, looked up once per device at curdkv_create.
constexpr int kScratchMaxHeads = 1024;                 // layers * kv_heads the static workspace covers
constexpr size_t kScratchBytes = workspace_bytes_for(kScratchMaxHeads, kScratchMaxHeads);   // 16 MiB + 12 KiB
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

hipError_t launch_adaptive(const curdkv_ctx* ctx, void* workspace, const float* scores, int64_t n, int32_t k,
                           int32_t sp, int32_t g, long long R, int32_t* budgets, hipStream_t stream) {
    const int H = ctx->cfg.kv_heads, L = ctx->cfg.layers;
    if (k <= sp || R <= 0) {           // nothing to allot: k each, or all covered by the safeguard
        const int32_t v = k <= sp ? k : sp + g;
        ada_uniform_kernel<<<dim3((unsigned)((ctx->heads + 255) / 256)), 256, 0, stream>>>(budgets, ctx->heads, v);
        return hipGetLastError();
    }
    uint32_t* ws_hist = reinterpret_cast<uint32_t*>(workspace);
    uint32_t* ws_above = ws_hist + (size_t)ctx->heads * kAdaMaxBins;
    AdaLayerState* state = reinterpret_cast<AdaLayerState*>(ws_above + ctx->heads);
    const int bits = level_bits(H);
    for (int decided = 0; decided < 32;) {
        const int B = bits < 32 - decided ? bits : 32 - decided;
        ada_hist_kernel<<<dim3((unsigned)ctx->heads), kAdaThreads, 0, stream>>>(scores, n, H, sp, decided, B, state, ws_hist);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        const size_t lds = (((size_t)H << B) + (size_t)H + (size_t)H * kAdaWaves) * 4;
        ada_resolve_kernel<<<dim3((unsigned)L), kAdaThreads, lds, stream>>>(ws_hist, H, decided, B, sp, g, R, state, ws_above, budgets);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        decided += B;
    }
    return hipSuccess;
}

}  // namespace curdkv
