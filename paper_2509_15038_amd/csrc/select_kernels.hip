// Selection kernels: Algorithm 1, lines "Preserve first s tokens as sink
// indices", "Select top-(k-s) indices from l[s:]" and "Combine", for gfx950.
// One 1024-thread workgroup per (layer, group).  The method is described in
// select_device.h; this file holds the kernels and their launcher.

#include "select_device.h"

namespace curdkv {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelFixedLds = 256 * kHistRep * 4;  // histogram bytes in the streaming kernel's dynamic LDS

// ---------------------------------------------------------------------------
// Streaming variant for n too large for the register-resident one: every pass
// re-reads the head's scores from memory (they sit in L2 / Infinity Cache).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kSelThreads) void select_stream_kernel(const float* __restrict__ scores,
                                                             int64_t n, int32_t n_sink,
                                                             const int64_t* __restrict__ offsets,
                                                             int32_t* __restrict__ indices) {
    extern __shared__ uint32_t dyn[];
    uint32_t* hist = dyn;                         // [256][kHistRep]
    __shared__ uint32_t bin_count[256];
    __shared__ uint32_t sh_digit, sh_want;
    __shared__ uint32_t wave_a[kSelWaves], wave_b[kSelWaves];

    const int head = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t o0 = offsets[head];
    const int64_t k = offsets[head + 1] - o0;
    int32_t* out = indices + o0;
    const float* sc = scores + (size_t)head * n;
    const int64_t s = n_sink;

    if (k <= 0) return;
    if (k <= s) {                                  // budget inside the sink block: tokens 0..k-1
        for (int64_t j = tid; j < k; j += kSelThreads) out[j] = (int32_t)j;
        return;
    }
    for (int64_t j = tid; j < s; j += kSelThreads) out[j] = (int32_t)j;
    const int64_t m = k - s;                       // picks among tokens [s, n)
    if (m >= n - s) {                              // everything is kept
        for (int64_t j = s + tid; j < n; j += kSelThreads) out[j] = (int32_t)j;
        return;
    }

    // ---- the range [kmin, kmax] of the candidates --------------------------------
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
    {
        const int64_t iters = (n + kSelThreads - 1) / kSelThreads;
        for (int64_t it = 0; it < iters; it += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t j = (it + u) * kSelThreads + tid;
                v[u] = j < n ? sc[j] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t j = (it + u) * kSelThreads + tid;
                if (j < n) {
                    const uint32_t key = order_key(v[u]);
                    if (j >= s) { kmin = key < kmin ? key : kmin; kmax = key > kmax ? key : kmax; }
                }
            }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const uint32_t a = __shfl_xor(kmin, off, 64), b = __shfl_xor(kmax, off, 64);
        kmin = a < kmin ? a : kmin;
        kmax = b > kmax ? b : kmax;
    }
    if (lane == 0) { wave_a[wave] = kmin; wave_b[wave] = kmax; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
        kmin = wave_a[w] < kmin ? wave_a[w] : kmin;
        kmax = wave_b[w] > kmax ? wave_b[w] : kmax;
    }
    auto key_at = [&](int64_t j) -> uint32_t { return order_key(sc[j]); };

    // ---- radix select on x = key - kmin: T = the m-th largest among tokens [s, n) ----
    const uint32_t range = kmax - kmin;
    int rem = range ? 32 - __clz(range) : 0;       // bits of x not yet decided
    uint32_t fixed = 0;                            // decided high part: x >> rem
    uint32_t want = (uint32_t)m;
    const int64_t span = n - s;
    const int64_t iters = (span + kSelThreads - 1) / kSelThreads;
    bool first = true;
    while (rem > 0) {
        const int w = rem < 8 ? rem : 8;
        const int shift = rem - w;
        const uint32_t dmask = (1u << w) - 1u;
        for (int i = tid; i < 256 * kHistRep; i += kSelThreads) hist[i] = 0;
        __syncthreads();
        for (int64_t it = 0; it < iters; ++it) {
            const int64_t j = s + it * kSelThreads + tid;
            if (j < n) {
                const uint32_t x = key_at(j) - kmin;
                if (first || (x >> rem) == fixed)
                    atomicAdd(&hist[((x >> shift) & dmask) * kHistRep + (lane & (kHistRep - 1))], 1u);
            }
        }
        __syncthreads();
        if (tid < 256) {
            uint32_t c = 0;
#pragma unroll
            for (int r = 0; r < kHistRep; ++r) c += hist[tid * kHistRep + r];
            bin_count[tid] = c;
        }
        __syncthreads();
        if (wave == 0) {
            // lane L looks at bins 255-4L .. 252-4L (descending); find the bin where the
            // count from the top reaches `want`
            uint32_t c[4], tot = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) { c[i] = bin_count[255 - 4 * lane - i]; tot += c[i]; }
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
                    if (want <= run + c[i]) { sh_digit = 255 - 4 * lane - i; sh_want = want - run; break; }
                    run += c[i];
                }
            }
        }
        __syncthreads();
        fixed = (fixed << w) | sh_digit;
        want = sh_want;
        rem = shift;
        first = false;
        __syncthreads();                           // sh_* are rewritten next pass
    }
    const uint32_t T = kmin + fixed;
    const uint32_t need = want;                    // keys equal to T still to be kept (>= 1)

    // ---- ordered compaction ----------------------------------------------------
    // wave w owns the contiguous token range [w*chunk, (w+1)*chunk)
    int64_t chunk = (n + kSelWaves - 1) / kSelWaves;
    chunk = (chunk + 63) & ~(int64_t)63;
    const int64_t j0 = (int64_t)wave * chunk;
    const int64_t j1 = j0 + chunk < n ? j0 + chunk : n;
    uint32_t cg = 0, ce = 0;
    for (int64_t j = j0 + lane; j < j1; j += 64) {
        if (j >= s) {
            const uint32_t key = key_at(j);
            cg += key > T;
            ce += key == T;
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        cg += __shfl_xor(cg, off, 64);
        ce += __shfl_xor(ce, off, 64);
    }
    __syncthreads();                               // wave_a / wave_b held the key range
    if (lane == 0) { wave_a[wave] = cg; wave_b[wave] = ce; }
    __syncthreads();
    uint32_t gt_before = 0, eq_before = 0;
    for (int w = 0; w < wave; ++w) { gt_before += wave_a[w]; eq_before += wave_b[w]; }

    const uint64_t lt_mask = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    for (int64_t jb = j0; jb < j1; jb += 64) {
        const int64_t j = jb + lane;
        bool g = false, e = false;
        if (j < j1 && j >= s) {
            const uint32_t key = key_at(j);
            g = key > T;
            e = key == T;
        }
        const uint64_t bg = __ballot(g), be = __ballot(e);
        const uint32_t pg = gt_before + (uint32_t)__popcll(bg & lt_mask);
        const uint32_t pe = eq_before + (uint32_t)__popcll(be & lt_mask);
        // positions stay below k by construction; the comparison keeps a write inside
        // the group's slice even if the scores were changed under the kernel
        const int64_t pos = s + pg + (pe < need ? pe : need);
        if ((g || (e && pe < need)) && pos < k) out[pos] = (int32_t)j;
        gt_before += (uint32_t)__popcll(bg);
        eq_before += (uint32_t)__popcll(be);
    }
}

// ---------------------------------------------------------------------------
// Register-resident variant (select_device.h) for n <= 1024 * KPT.  The chosen
// indices are collected in LDS and written out coalesced.
// ---------------------------------------------------------------------------
template <int KPT>
__global__ __launch_bounds__(kSelThreads) void select_reg_kernel(const float* __restrict__ scores,
                                                                 int32_t n, int32_t n_sink,
                                                                 const int64_t* __restrict__ offsets,
                                                                 int32_t* __restrict__ indices, int32_t cap) {
    extern __shared__ int32_t stage[];             // [cap]
    __shared__ SelectShared<kSelThreads, KPT> sm;
    const int head = blockIdx.x;
    const int tid = threadIdx.x;
    const int64_t o0 = offsets[head];
    const int32_t k = (int32_t)(offsets[head + 1] - o0);
    if (k <= 0) return;
    int32_t* out = indices + o0;
    const float* sc = scores + (size_t)head * n;
    const int32_t s = n_sink < n ? n_sink : n;

    uint32_t x[KPT];
    {
        float v[KPT];
#pragma unroll
        for (int it = 0; it < KPT; ++it) {
            const int32_t j = it * kSelThreads + tid;
            v[it] = j < n ? sc[j] : 0.f;
        }
#pragma unroll
        for (int it = 0; it < KPT; ++it) x[it] = order_key(v[it]);
    }
    select_core<kSelThreads, KPT>(x, n, s, k, sm, stage, cap, out);
    const int32_t staged = k < cap ? k : cap;
    for (int32_t p = tid; p < staged; p += kSelThreads) out[p] = stage[p];
}

template <int KPT>
static hipError_t launch_reg(const curdkv_ctx* ctx, const float* scores, int32_t n, int32_t n_sink,
                             const int64_t* d_offsets, int32_t* indices, hipStream_t stream) {
    const size_t fixed = sizeof(SelectShared<kSelThreads, KPT>) + 256;
    int64_t cap = ((int64_t)ctx->lds_limit - (int64_t)fixed) / 4;
    if (cap > n) cap = n;
    if (cap < 0) cap = 0;
    select_reg_kernel<KPT><<<dim3((unsigned)ctx->heads), kSelThreads, (size_t)cap * 4, stream>>>(
        scores, n, n_sink, d_offsets, indices, (int32_t)cap);
    return hipGetLastError();
}

hipError_t configure_select(curdkv_ctx* ctx) {
    const int dyn = ctx->lds_limit - 16 * 1024;
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

hipError_t launch_select(const curdkv_ctx* ctx, const float* scores, int64_t n, int32_t n_sink,
                         const int64_t* d_offsets, int32_t* indices, hipStream_t stream) {
    const int32_t n32 = (int32_t)n;
    if (n <= 4 * kSelThreads) return launch_reg<4>(ctx, scores, n32, n_sink, d_offsets, indices, stream);
    if (n <= 8 * kSelThreads) return launch_reg<8>(ctx, scores, n32, n_sink, d_offsets, indices, stream);
    if (n <= 16 * kSelThreads) return launch_reg<16>(ctx, scores, n32, n_sink, d_offsets, indices, stream);
    if (n <= 32 * kSelThreads) return launch_reg<32>(ctx, scores, n32, n_sink, d_offsets, indices, stream);
    if (n <= 36 * kSelThreads) return launch_reg<36>(ctx, scores, n32, n_sink, d_offsets, indices, stream);
    select_stream_kernel<<<dim3((unsigned)ctx->heads), kSelThreads, kSelFixedLds, stream>>>(
        scores, n, n_sink, d_offsets, indices);
    return hipGetLastError();
}

}  // namespace curdkv
