// Selection kernel: Algorithm 1, lines "Preserve first s tokens as sink
// indices", "Select top-(k-s) indices from l[s:]" and "Combine", for gfx950.
//
// One 1024-thread workgroup per (layer, group).  The scores are turned into
// order-preserving 32-bit keys and, when they fit, held in LDS for the whole
// kernel.  A most-significant-digit radix select (four 8-bit digits) finds the
// key T of the (k-s)-th largest candidate and how many keys equal to T are
// still needed; an ordered compaction then writes, in ascending token order,
// the sinks, every candidate above T, and the first `need` candidates equal to
// T.  That realises "larger score first, then smaller index" exactly.

#include "curdkv_internal.h"

namespace curdkv {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kHistRep = 8;                       // replicated bins to thin out LDS atomic collisions
constexpr int kSelFixedLds = 256 * kHistRep * 4;  // histogram bytes in dynamic LDS

__device__ __forceinline__ uint32_t order_key(float x) {
    x = x + 0.0f;                                 // -0 -> +0
    const uint32_t b = __float_as_uint(x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

template <bool LDS_KEYS>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const float* __restrict__ scores,
                                                             int64_t n, int32_t n_sink,
                                                             const int64_t* __restrict__ offsets,
                                                             int32_t* __restrict__ indices) {
    extern __shared__ uint32_t dyn[];
    uint32_t* hist = dyn;                         // [256][kHistRep]
    uint32_t* keys = dyn + 256 * kHistRep;        // [n] when LDS_KEYS
    __shared__ uint32_t bin_count[256];
    __shared__ uint32_t sh_digit, sh_want;
    __shared__ uint32_t wave_gt[kSelWaves], wave_eq[kSelWaves];

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

    if (LDS_KEYS) {
        for (int64_t j = tid; j < n; j += kSelThreads) keys[j] = order_key(sc[j]);
    }
    auto key_at = [&](int64_t j) -> uint32_t { return LDS_KEYS ? keys[j] : order_key(sc[j]); };

    // ---- radix select: T = the m-th largest key among tokens [s, n) ----------
    uint32_t prefix = 0, mask = 0, want = (uint32_t)m;
    const int64_t span = n - s;
    const int64_t iters = (span + kSelThreads - 1) / kSelThreads;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        for (int i = tid; i < 256 * kHistRep; i += kSelThreads) hist[i] = 0;
        __syncthreads();                           // also orders the key stores above
        for (int64_t it = 0; it < iters; ++it) {
            const int64_t j = s + it * kSelThreads + tid;
            bool valid = j < n;
            uint32_t digit = 0;
            if (valid) {
                const uint32_t key = key_at(j);
                valid = (key & mask) == prefix;
                digit = (key >> shift) & 255u;
            }
            if (pass == 0) {
                // leading digits are few (sign and high exponent bits): count them per
                // wave with ballots, one LDS atomic per distinct digit
                uint64_t active = __ballot(valid);
                while (active) {
                    const int leader = __ffsll((unsigned long long)active) - 1;
                    const uint32_t d0 = __shfl(digit, leader, 64);
                    const uint64_t same = __ballot(valid && digit == d0);
                    if (lane == leader) atomicAdd(&hist[d0 * kHistRep + (wave & (kHistRep - 1))], (uint32_t)__popcll(same));
                    if (digit == d0) valid = false;
                    active &= ~same;
                }
            } else if (valid) {
                atomicAdd(&hist[digit * kHistRep + (lane & (kHistRep - 1))], 1u);
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
        prefix |= sh_digit << shift;
        mask |= 255u << shift;
        want = sh_want;
        __syncthreads();                           // sh_* are rewritten next pass
    }
    const uint32_t T = prefix;
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
    if (lane == 0) { wave_gt[wave] = cg; wave_eq[wave] = ce; }
    __syncthreads();
    uint32_t gt_before = 0, eq_before = 0;
    for (int w = 0; w < wave; ++w) { gt_before += wave_gt[w]; eq_before += wave_eq[w]; }

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

static size_t select_lds_bytes(int64_t n) { return (size_t)kSelFixedLds + (size_t)n * 4; }
constexpr size_t kSelStaticLds = 2048;   // bin counts, flags and wave counters, rounded up

hipError_t configure_select(curdkv_ctx* ctx) {
    const int dyn = ctx->lds_limit - (int)kSelStaticLds;
    if (dyn <= 48 * 1024) return hipSuccess;
    return hipFuncSetAttribute((const void*)select_kernel<true>,
                               hipFuncAttributeMaxDynamicSharedMemorySize, dyn);
}

hipError_t launch_select(const curdkv_ctx* ctx, const float* scores, int64_t n, int32_t n_sink,
                         const int64_t* d_offsets, int32_t* indices, hipStream_t stream) {
    // static LDS of the kernel: bin_count + flags + wave counters
    const bool fits = select_lds_bytes(n) + kSelStaticLds <= (size_t)ctx->lds_limit;
    if (fits) {
        const size_t lds = select_lds_bytes(n);
        select_kernel<true><<<dim3((unsigned)ctx->heads), kSelThreads, lds, stream>>>(scores, n, n_sink, d_offsets, indices);
    } else {
        select_kernel<false><<<dim3((unsigned)ctx->heads), kSelThreads, kSelFixedLds, stream>>>(scores, n, n_sink, d_offsets, indices);
    }
    return hipGetLastError();
}

}  // namespace curdkv
