// Fused kernel: the whole of Algorithm 1 for one (layer, group) per workgroup --
// project, row-norm squared, combine, normalise, sinks + top-k, gather -- for
// gfx950, bf16 storage, n <= 512 * KPT and sketch width <= 64.
//
// Why one workgroup per head: a head's n scores (128 KB at n = 32768) fit in one
// CU's LDS, so they never have to travel through HBM between the steps, the sum
// that normalises them is a plain workgroup reduction, and the selection reads
// its keys from LDS.  Llama-3-8B / Mistral-7B caches have 32 x 8 = 256 KV heads,
// one per CU of the MI355X.  The phases are:
//   1. eight waves stream the head's K and V once (scan_device.h), scores -> LDS;
//   2. workgroup sum in a fixed order, in double;
//   3. scale, write the normalised scores out (optional), form the sort keys in
//      registers; the LDS array is then free and becomes the index staging area;
//   4. radix select + ordered compaction (select_device.h), indices -> LDS -> HBM;
//   5. gather the chosen rows of K and V into the packed output, 16 bytes per
//      lane, non-temporal.
// All workgroups run phase 1 together, so HBM sees a pure read stream there and
// a pure copy stream in phase 5.

#include "scan_device.h"
#include "select_device.h"

namespace curdkv {

constexpr int kFusedThreads = 512;
constexpr int kFusedWaves = kFusedThreads / 64;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int CB, int KPT, int SRC, bool PROJ>
__global__ __launch_bounds__(kFusedThreads, 2) void fused_kernel(
    const uint4* __restrict__ K, const uint4* __restrict__ V, const uint4* __restrict__ Gp,
    int32_t n, int32_t n_sink, const int64_t* __restrict__ offsets, float* __restrict__ scores_out,
    int32_t* __restrict__ indices, u32x4* __restrict__ K_out, u32x4* __restrict__ V_out,
    uint32_t* __restrict__ hist_out, AdaLayerState* __restrict__ layer_state, int heads_per_layer) {
    extern __shared__ float sc[];                  // [n rounded up to 64]; later int32 stage[n]
    __shared__ SelectShared<kFusedThreads, KPT> sm;
    __shared__ float wsum[kFusedWaves];

    const int head = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint4* Kh = K + (size_t)head * n * 16;   // 16 chunks of 16 bytes per row
    const uint4* Vh = V + (size_t)head * n * 16;

    // ---- 1. scores of the whole head into LDS ---------------------------------------
    float acc;
    {
        SketchRegs<CB> G;
        if (PROJ) load_sketch<CB>(G, Gp + (size_t)head * (CB * 4 * 64), lane);
        const int32_t tiles = (n + kTileTokens - 1) / kTileTokens;
        int32_t per_wave = (tiles + kFusedWaves - 1) / kFusedWaves;
        per_wave += per_wave & 1;                  // whole pairs
        const int32_t t_begin = wave * per_wave;
        const int32_t t_end = t_begin + per_wave < tiles ? t_begin + per_wave : tiles;
        acc = scan_tiles<CB, SRC, PROJ>(G, Kh, Vh, n, t_begin, t_end, sc, 0, lane, scan_phase(head, wave));
    }
    // ---- 2. sum over the head ----------------------------------------------------------
    acc = wave_sum(acc);
    if (lane == 0) wsum[wave] = acc;
    __syncthreads();
    double tot = 0.0;
#pragma unroll
    for (int w = 0; w < kFusedWaves; ++w) tot += (double)wsum[w];
    const bool zero = !(tot > 0.0);
    const float inv = zero ? 0.f : (float)(1.0 / tot);
    const float uniform = (float)(1.0 / (double)n);

    // ---- 3. normalise, write out, keys into registers ----------------------------------
    uint32_t x[KPT];
    float* so = scores_out ? scores_out + (size_t)head * n : nullptr;
#pragma unroll
    for (int it = 0; it < KPT; ++it) {
        const int32_t j = it * kFusedThreads + tid;
        float v = 0.f;
        if (j < n) {
            v = zero ? uniform : sc[j] * inv;
            if (so) so[j] = v;
        }
        x[it] = order_key(v);
    }
    const int32_t s = n_sink < n ? n_sink : n;
    if (hist_out) {
        // for the head-wise budget allocation: the bin12 histogram of this head's candidates,
        // made here because the keys are in registers anyway
        build_hist12<kFusedThreads, KPT>(x, n, s, sm);
        uint32_t* dst = hist_out + (size_t)head * kBins12;
        for (int i = tid; i < kBins12; i += kFusedThreads) dst[i] = sm.hist[i];
        if (tid == 0 && head % heads_per_layer == 0) {       // a fresh count of finished workgroups for the layer
            layer_state[head / heads_per_layer].done = 0;
            layer_state[head / heads_per_layer].overflow = 0;
        }
    }
    const int64_t o0 = offsets[head];
    const int32_t k = (int32_t)(offsets[head + 1] - o0);
    if (k <= 0) return;
    __syncthreads();                               // sc[] has been read by everyone: reuse it

    // ---- 4. selection ------------------------------------------------------------------
    int32_t* stage = reinterpret_cast<int32_t*>(sc);
    int32_t* out = indices + o0;
    select_core<kFusedThreads, KPT>(x, n, s, k, sm, stage, n, out);
    for (int32_t p = tid; p < k; p += kFusedThreads) out[p] = stage[p];

    // ---- 5. gather ---------------------------------------------------------------------
    // The head's K rows first, then its V rows: one source and one destination stream at a
    // time (a plain copy kernel is some 8 % faster on one array than on two interleaved, and
    // this order measured 0.3-0.5 % on the whole kernel), 16 rows in flight per thread.
    constexpr int kRowsPerIter = kFusedThreads / 16;      // 32 rows per instruction
    constexpr int kIters = 16;
    const int c = tid & 15, rsub = tid >> 4;
#pragma unroll 1
    for (int which = 0; which < 2; ++which) {
        const u32x4* src = reinterpret_cast<const u32x4*>(which ? Vh : Kh);
        u32x4* dst = (which ? V_out : K_out) + (size_t)o0 * 16;
#pragma unroll 1
        for (int32_t p0 = 0; p0 < k; p0 += kRowsPerIter * kIters) {
            int32_t idx[kIters];
#pragma unroll
            for (int it = 0; it < kIters; ++it) {
                const int32_t p = p0 + it * kRowsPerIter + rsub;
                idx[it] = stage[p < k ? p : k - 1];
            }
            u32x4 v[kIters];
#pragma unroll
            for (int it = 0; it < kIters; ++it) v[it] = __builtin_nontemporal_load(src + (size_t)idx[it] * 16 + c);
#pragma unroll
            for (int it = 0; it < kIters; ++it) {
                const int32_t p = p0 + it * kRowsPerIter + rsub;
                if (p < k) __builtin_nontemporal_store(v[it], dst + (size_t)p * 16 + c);
            }
        }
    }
}

struct FusedArgs {
    const curdkv_ctx* ctx;
    const void *K, *V;
    int32_t n, n_sink;
    const int64_t* d_offsets;
    float* scores;
    int32_t* indices;
    void *K_out, *V_out;
    uint32_t* hist_out;
    AdaLayerState* layer_state;
    hipStream_t stream;
    int dyn;                 // >= 0: only raise the kernel's dynamic LDS limit to this, no launch
};

template <int CB, int KPT, int SRC, bool PROJ>
static hipError_t one(const FusedArgs& a) {
    if (a.dyn >= 0)
        return hipFuncSetAttribute((const void*)fused_kernel<CB, KPT, SRC, PROJ>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize, a.dyn);
    const size_t lds = (((size_t)a.n + 63) & ~(size_t)63) * 4;
    fused_kernel<CB, KPT, SRC, PROJ><<<dim3((unsigned)a.ctx->heads), kFusedThreads, lds, a.stream>>>(
        (const uint4*)a.K, (const uint4*)a.V, (const uint4*)a.ctx->d_G, a.n, a.n_sink, a.d_offsets,
        a.scores, a.indices, (u32x4*)a.K_out, (u32x4*)a.V_out, a.hist_out, a.layer_state,
        a.ctx->cfg.kv_heads);
    return hipGetLastError();
}

template <int CB, int KPT, bool PROJ>
static hipError_t by_source(const FusedArgs& a, int source) {
    switch (source) {
        case CURDKV_SCORE_KEY: return one<CB, KPT, kSrcK, PROJ>(a);
        case CURDKV_SCORE_VALUE: return one<CB, KPT, kSrcV, PROJ>(a);
        default: return one<CB, KPT, kSrcKV, PROJ>(a);
    }
}

template <int CB, bool PROJ>
static hipError_t by_keys(const FusedArgs& a, int kpt, int source) {
    switch (kpt) {
        case 4: return by_source<CB, 4, PROJ>(a, source);
        case 8: return by_source<CB, 8, PROJ>(a, source);
        case 16: return by_source<CB, 16, PROJ>(a, source);
        case 32: return by_source<CB, 32, PROJ>(a, source);
        default: return by_source<CB, 64, PROJ>(a, source);
    }
}

// keys per thread in the selection: the smallest of 4, 8, 16, 32, 64 that covers n with 512 threads
// (every pass of the selection walks all of a thread's keys, present or not)
static int keys_per_thread(int64_t n) {
    for (int kpt = 4; kpt < 64; kpt *= 2)
        if (n <= (int64_t)kpt * kFusedThreads) return kpt;
    return 64;
}
constexpr int kKeyVariants[5] = {4, 8, 16, 32, 64};

// picks the instantiation for (sketch width, n, score source, projection)
static hipError_t dispatch(const FusedArgs& a, int col_blocks, int kpt, int source, bool proj) {
    if (!proj) return by_keys<2, false>(a, kpt, source);
    if (col_blocks == 1) return by_keys<2, true>(a, kpt, source);
    return by_keys<4, true>(a, kpt, source);
}

hipError_t configure_fused(curdkv_ctx* ctx) {
    const int dyn = ctx->lds_limit - 28 * 1024;      // what the kernels' static LDS leaves
    if (dyn <= 48 * 1024) return hipSuccess;
    if (ctx->cfg.dtype != CURDKV_DTYPE_BF16 || ctx->col_blocks > 2) return hipSuccess;
    FusedArgs a{};
    a.dyn = dyn;
    for (int kpt : kKeyVariants) {
        const hipError_t e = dispatch(a, ctx->col_blocks, kpt, ctx->cfg.score_source, !ctx->cfg.no_projection);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// The fused kernel applies when a head's scores fit in LDS and there are enough
// heads to occupy the GPU with one workgroup each.
bool fused_applicable(const curdkv_ctx* ctx, int64_t n) {
    if (ctx->cfg.dtype != CURDKV_DTYPE_BF16) return false;
    if (ctx->col_blocks > 2 && !ctx->cfg.no_projection) return false;
    if (n > 64 * kFusedThreads) return false;
    const size_t lds = (((size_t)n + 63) & ~(size_t)63) * 4 + sizeof(SelectShared<kFusedThreads, 64>) + 1024;
    if (lds > (size_t)ctx->lds_limit) return false;
    // One workgroup per head and one workgroup per CU at a time: the heads go through the chip
    // in rounds of num_cu, and a last round that is mostly empty costs a full scan time.  Measured
    // at n = 32768: 256, 512, 768 heads are faster fused; 128, 288, 384, 640 heads are faster
    // with the general kernels, 192 is a tie.
    const int64_t rounds = (ctx->heads + ctx->num_cu - 1) / ctx->num_cu;
    return (int64_t)ctx->heads * 10 >= rounds * ctx->num_cu * 9;
}

hipError_t launch_fused(const curdkv_ctx* ctx, const void* K, const void* V, int64_t n, int32_t n_sink,
                        const int64_t* d_offsets, float* scores, int32_t* indices, void* K_out,
                        void* V_out, hipStream_t stream, uint32_t* hist_out, AdaLayerState* layer_state) {
    if (!layer_state) hist_out = nullptr;          // the two go together
    FusedArgs a{ctx, K, V, (int32_t)n, n_sink, d_offsets, scores, indices, K_out, V_out, hist_out, layer_state, stream, -1};
    return dispatch(a, ctx->col_blocks, keys_per_thread(n), ctx->cfg.score_source, !ctx->cfg.no_projection);
}

}  // namespace curdkv
