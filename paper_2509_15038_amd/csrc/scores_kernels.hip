// Scoring kernels: the projection, row-norm-squared, combination and
// normalisation steps of Algorithm 1, for gfx950.
//
// One pass over K and V.  The projection is computed transposed,
//     Y^T = G^T A^T   (A = K_i or V_i),
// with G^T as the MFMA A operand (M = sketch columns) and a tile of token rows
// as the B operand (N = tokens).  In the accumulator layout a lane then owns
// several sketch coordinates of ONE token (its column), so the row-norm squared
// is a sum inside the lane plus one or two lane exchanges.  The projected rows
// never leave registers.  The bf16 inner loop lives in scan_device.h.

#include "scan_device.h"

namespace curdkv {

// Sum the four wave totals of a 256-thread block in a fixed order and store it.  A head
// scored by a single block (few new tokens during generation) can fold the total into the
// head's running sum right here: sum = (restart ? 0 : sum) + total, in double, which is
// what accumulate_sums_kernel computes from one partial.
__device__ __forceinline__ void block_partial_store(float wave_total, float* dst, double* running, int restart) {
    __shared__ float wsum[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) wsum[wave] = wave_total;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float total = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
        *dst = total;
        if (running) *running = (restart ? 0.0 : *running) + (double)total;
    }
}

// ---------------------------------------------------------------------------
// bf16 storage.  Each wave scores a contiguous range of tiles (scan_device.h),
// collecting the scores in its own slice of LDS, and writes them out in one
// burst per stage: no global store sits inside the streaming loop.  Score
// writes that mingle with the read streams of other waves are dear on this
// memory system (1 % of the bytes cost 7 % of the time with 8 KB stages), so the
// stages are as large as LDS allows, normally a wave's whole range, and the
// stores are non-temporal: the workgroups of one round then end, and write,
// at about the same time.
// ---------------------------------------------------------------------------
template <int CB> struct Stage {    // tiles (of 32 tokens) a wave collects between bursts
    static constexpr int kTiles = CB > 4 ? 256 : 128;     // one workgroup per CU: 128 KB; two: 64 KB each
};

template <int CB, int SRC, bool PROJ>
__global__ __launch_bounds__(256, (CB <= 4 ? 2 : 1)) void scores_bf16_kernel(
    const uint4* __restrict__ K, const uint4* __restrict__ V, const uint4* __restrict__ Gp,
    float* __restrict__ scores, float* __restrict__ partial, int64_t n, int blocks_per_head,
    int64_t out_stride, int64_t out_offset, double* __restrict__ sums, int restart) {
    constexpr int kStageTiles = Stage<CB>::kTiles;
    __shared__ float stage[4][kStageTiles * kTileTokens];
    const int head = blockIdx.x / blocks_per_head;
    const int blk = blockIdx.x - head * blocks_per_head;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    SketchRegs<CB> G;
    if (PROJ) load_sketch<CB>(G, Gp + (size_t)head * (CB * 4 * 64), lane);

    const int32_t n32 = (int32_t)n;
    const int32_t tiles = (n32 + kTileTokens - 1) / kTileTokens;
    const int32_t waves_per_head = blocks_per_head * 4;
    int32_t per_wave = (tiles + waves_per_head - 1) / waves_per_head;
    per_wave += per_wave & 1;                                   // whole pairs
    const int32_t t_begin = (blk * 4 + wave) * per_wave;
    const int32_t t_end = t_begin + per_wave < tiles ? t_begin + per_wave : tiles;
    const uint4* Kh = K + (size_t)head * n * 16;                // 16 chunks of 16 bytes per row
    const uint4* Vh = V + (size_t)head * n * 16;
    float* sh = scores + (size_t)head * out_stride + out_offset;   // score of row j goes to sh[j]
    float* mine = stage[wave];
    float acc_sum = 0.f;
    for (int32_t seg = t_begin; seg < t_end; seg += kStageTiles) {
        const int32_t seg_end = seg + kStageTiles < t_end ? seg + kStageTiles : t_end;
        const int32_t r0 = seg * kTileTokens;
        acc_sum += scan_tiles<CB, SRC, PROJ>(G, Kh, Vh, n32, seg, seg_end, mine, r0, lane,
                                             scan_phase(head, blk * 4 + wave));
        const int32_t r1 = seg_end * kTileTokens < n32 ? seg_end * kTileTokens : n32;
        for (int32_t r = r0 + lane; r < r1; r += 64) __builtin_nontemporal_store(mine[r - r0], &sh[r]);
    }
    block_partial_store(wave_sum(acc_sum), partial + (size_t)head * kMaxBlocksPerHead + blk,
                        sums ? sums + head : nullptr, restart);
}

// ---------------------------------------------------------------------------
// fp32 storage: the same structure with mfma_f32_16x16x4f32 (scan_device.h).  A lane's two
// tile buffers take 256 registers, so a SIMD holds one wave and a compute unit one workgroup.
// CB = 16-column blocks of the padded sketch: 2 and 4 keep the sketch in registers, 8 reads it
// from LDS.  Up to 32 columns the kernel is bound by HBM, from 64 on by the fp32 matrix rate
// (4*d*r flop per 1024 bytes of a token's K and V rows is 32 flop/B at r = 64).
// ---------------------------------------------------------------------------
template <int CB> struct StageF32 {
    static constexpr int kTiles = CB > 4 ? 128 : 256;     // 64 KB beside a 64 KB sketch, else 128 KB
};

template <int CB, int SRC, bool PROJ>
__global__ __launch_bounds__(256, 1) void scores_f32_kernel(
    const float4* __restrict__ K, const float4* __restrict__ V, const float4* __restrict__ Gp,
    float* __restrict__ scores, float* __restrict__ partial, int64_t n, int blocks_per_head,
    int64_t out_stride, int64_t out_offset, double* __restrict__ sums, int restart) {
    constexpr bool kInRegs = CB <= 4;             // (PROJ = false comes with CB = 2 and never touches the sketch)
    constexpr int kStageTiles = StageF32<CB>::kTiles;
    __shared__ float stage[4][kStageTiles * kTileTokens];
    __shared__ float4 gs[kInRegs ? 1 : CB * 8 * 64];
    const int head = blockIdx.x / blocks_per_head;
    const int blk = blockIdx.x - head * blocks_per_head;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    const float4* Gh = Gp + (size_t)head * (CB * 8 * 64);
    SketchF32<CB, kInRegs> G;
    if (!PROJ) {
    } else if (kInRegs) {
#pragma unroll
        for (int cb = 0; cb < (kInRegs ? CB : 1); ++cb)
#pragma unroll
            for (int s = 0; s < 8; ++s) G.g[cb][s] = Gh[(cb * 8 + s) * 64 + lane];
    } else {
        for (int i = threadIdx.x; i < CB * 8 * 64; i += 256) gs[i] = Gh[i];
        __syncthreads();
    }

    const int32_t n32 = (int32_t)n;
    const int32_t tiles = (n32 + kTileTokens - 1) / kTileTokens;
    const int32_t waves_per_head = blocks_per_head * 4;
    int32_t per_wave = (tiles + waves_per_head - 1) / waves_per_head;
    per_wave += per_wave & 1;                                   // whole pairs
    const int32_t t_begin = (blk * 4 + wave) * per_wave;
    const int32_t t_end = t_begin + per_wave < tiles ? t_begin + per_wave : tiles;
    const float4* Kh = K + (size_t)head * n * 32;               // 32 chunks of 16 bytes per row
    const float4* Vh = V + (size_t)head * n * 32;
    float* sh = scores + (size_t)head * out_stride + out_offset;
    float* mine = stage[wave];
    float acc_sum = 0.f;
    for (int32_t seg = t_begin; seg < t_end; seg += kStageTiles) {
        const int32_t seg_end = seg + kStageTiles < t_end ? seg + kStageTiles : t_end;
        const int32_t r0 = seg * kTileTokens;
        acc_sum += scan_tiles_f32<CB, kInRegs, SRC, PROJ>(G, gs, Kh, Vh, n32, seg, seg_end, mine, r0, lane,
                                                          scan_phase(head, blk * 4 + wave));
        const int32_t r1 = seg_end * kTileTokens < n32 ? seg_end * kTileTokens : n32;
        for (int32_t r = r0 + lane; r < r1; r += 64) __builtin_nontemporal_store(mine[r - r0], &sh[r]);
    }
    block_partial_store(wave_sum(acc_sum), partial + (size_t)head * kMaxBlocksPerHead + blk,
                        sums ? sums + head : nullptr, restart);
}

// ---------------------------------------------------------------------------
// Normalisation step of Algorithm 1: divide by the sum over all n rows of the head.  The per-block
// partial sums are added in index order in double, so the result does not
// depend on scheduling.  A zero sum gives 1/n everywhere.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void normalise_kernel(float* __restrict__ scores,
                                                        const float* __restrict__ partial,
                                                        int64_t n, int blocks_per_head,
                                                        int chunks_per_head) {
    const int head = blockIdx.x / chunks_per_head;
    const int chunk = blockIdx.x - head * chunks_per_head;
    double tot = 0.0;
    for (int i = 0; i < blocks_per_head; ++i) tot += (double)partial[(size_t)head * kMaxBlocksPerHead + i];
    const bool zero = !(tot > 0.0);
    const float inv = zero ? 0.f : (float)(1.0 / tot);
    const float uniform = (float)(1.0 / (double)n);
    float* sh = scores + (size_t)head * n;
    constexpr int kInFlight = 8;                   // loads issued before the first store
    const int64_t stride = (int64_t)chunks_per_head * blockDim.x;
    for (int64_t j0 = (int64_t)chunk * blockDim.x + threadIdx.x; j0 < n; j0 += kInFlight * stride) {
        float v[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const int64_t j = j0 + u * stride;
            v[u] = j < n ? sh[j] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const int64_t j = j0 + u * stride;
            if (j < n) sh[j] = zero ? uniform : v[u] * inv;
        }
    }
}

// GQA fold: mean over the query heads of a group.  The sum is taken in double,
// where adding a handful of floats is exact, so equal inputs come back unchanged.
__global__ __launch_bounds__(256) void fold_kernel(const float* __restrict__ sq,
                                                   float* __restrict__ out, int64_t n, int group,
                                                   int chunks_per_head) {
    const int head = blockIdx.x / chunks_per_head;
    const int chunk = blockIdx.x - head * chunks_per_head;
    const float* src = sq + (size_t)head * group * n;
    float* dst = out + (size_t)head * n;
    for (int64_t j = (int64_t)chunk * blockDim.x + threadIdx.x; j < n;
         j += (int64_t)chunks_per_head * blockDim.x) {
        double s = 0.0;
        for (int q = 0; q < group; ++q) s += (double)src[(size_t)q * n + j];
        dst[j] = (float)(s / (double)group);
    }
}

// Workgroups per head.  A workgroup should be long-lived (its start-up and the pipeline fill
// are paid per workgroup) and write its scores once, at its end, so the lower bound is what
// makes a wave's share fit its LDS stage.  Above that, the smallest count is taken that fills
// the rounds in which the workgroups pass through the chip to within 3 % of the best
// (measured at n = 32768: 4 per head for 384 heads, 7-8 for 288).  With no more heads than
// compute units the busiest unit decides: workgroups are dealt round-robin, so the cost is
// the number of workgroups a unit gets times their length, and ties go to the fewer, longer
// ones (measured at n = 32768, scoring and normalisation: 32 heads 8 per head, 64 heads 4,
// 128 heads 2; 2 to 5 % faster than filling two workgroups per unit).
// One exception, measured at n = 32768 with the two-per-unit kernel: where one workgroup per
// head already puts four waves on three quarters of the compute units (192 or 224 heads of
// 256, or 448 of 512 places), HBM is saturated by those alone, and one long-lived workgroup per
// head, writing its scores in two bursts, beats any split by 2.5-3.5 % although units stay idle
// (192 heads: 562 us against 576 for four per head; 224: 649 against 671; 448: 1305 against
// 1338).
static int pick_blocks_per_head(const curdkv_ctx* ctx, int64_t n) {
    const int64_t tiles = (n + kTileTokens - 1) / kTileTokens;
    const bool wide = ctx->cfg.dtype == CURDKV_DTYPE_BF16 && ctx->col_blocks > 2 && !ctx->cfg.no_projection;
    const bool f32 = ctx->cfg.dtype == CURDKV_DTYPE_F32;         // one workgroup per compute unit, like the wide kernel
    const int64_t stage = f32 ? (ctx->col_blocks > 2 && !ctx->cfg.no_projection ? StageF32<8>::kTiles : StageF32<4>::kTiles)
                              : (wide ? Stage<8>::kTiles : Stage<4>::kTiles);
    const int64_t slots = (int64_t)ctx->num_cu * ((wide || f32 || ctx->heads <= ctx->num_cu) ? 1 : 2);
    int64_t cap = (tiles + 3) / 4;                                     // at least one tile per wave
    if (cap > kMaxBlocksPerHead) cap = kMaxBlocksPerHead;
    int64_t lo = (tiles + 4 * stage - 1) / (4 * stage);
    if (lo > cap) lo = cap;
    if (lo < 1) lo = 1;
    if (!wide && !f32 && lo <= 2 && ctx->heads <= 2 * (int64_t)ctx->num_cu) {
        const int64_t in_last = ctx->heads - (ctx->heads > ctx->num_cu ? ctx->num_cu : 0);   // heads in the last round
        if (in_last * 4 >= 3 * (int64_t)ctx->num_cu) return 1;
    }
    const int64_t hi = lo + 15 < cap ? lo + 15 : cap;
    auto cost = [&](int64_t b) {                                       // rounds x tiles a wave works through
        const int64_t rounds = ((int64_t)ctx->heads * b + slots - 1) / slots;
        int64_t per_wave = (tiles + 4 * b - 1) / (4 * b);
        per_wave += per_wave & 1;                                      // whole pairs, as in the kernel
        return rounds * per_wave;
    };
    int64_t best = cost(lo);
    for (int64_t b = lo + 1; b <= hi; ++b) best = cost(b) < best ? cost(b) : best;
    for (int64_t b = lo; b <= hi; ++b)
        if (cost(b) * 100 <= best * 103) return (int)b;
    return (int)lo;
}

hipError_t configure_kernels(curdkv_ctx* ctx) {
    (void)ctx;                     // every scoring kernel uses static LDS only
    return hipSuccess;
}

hipError_t launch_scores(const curdkv_ctx* ctx, const void* K, const void* V, int64_t n,
                         float* scores, hipStream_t stream, bool normalise, int* blocks_per_head,
                         int64_t out_stride, int64_t out_offset, double* sums, bool restart,
                         bool* summed) {
    if (out_stride <= 0) out_stride = n;
    const int bph = pick_blocks_per_head(ctx, n);
    if (blocks_per_head) *blocks_per_head = bph;
    if (bph != 1) sums = nullptr;                 // several blocks per head: the caller adds the partials
    if (summed) *summed = sums != nullptr;
    const int rs = restart ? 1 : 0;
    const dim3 grid((unsigned)(ctx->heads * bph)), block(256);
    if (ctx->cfg.dtype == CURDKV_DTYPE_BF16) {
        const uint4* k = (const uint4*)K; const uint4* v = (const uint4*)V; const uint4* g = (const uint4*)ctx->d_G;
        float* part = ctx->d_partial;
#define CURDKV_LAUNCH(CBV, SRCV, PROJV) \
    scores_bf16_kernel<CBV, SRCV, PROJV><<<grid, block, 0, stream>>>(k, v, g, scores, part, n, bph, out_stride, out_offset, sums, rs)
#define CURDKV_BY_SRC(CBV, PROJV)                                                   \
    switch (ctx->cfg.score_source) {                                                \
        case CURDKV_SCORE_KEY: CURDKV_LAUNCH(CBV, kSrcK, PROJV); break;             \
        case CURDKV_SCORE_VALUE: CURDKV_LAUNCH(CBV, kSrcV, PROJV); break;           \
        default: CURDKV_LAUNCH(CBV, kSrcKV, PROJV); break;                          \
    }
        if (ctx->cfg.no_projection) {
            CURDKV_BY_SRC(2, false)
        } else {
            switch (ctx->col_blocks) {   // 16-column MFMA blocks = 2 per 32 padded columns
                case 1: CURDKV_BY_SRC(2, true) break;
                case 2: CURDKV_BY_SRC(4, true) break;
                default: CURDKV_BY_SRC(8, true) break;
            }
        }
#undef CURDKV_BY_SRC
#undef CURDKV_LAUNCH
    } else {
        const float4* k = (const float4*)K; const float4* v = (const float4*)V; const float4* g = (const float4*)ctx->d_G;
        float* part = ctx->d_partial;
#define CURDKV_LAUNCH(CBV, SRCV, PROJV) \
    scores_f32_kernel<CBV, SRCV, PROJV><<<grid, block, 0, stream>>>(k, v, g, scores, part, n, bph, out_stride, out_offset, sums, rs)
#define CURDKV_BY_SRC(CBV, PROJV)                                                   \
    switch (ctx->cfg.score_source) {                                                \
        case CURDKV_SCORE_KEY: CURDKV_LAUNCH(CBV, kSrcK, PROJV); break;             \
        case CURDKV_SCORE_VALUE: CURDKV_LAUNCH(CBV, kSrcV, PROJV); break;           \
        default: CURDKV_LAUNCH(CBV, kSrcKV, PROJV); break;                          \
    }
        if (ctx->cfg.no_projection) {
            CURDKV_BY_SRC(2, false)
        } else {
            switch (ctx->col_blocks) {   // 16-column MFMA blocks = 2 per 32 padded columns
                case 1: CURDKV_BY_SRC(2, true) break;
                case 2: CURDKV_BY_SRC(4, true) break;
                default: CURDKV_BY_SRC(8, true) break;
            }
        }
#undef CURDKV_BY_SRC
#undef CURDKV_LAUNCH
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !normalise) return e;
    int64_t nb = (n + 1023) / 1024;
    if (nb > 64) nb = 64;
    normalise_kernel<<<dim3((unsigned)(nb * ctx->heads)), 256, 0, stream>>>(scores, ctx->d_partial, n, bph, (int)nb);
    return hipGetLastError();
}

// Decode-phase bookkeeping: running sum of a head's un-normalised scores, and the
// normalisation by it.  Partial sums are added in index order, in double.
__global__ void accumulate_sums_kernel(const float* __restrict__ partial, int blocks_per_head,
                                       double* __restrict__ sums, int heads, int reset) {
    const int head = blockIdx.x * blockDim.x + threadIdx.x;
    if (head >= heads) return;
    double tot = reset ? 0.0 : sums[head];
    for (int i = 0; i < blocks_per_head; ++i) tot += (double)partial[(size_t)head * kMaxBlocksPerHead + i];
    sums[head] = tot;
}

__global__ __launch_bounds__(256) void normalise_sums_kernel(const float* __restrict__ raw,
                                                             const double* __restrict__ sums,
                                                             int64_t stride, int64_t n,
                                                             float* __restrict__ scores,
                                                             int chunks_per_head) {
    const int head = blockIdx.x / chunks_per_head;
    const int chunk = blockIdx.x - head * chunks_per_head;
    const double tot = sums[head];
    const bool zero = !(tot > 0.0);
    const float inv = zero ? 0.f : (float)(1.0 / tot);
    const float uniform = (float)(1.0 / (double)n);
    const float* src = raw + (size_t)head * stride;
    float* dst = scores + (size_t)head * n;
    for (int64_t j = (int64_t)chunk * blockDim.x + threadIdx.x; j < n;
         j += (int64_t)chunks_per_head * blockDim.x)
        dst[j] = zero ? uniform : src[j] * inv;
}

hipError_t launch_accumulate(const curdkv_ctx* ctx, int blocks_per_head, double* sums, bool reset,
                             hipStream_t stream) {
    accumulate_sums_kernel<<<dim3((unsigned)((ctx->heads + 255) / 256)), 256, 0, stream>>>(
        ctx->d_partial, blocks_per_head, sums, ctx->heads, reset ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_normalise_sums(const curdkv_ctx* ctx, const float* raw, const double* sums,
                                 int64_t stride, int64_t n, float* scores, hipStream_t stream) {
    int64_t nb = (n + 1023) / 1024;
    if (nb > 64) nb = 64;
    normalise_sums_kernel<<<dim3((unsigned)(nb * ctx->heads)), 256, 0, stream>>>(raw, sums, stride, n, scores, (int)nb);
    return hipGetLastError();
}

hipError_t launch_fold(const curdkv_ctx* ctx, const float* scores_q, int64_t n, float* scores,
                       hipStream_t stream) {
    int64_t nb = (n + 1023) / 1024;
    if (nb > 64) nb = 64;
    fold_kernel<<<dim3((unsigned)(nb * ctx->heads)), 256, 0, stream>>>(scores_q, scores, n, ctx->cfg.group_size, (int)nb);
    return hipGetLastError();
}

}  // namespace curdkv
