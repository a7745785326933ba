// Gather-compact kernel: Algorithm 1, last line, K'_i = K_i[S_i], V'_i = V_i[S_i]
// (rows of the original cache), for gfx950.
//
// The packed output is one long list of rows; work is split by output row, not
// by head, so ragged budgets balance by themselves.  A row is copied by a group
// of lanes, 16 bytes per lane, which makes every load and store of a wave cover
// whole rows: 256-byte rows are read at scattered (ascending) addresses and
// written contiguously.

#include "curdkv_internal.h"

namespace curdkv {

constexpr int kRowsPerBlock = 64;

// first head h with offsets[h+1] > p  (offsets non-decreasing, offsets[heads] > p)
__device__ __forceinline__ int head_of_row(const int64_t* __restrict__ offsets, int heads, int64_t p) {
    int lo = 0, hi = heads - 1;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (offsets[mid + 1] > p) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// ROW_U4: 16-byte chunks per row (16 for bf16 d=128, 32 for fp32 d=128)
template <int ROW_U4>
__global__ __launch_bounds__(256) void compact_kernel(
    const uint4* __restrict__ K, const uint4* __restrict__ V, int64_t n,
    const int32_t* __restrict__ indices, const int64_t* __restrict__ offsets, int heads,
    int64_t total, uint4* __restrict__ K_out, uint4* __restrict__ V_out) {
    constexpr int kRowsPerIter = 256 / ROW_U4;
    constexpr int kIters = kRowsPerBlock / kRowsPerIter;
    const int c = threadIdx.x % ROW_U4;
    const int rsub = threadIdx.x / ROW_U4;
    const int64_t p0 = (int64_t)blockIdx.x * kRowsPerBlock;
    const int h0 = head_of_row(offsets, heads, p0);            // block-uniform

    const uint4* src_k[kIters];
    const uint4* src_v[kIters];
    bool ok[kIters];
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
        const int64_t p = p0 + it * kRowsPerIter + rsub;
        ok[it] = p < total;
        int64_t idx = 0;
        int h = h0;
        if (ok[it]) {
            while (offsets[h + 1] <= p) ++h;                    // skips empty heads too
            idx = indices[p];
            ok[it] = idx >= 0 && idx < n;                       // never read outside the cache
        }
        const size_t row = ((size_t)h * n + (ok[it] ? idx : 0)) * ROW_U4 + c;
        src_k[it] = K + row;
        src_v[it] = V + row;
    }
    uint4 vk[kIters], vv[kIters];
#pragma unroll
    for (int it = 0; it < kIters; ++it)
        if (ok[it]) { vk[it] = *src_k[it]; vv[it] = *src_v[it]; }
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
        const int64_t p = p0 + it * kRowsPerIter + rsub;
        if (ok[it]) {
            K_out[(size_t)p * ROW_U4 + c] = vk[it];
            V_out[(size_t)p * ROW_U4 + c] = vv[it];
        }
    }
}

hipError_t launch_compact(const curdkv_ctx* ctx, const void* K, const void* V, int64_t n,
                          const int32_t* indices, const int64_t* d_offsets, int64_t total,
                          void* K_out, void* V_out, hipStream_t stream) {
    if (total == 0) return hipSuccess;
    const int64_t blocks = (total + kRowsPerBlock - 1) / kRowsPerBlock;
    if (ctx->cfg.dtype == CURDKV_DTYPE_BF16) {
        compact_kernel<16><<<dim3((unsigned)blocks), 256, 0, stream>>>(
            (const uint4*)K, (const uint4*)V, n, indices, d_offsets, ctx->heads, total,
            (uint4*)K_out, (uint4*)V_out);
    } else {
        compact_kernel<32><<<dim3((unsigned)blocks), 256, 0, stream>>>(
            (const uint4*)K, (const uint4*)V, n, indices, d_offsets, ctx->heads, total,
            (uint4*)K_out, (uint4*)V_out);
    }
    return hipGetLastError();
}

}  // namespace curdkv
